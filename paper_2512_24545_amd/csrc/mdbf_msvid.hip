// MSVID_l on the GPU: the projection step of the layer-wise quantizer (paper Sec. 4.2, Eq. "msvid-def"):
//
//   MSVID_l[Z] = sign(Z) o TSVD_l(|Z|),      TSVD_l(|Z|) = A Q^T  (rank l, best in Frobenius norm)
//
// with the singular values split evenly between the factors, A = U_l sqrt(Sigma_l), Q = V_l sqrt(Sigma_l).
// By Theorem 1 (Eq. "rankl-error") the error of the result is the tail of |Z|'s spectrum.
//
// The truncated SVD is taken by block subspace iteration with b = l + oversampling columns and a
// Rayleigh-Ritz step at the end; everything runs on the stream, nothing is read back by the host:
//   V <- caller's start block (cols x b)
//   repeat `iters` times:   B = |Z| V,  orthonormalise;   V = |Z|^T B,  orthonormalise
//   B = |Z| V;   B^T B = W L W^T (Jacobi, fp64);   sigma = sqrt(L);   A = B W_l Sigma_l^(-1/2),   Q = V W_l Sigma_l^(1/2)
// The two products are the whole cost: each reads Z once (HBM-bound, 4 bytes per 2 b multiply-adds).  Both are
// run by one kernel, "lanes own columns" (coalesced reads, no cross-lane sums): |Z|^T B on Z itself, |Z| V
// on a transposed copy of Z made once at the start (the sign matrix is written in the same pass).
// Orthonormalisation is Cholesky-QR: Gram matrix from per-workgroup partial sums (fp32) added in fp64, Cholesky
// factor R in fp64, and the next product applies R^(-1) to the rows of its input block as it stages them.
#include "mdbf_internal.h"

namespace mdbf {
namespace msvid {

constexpr int kThreads = 256;
constexpr int kStrip = 128;           // columns per workgroup of the product kernel: two per lane, 4 waves share the rows
constexpr int kChunkRows = 128;       // rows per workgroup of the product kernel
constexpr int kBatchRows = 16;        // rows whose loads a wave issues before their arithmetic
constexpr int kSmallThreads = 1024;   // the b x b kernels (a thread per matrix entry, b <= 32) and the chunk reduction
                                      // (few workgroups: many loads in flight in each)
constexpr int kGramRows = 64;         // rows per workgroup of the reduce + Gram kernel

// ---- S = sign(Z) as int8 (+1 / -1, sign(0) = +1: Sec. 2, Notation) and Zt = Z^T, 64 x 64 tiles through LDS
__global__ __launch_bounds__(kThreads) void sign_transpose_kernel(const float* __restrict__ Z, int rows, int cols,
                                                                  int64_t ld, int8_t* __restrict__ S,
                                                                  float* __restrict__ Zt) {
  __shared__ float tile[64][65];
  const int c0 = blockIdx.x * 64, r0 = blockIdx.y * 64;
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  for (int i = ty; i < 64; i += 4) {
    const int r = r0 + i, c = c0 + tx;
    float z = 0.f;
    if (r < rows && c < cols) {
      z = Z[(int64_t)r * ld + c];
      S[(int64_t)r * cols + c] = (z < 0.f) ? (int8_t)-1 : (int8_t)1;
    }
    tile[i][tx] = z;
  }
  __syncthreads();
  for (int i = ty; i < 64; i += 4) {
    const int c = c0 + i, r = r0 + tx;
    if (r < rows && c < cols) Zt[(int64_t)c * rows + r] = tile[tx][i];
  }
}

// ---- P[chunk][c][:] = sum over the chunk's rows r of |M[r, c]| * X'[r, :],   X' = X Tm  (Tm null: X' = X)
// M: R_ x C_ row-major; X: R_ x BB; Tm: BB x BB (fp64, row-major).  Grid: (column strips, row chunks).
// A lane owns columns c and c + 64 of the strip; the four waves take every fourth group of kBatchRows rows, with
// the loads of a group issued before its arithmetic (a load is a trip to HBM: what bounds the kernel is how many
// are in flight), and add their sums through LDS in a fixed order.
template <int BB>
__global__ __launch_bounds__(kThreads) void abs_t_mul_kernel(const float* __restrict__ M, int R_, int C_, int64_t ldm,
                                                             const float* __restrict__ X,
                                                             const double* __restrict__ Tm, float* __restrict__ P) {
  __shared__ __attribute__((aligned(16))) float xs[kChunkRows][BB];
  __shared__ float red[2 * kStrip * BB];
  __shared__ float tms[BB * BB];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r0 = blockIdx.y * kChunkRows;
  const int nr = min(kChunkRows, R_ - r0);
  if (Tm) {
    for (int p = tid; p < BB * BB; p += kThreads) tms[p] = (float)Tm[p];
    __syncthreads();
  }
  for (int idx = tid; idx < kChunkRows * BB; idx += kThreads) {
    const int r = idx / BB, j = idx - r * BB;
    float v = 0.f;                                   // rows past the chunk's end contribute nothing
    if (r < nr) {
      const float* xr = X + (size_t)(r0 + r) * BB;
      if (Tm) {
        float sum = 0.f;                               // (the span is what matters here; the last block is
#pragma unroll                                         //  orthonormalised in fp64 by apply_kernel)
        for (int i = 0; i < BB; ++i) sum = fmaf(xr[i], tms[i * BB + j], sum);
        v = sum;
      } else {
        v = xr[j];
      }
    }
    xs[r][j] = v;
  }
  __syncthreads();
  const int c_a = blockIdx.x * kStrip + lane, c_b = c_a + 64;
  const float* pa = M + (size_t)r0 * ldm + min(c_a, C_ - 1);
  const float* pb = M + (size_t)r0 * ldm + min(c_b, C_ - 1);
  float acc_a[BB], acc_b[BB];
#pragma unroll
  for (int j = 0; j < BB; ++j) { acc_a[j] = 0.f; acc_b[j] = 0.f; }
#pragma unroll 1
  for (int g = wave * kBatchRows; g < nr; g += 4 * kBatchRows) {
    float ma[kBatchRows], mb[kBatchRows];
#pragma unroll
    for (int u = 0; u < kBatchRows; ++u) {
      const size_t ro = (size_t)min(g + u, nr - 1) * ldm;     // (the repeated row meets a zero row of xs)
      ma[u] = fabsf(pa[ro]);
      mb[u] = fabsf(pb[ro]);
    }
#pragma unroll
    for (int u = 0; u < kBatchRows; ++u) {
#pragma unroll
      for (int j = 0; j < BB; ++j) {
        const float x = xs[g + u][j];
        acc_a[j] = fmaf(ma[u], x, acc_a[j]);
        acc_b[j] = fmaf(mb[u], x, acc_b[j]);
      }
    }
  }
  // the waves' sums through LDS in a fixed order: (wave 0 + wave 2) + (wave 1 + wave 3)
  static_assert(kChunkRows % kBatchRows == 0 && kStrip == 128, "row groups tile a chunk; two columns per lane");
  if (wave >= 2) {
#pragma unroll
    for (int j = 0; j < BB; ++j) {
      red[((wave - 2) * 128 + lane) * BB + j] = acc_a[j];
      red[((wave - 2) * 128 + 64 + lane) * BB + j] = acc_b[j];
    }
  }
  __syncthreads();
  if (wave < 2) {
#pragma unroll
    for (int j = 0; j < BB; ++j) {
      acc_a[j] += red[(wave * 128 + lane) * BB + j];
      acc_b[j] += red[(wave * 128 + 64 + lane) * BB + j];
    }
  }
  __syncthreads();
  if (wave == 1) {
#pragma unroll
    for (int j = 0; j < BB; ++j) {
      red[lane * BB + j] = acc_a[j];
      red[(64 + lane) * BB + j] = acc_b[j];
    }
  }
  __syncthreads();
  if (wave == 0) {
    if (c_a < C_) {
      float* out = P + ((size_t)blockIdx.y * C_ + c_a) * BB;
#pragma unroll
      for (int j = 0; j < BB; ++j) out[j] = acc_a[j] + red[lane * BB + j];
    }
    if (c_b < C_) {
      float* out = P + ((size_t)blockIdx.y * C_ + c_b) * BB;
#pragma unroll
      for (int j = 0; j < BB; ++j) out[j] = acc_b[j] + red[(64 + lane) * BB + j];
    }
  }
}

// ---- Y = sum over chunks of P (in chunk order), and this workgroup's part of Y^T Y
template <int BB>
__global__ __launch_bounds__(kSmallThreads) void reduce_gram_kernel(const float* __restrict__ P, int nchunks, int n,
                                                               float* __restrict__ Y, float* __restrict__ Gp) {
  __shared__ float ys[kGramRows * BB];
  const int tid = threadIdx.x;
  const int row0 = blockIdx.x * kGramRows;
  const int nrow = min(kGramRows, n - row0);
  const size_t plane = (size_t)n * BB;
  for (int idx = tid; idx < kGramRows * BB; idx += blockDim.x) {
    float y = 0.f;
    if (idx < nrow * BB) {
      const size_t e = (size_t)row0 * BB + idx;
      for (int c0 = 0; c0 < nchunks; c0 += 8) {        // eight loads in flight, added in chunk order
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = P[(size_t)min(c0 + u, nchunks - 1) * plane + e];
#pragma unroll
        for (int u = 0; u < 8; ++u)
          if (c0 + u < nchunks) y += v[u];
      }
      Y[e] = y;
    }
    ys[idx] = y;
  }
  __syncthreads();
  for (int p = tid; p < BB * BB; p += blockDim.x) {
    const int i = p / BB, j = p - i * BB;
    float g = 0.f;
    for (int r = 0; r < kGramRows; ++r) g = fmaf(ys[r * BB + i], ys[r * BB + j], g);
    Gp[(size_t)blockIdx.x * BB * BB + p] = g;
  }
}

// G = sum of the workgroups' parts, in fp64, in part order (thread p owns entries p, p + blockDim.x, ...)
template <int BB>
__device__ void gather_gram(const float* __restrict__ Gp, int nparts, double (&G)[BB][BB]) {
  for (int p = threadIdx.x; p < BB * BB; p += blockDim.x) {
    double sum = 0.0;
    for (int w0 = 0; w0 < nparts; w0 += 16) {       // sixteen loads in flight, added in part order
      float v[16];
#pragma unroll
      for (int u = 0; u < 16; ++u) v[u] = Gp[(size_t)min(w0 + u, nparts - 1) * BB * BB + p];
#pragma unroll
      for (int u = 0; u < 16; ++u)
        if (w0 + u < nparts) sum += (double)v[u];
    }
    G[p / BB][p % BB] = sum;
  }
  __syncthreads();
}

// a double held by lane `src` (a compile-time or wave-uniform index), in every lane
__device__ __forceinline__ double lane_value(double v, int src) {
  const uint64_t u = __builtin_bit_cast(uint64_t, v);
  const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)u, src);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(u >> 32), src);
  return __builtin_bit_cast(double, ((uint64_t)hi << 32) | lo);
}

// ---- Cholesky-QR: G = R^T R (R upper triangular), Tm = R^(-1): Y Tm has orthonormal columns.
// The whole workgroup adds up the Gram parts; the factorisation itself runs in one wave, lane j holding column j
// of the matrix in registers (right-looking: after step k the trailing columns hold the Schur complement), with
// row k passed round by lane reads: no LDS traffic and no barrier inside the b steps.
// A column that the earlier ones span (|Z| of lower rank than the block is wide: a member of the format is) has
// a pivot at the level of the Gram matrix's rounding, 1e-6 of its diagonal entry (fp32 partial sums): such a
// column is dropped (its column of Tm is zero, and stays zero through the products that follow).
template <int BB>
__global__ __launch_bounds__(kSmallThreads) void chol_kernel(const float* __restrict__ Gp, int nparts, double* __restrict__ Tm) {
  __shared__ double G[BB][BB];
  gather_gram<BB>(Gp, nparts, G);
  if (threadIdx.x >= 64) return;                       // (no barrier below)
  const int j = (int)threadIdx.x;
  const int jc = min(j, BB - 1);                       // lanes past the last column shadow it and store nothing
  double a[BB], rk[BB], rinv[BB];
  uint32_t dead = 0;
#pragma unroll
  for (int i = 0; i < BB; ++i) a[i] = G[i][jc];
#pragma unroll
  for (int k = 0; k < BB; ++k) {
    const double piv = lane_value(a[k], k);            // the Schur complement's diagonal entry
    const double g0 = G[k][k];
    const bool drop = !(piv > 1e-6 * g0) || !(g0 > 0.0);
    const double rd = drop ? 1.0 : 1.0 / sqrt(piv);
    rinv[k] = rd;
    dead |= drop ? (1u << k) : 0u;
    rk[k] = (jc < k) ? 0.0 : (jc == k) ? (drop ? 1.0 : piv * rd) : (drop ? 0.0 : a[k] * rd);   // R[k][jc]
#pragma unroll
    for (int i = k + 1; i < BB; ++i) a[i] -= lane_value(rk[k], i) * rk[k];
  }
  // column jc of R^(-1) by back substitution on R X = I (entries below the diagonal come out zero)
  double x[BB];
#pragma unroll
  for (int i = BB - 1; i >= 0; --i) {
    double sum = (i == jc) ? 1.0 : 0.0;
#pragma unroll
    for (int m = i + 1; m < BB; ++m) sum -= lane_value(rk[i], m) * x[m];
    x[i] = sum * rinv[i];
  }
  if (j < BB) {
    const bool gone = (dead >> j) & 1u;
#pragma unroll
    for (int i = 0; i < BB; ++i) Tm[i * BB + j] = gone ? 0.0 : x[i];
  }
}

// ---- Rayleigh-Ritz: G = B^T B = W L W^T by cyclic Jacobi in fp64; Ritz values sigma_i = sqrt(L_i), descending.
// MA = W_l Sigma_l^(-1/2) (A = B MA), MQ = W_l Sigma_l^(1/2) (Q = V MQ); both BB x BB row-major, columns >= l zero.
template <int BB>
__global__ __launch_bounds__(kSmallThreads) void ritz_kernel(const float* __restrict__ Gp, int nparts, int l,
                                                  double* __restrict__ MA, double* __restrict__ MQ,
                                                  float* __restrict__ sigma) {
  __shared__ double a[BB][BB];
  __shared__ double w[BB][BB];
  __shared__ double cc[BB / 2], ss[BB / 2];
  __shared__ int pp[BB / 2], qq[BB / 2];
  __shared__ int order[BB];
  __shared__ int rotated;
  const int t = threadIdx.x;
  gather_gram<BB>(Gp, nparts, a);
  for (int p = t; p < BB * BB; p += blockDim.x) w[p / BB][p % BB] = (p / BB == p % BB) ? 1.0 : 0.0;
  __syncthreads();
  // Cyclic Jacobi with the round-robin ordering: a step rotates BB / 2 disjoint index pairs at once (player
  // BB - 1 stays, the others move round a circle), BB - 1 steps visit every pair once.  The rotations of a step
  // are all computed from the matrix as it stands before the step; disjoint pairs touch disjoint rows and columns.
  static_assert(BB % 2 == 0, "pairs");
  constexpr int H = BB / 2;
  for (int sweep = 0; sweep < 12; ++sweep) {
    if (t == 0) rotated = 0;
    __syncthreads();
    for (int step = 0; step < BB - 1; ++step) {
      if (t < H) {
        int p, q;
        if (t == 0) {
          p = BB - 1;
          q = step;
        } else {
          p = (step + t) % (BB - 1);
          q = (step - t + (BB - 1)) % (BB - 1);
        }
        if (p > q) { const int tmp = p; p = q; q = tmp; }
        const double apq = a[p][q], app = a[p][p], aqq = a[q][q];
        double c = 1.0, sn = 0.0;
        if (fabs(apq) > 1e-300 && fabs(apq) > 1e-16 * sqrt(fabs(app * aqq))) {
          const double tau = (aqq - app) / (2.0 * apq);
          const double tt = (tau >= 0.0 ? 1.0 : -1.0) / (fabs(tau) + sqrt(1.0 + tau * tau));
          c = 1.0 / sqrt(1.0 + tt * tt);
          sn = tt * c;
          rotated = 1;                                 // (any writer writes 1)
        }
        pp[t] = p;
        qq[t] = q;
        cc[t] = c;
        ss[t] = sn;
      }
      __syncthreads();
      for (int idx = t; idx < BB * H; idx += blockDim.x) {     // columns p, q of a and of w
        const int k = idx / H, pr = idx - k * H;
        const int p = pp[pr], q = qq[pr];
        const double c = cc[pr], sn = ss[pr];
        const double akp = a[k][p], akq = a[k][q];
        a[k][p] = c * akp - sn * akq;
        a[k][q] = sn * akp + c * akq;
        const double wkp = w[k][p], wkq = w[k][q];
        w[k][p] = c * wkp - sn * wkq;
        w[k][q] = sn * wkp + c * wkq;
      }
      __syncthreads();
      for (int idx = t; idx < BB * H; idx += blockDim.x) {     // rows p, q of a
        const int k = idx / H, pr = idx - k * H;
        const int p = pp[pr], q = qq[pr];
        const double c = cc[pr], sn = ss[pr];
        const double apk = a[p][k], aqk = a[q][k];
        a[p][k] = c * apk - sn * aqk;
        a[q][k] = sn * apk + c * aqk;
      }
      __syncthreads();
    }
    if (!rotated) break;                               // a whole sweep without a rotation: diagonal to working precision
  }
  if (t == 0) {            // eigenvalues in descending order (insertion sort of at most 32 indices)
    for (int i = 0; i < BB; ++i) order[i] = i;
    for (int i = 1; i < BB; ++i) {
      const int oi = order[i];
      int j = i - 1;
      while (j >= 0 && a[order[j]][order[j]] < a[oi][oi]) { order[j + 1] = order[j]; --j; }
      order[j + 1] = oi;
    }
  }
  __syncthreads();
  if (t < BB) sigma[t] = (float)sqrt(fmax(a[order[t]][order[t]], 0.0));
  for (int p = t; p < BB * BB; p += blockDim.x) {
    const int i = p / BB, j = p - i * BB;
    double ma = 0.0, mq = 0.0;
    if (j < l) {
      const double sg = sqrt(fmax(a[order[j]][order[j]], 0.0));
      const double sg_max = sqrt(fmax(a[order[0]][order[0]], 0.0));
      if (sg > 1e-7 * sg_max) {    // a mode at the level of fp32 rounding of the largest is a null mode of |Z|
        const double rs = sqrt(sg);
        mq = w[i][order[j]] * rs;
        ma = w[i][order[j]] / rs;
      }
    }
    MA[p] = ma;
    MQ[p] = mq;
  }
}

// ---- Out (n x lo) = Y (n x BB) . Mm (BB x BB, its first lo columns), fp64 accumulation
template <int BB>
__global__ __launch_bounds__(kThreads) void apply_kernel(const float* __restrict__ Y, int n, const double* __restrict__ Mm,
                                                         int lo, float* __restrict__ Out) {
  __shared__ double ms[BB * BB];
  for (int p = threadIdx.x; p < BB * BB; p += kThreads) ms[p] = Mm[p];
  __syncthreads();
  const size_t total = (size_t)n * lo;
  for (size_t e = (size_t)blockIdx.x * kThreads + threadIdx.x; e < total; e += (size_t)gridDim.x * kThreads) {
    const size_t r = e / lo;
    const int j = (int)(e - r * lo);
    const float* yr = Y + r * BB;
    double s = 0.0;
#pragma unroll
    for (int i = 0; i < BB; ++i) s += (double)yr[i] * ms[i * BB + j];
    Out[e] = (float)s;
  }
}

struct Layout {
  size_t zt, p, yb, yc, v1, gp, tm, ma, mq, total;
  int nparts_max;
};

template <int BB>
static int run(const float* Z, int rows, int cols, int64_t ld, int l, int iters, const float* X0, int8_t* S, float* A,
               float* Q, float* sigma, unsigned char* ws, const Layout& L, hipStream_t s) {
  float* Zt = (float*)(ws + L.zt);
  float* P = (float*)(ws + L.p);
  float* Yb = (float*)(ws + L.yb);     // rows x BB
  float* Yc = (float*)(ws + L.yc);     // cols x BB
  float* V1 = (float*)(ws + L.v1);     // cols x BB
  float* Gp = (float*)(ws + L.gp);
  double* Tm = (double*)(ws + L.tm);
  double* MA = (double*)(ws + L.ma);
  double* MQ = (double*)(ws + L.mq);
  const dim3 blk(kThreads);
  hipLaunchKernelGGL(sign_transpose_kernel, dim3((cols + 63) / 64, (rows + 63) / 64), blk, 0, s, Z, rows, cols, ld, S, Zt);
  // Y (n_out x BB) = |Mx|^T-style product over the matrix Mx (R_ x C_), then Y's Gram parts
  auto product = [&](const float* Mx, int R_, int C_, int64_t ldm, const float* X, const double* Tx, float* Y) {
    const int nchunks = (R_ + kChunkRows - 1) / kChunkRows;
    hipLaunchKernelGGL(abs_t_mul_kernel<BB>, dim3((C_ + kStrip - 1) / kStrip, nchunks), blk, 0, s, Mx, R_, C_, ldm, X, Tx, P);
    const int nparts = (C_ + kGramRows - 1) / kGramRows;
    hipLaunchKernelGGL(reduce_gram_kernel<BB>, dim3(nparts), dim3(kSmallThreads), 0, s, P, nchunks, C_, Y, Gp);
    return nparts;
  };
  const float* X = X0;
  const double* Tx = nullptr;
  for (int it = 0; it < iters; ++it) {
    int np = product(Zt, cols, rows, rows, X, Tx, Yb);                 // B = |Z| V
    hipLaunchKernelGGL(chol_kernel<BB>, dim3(1), dim3(kSmallThreads), 0, s, Gp, np, Tm);
    np = product(Z, rows, cols, ld, Yb, Tm, Yc);                       // V = |Z|^T B
    hipLaunchKernelGGL(chol_kernel<BB>, dim3(1), dim3(kSmallThreads), 0, s, Gp, np, Tm);
    X = Yc;
    Tx = Tm;
  }
  // an orthonormal V: Cholesky-QR twice (iters == 0: on the start block itself)
  const int grid_apply = 1024;
  const int npc = (cols + kGramRows - 1) / kGramRows;
  if (iters == 0) {
    hipLaunchKernelGGL(reduce_gram_kernel<BB>, dim3(npc), dim3(kSmallThreads), 0, s, X0, 1, cols, Yc, Gp);
    hipLaunchKernelGGL(chol_kernel<BB>, dim3(1), dim3(kSmallThreads), 0, s, Gp, npc, Tm);
  }
  hipLaunchKernelGGL(apply_kernel<BB>, dim3(grid_apply), blk, 0, s, Yc, cols, Tm, BB, V1);
  hipLaunchKernelGGL(reduce_gram_kernel<BB>, dim3(npc), dim3(kSmallThreads), 0, s, V1, 1, cols, Yc, Gp);   // (Yc = copy of V1)
  hipLaunchKernelGGL(chol_kernel<BB>, dim3(1), dim3(kSmallThreads), 0, s, Gp, npc, Tm);
  hipLaunchKernelGGL(apply_kernel<BB>, dim3(grid_apply), blk, 0, s, Yc, cols, Tm, BB, V1);        // V1 = V, orthonormal
  // Rayleigh-Ritz on B = |Z| V
  const int npb = product(Zt, cols, rows, rows, V1, nullptr, Yb);
  hipLaunchKernelGGL(ritz_kernel<BB>, dim3(1), dim3(kSmallThreads), 0, s, Gp, npb, l, MA, MQ, sigma);
  hipLaunchKernelGGL(apply_kernel<BB>, dim3(grid_apply), blk, 0, s, Yb, rows, MA, l, A);
  hipLaunchKernelGGL(apply_kernel<BB>, dim3(grid_apply), blk, 0, s, V1, cols, MQ, l, Q);
  return (int)hipGetLastError();
}

}  // namespace msvid

int msvid_block(int l) { return l <= 8 ? 16 : l <= 16 ? 24 : 32; }

static msvid::Layout msvid_layout(int rows, int cols, int b) {
  auto up = [](size_t v) { return (v + 255) / 256 * 256; };
  msvid::Layout L;
  size_t off = 0;
  L.zt = off; off = up(off + (size_t)rows * cols * 4u);
  const size_t chunks_a = (size_t)(cols + msvid::kChunkRows - 1) / msvid::kChunkRows;   // product over Zt: output rows x b
  const size_t chunks_b = (size_t)(rows + msvid::kChunkRows - 1) / msvid::kChunkRows;   // product over Z: output cols x b
  const size_t pa = chunks_a * (size_t)rows * b * 4u, pb = chunks_b * (size_t)cols * b * 4u;
  L.p = off; off = up(off + (pa > pb ? pa : pb));
  L.yb = off; off = up(off + (size_t)rows * b * 4u);
  L.yc = off; off = up(off + (size_t)cols * b * 4u);
  L.v1 = off; off = up(off + (size_t)cols * b * 4u);
  const int big = rows > cols ? rows : cols;
  L.nparts_max = (big + msvid::kGramRows - 1) / msvid::kGramRows;
  L.gp = off; off = up(off + (size_t)L.nparts_max * b * b * 4u);
  L.tm = off; off = up(off + (size_t)b * b * 8u);
  L.ma = off; off = up(off + (size_t)b * b * 8u);
  L.mq = off; off = up(off + (size_t)b * b * 8u);
  L.total = off;
  return L;
}

size_t msvid_ws_bytes(int rows, int cols, int l) { return msvid_layout(rows, cols, msvid_block(l)).total; }

int launch_msvid(const float* Z, int rows, int cols, int64_t ld, int l, int iters, const float* X0, int8_t* S, float* A,
                 float* Q, float* sigma, void* ws, hipStream_t s) {
  const int b = msvid_block(l);
  const msvid::Layout L = msvid_layout(rows, cols, b);
  unsigned char* w = (unsigned char*)ws;
  switch (b) {
    case 16: return msvid::run<16>(Z, rows, cols, ld, l, iters, X0, S, A, Q, sigma, w, L, s);
    case 24: return msvid::run<24>(Z, rows, cols, ld, l, iters, X0, S, A, Q, sigma, w, L, s);
    default: return msvid::run<32>(Z, rows, cols, ld, l, iters, X0, S, A, Q, sigma, w, L, s);
  }
}

}  // namespace mdbf
