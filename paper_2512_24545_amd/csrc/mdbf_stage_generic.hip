// Matrix-core evaluation of one envelope-scaled binary product on gfx950: the GENERAL variant
// (any dtype of envelopes and activations, any l <= 16, any K).  Same arithmetic as the fast
// variant in mdbf_stage_mfma.hip; element-wise staging loads, column sums on the vector ALU.
//
//   out[r] = sum_c Eout[r,c] * P[r,c],     P[r,c] = sum_j S[r,j] * xs[j,c],   xs[j,c] = fp16(Ein[j,c] * vin[j])
//
// (paper Eq. "me-dbf-expand": per factor, l envelope-scaled copies of the shared sign basis).
// P is a skinny GEMM (rows x K) . (K x 16): exactly one 16x16x32 fp16 MFMA tile wide.
//
// Work decomposition: a workgroup of four wavefronts owns up to 4*R row tiles (16 rows each) of
// one problem and the whole contraction; wave w owns tiles w, w+4, ...  The scaled activations xs
// are staged chunk by chunk (1024 columns) in LDS in the order the MFMA B operand wants them and
// shared by all tiles of the workgroup; sign words stream from HBM with 128-bit loads.
//
// Sign expansion without shifts: with bit t=1 meaning -1,  S = 1 - 2t, hence
//      P[r,c] = colsum[c] - 2 * sum_j t[r,j] xs[j,c].
// The A operand of an MFMA step is  w & mask : the two selected bits of a word, read as two fp16
// values, are 0 or 2^(p-24) (p = bit position 0..7; fp16 denormals are honoured by the MFMA).  The
// staged activation of the entry at position p = 4c+i carries the factor 2^-i, so every product of
// class c (positions 4c..4c+3) is scaled by 2^(4c-24) exactly, and each class has its own fp32
// accumulator.  Bits 8..15 of each half word are brought down with one shift per word.
#include "mdbf_internal.h"

namespace mdbf {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int CB = 8;                      // 128-column blocks per LDS chunk
constexpr int kChunkVecs = CB * 4 * 64;    // 16-byte vectors per chunk buffer (32 KB)
constexpr int kSmemBytes = 2 * kChunkVecs * 16 + 4 * 16 * 4;

__device__ inline half8 expand(uint32_t src, int c) {
  // class c: bit positions 4c..4c+3 and 16 above
  const uint32_t m0 = 0x00010001u << (4 * c);
  u32x4 a;
  a.x = src & m0;
  a.y = src & (m0 << 1);
  a.z = src & (m0 << 2);
  a.w = src & (m0 << 3);
  return __builtin_bit_cast(half8, a);
}

template <int R>
__global__ __launch_bounds__(256) void stage_generic_kernel(const StageProb* __restrict__ probs,
                                                         const WorkItem* __restrict__ items,
                                                         StageProb single, int tiles_per_item) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  u32x4* buf = reinterpret_cast<u32x4*>(smem);
  float* red = reinterpret_cast<float*>(smem + 2 * kChunkVecs * 16);

  const StageProb* pp;
  int tile0, ntl;
  if (probs) {
    const WorkItem& it = items[blockIdx.x];
    pp = &probs[it.prob];
    tile0 = it.tile0;
    ntl = it.ntiles;
  } else {
    pp = &single;
    tile0 = blockIdx.x * tiles_per_item;
    ntl = min(tiles_per_item, single.ntiles - tile0);
  }
  const StageProb p = *pp;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // tiles of this wave: tile0 + wave + 4*jj for jj < nt
  int nt = (ntl - wave + 3) / 4;
  nt = nt < 0 ? 0 : (nt > R ? R : nt);
  const int KB = p.KB;
  const int ngroups = (KB + 3) >> 2;
  const int nchunks = (KB + CB - 1) / CB;

  // an item lies inside one group of tiles: one block stride for all its tiles
  const size_t bstride = (size_t)group_tiles(tile0, p.ntiles) * 64u;
  const MDBF_GLOBAL uint32_t* sbase[R];
#pragma unroll
  for (int r = 0; r < R; ++r) sbase[r] = (const MDBF_GLOBAL uint32_t*)p.S + tile_base_words(min(tile0 + wave + 4 * r, p.ntiles - 1), KB);

  auto load_group = [&](int g, u32x4 (&w)[R]) {
#pragma unroll
    for (int r = 0; r < R; ++r) {
      u32x4 t = {0u, 0u, 0u, 0u};
      if (r < nt) {
        const MDBF_GLOBAL uint32_t* tb = sbase[r] + (size_t)(4 * g) * bstride + lane;
        t.x = tb[0];
        if (4 * g + 1 < KB) t.y = tb[bstride];
        if (4 * g + 2 < KB) t.z = tb[2 * bstride];
        if (4 * g + 3 < KB) t.w = tb[3 * bstride];
      }
      w[r] = t;
    }
  };

  for (int b = 0; b < p.T; ++b) {
    floatx4 acc[R][2];
#pragma unroll
    for (int r = 0; r < R; ++r) {
      acc[r][0] = floatx4{0.f, 0.f, 0.f, 0.f};
      acc[r][1] = floatx4{0.f, 0.f, 0.f, 0.f};
    }
    float cs[8];
#pragma unroll
    for (int cc = 0; cc < 8; ++cc) cs[cc] = 0.f;

    u32x4 wnext[R];
#pragma unroll
    for (int r = 0; r < R; ++r) wnext[r] = u32x4{0u, 0u, 0u, 0u};
    load_group(0, wnext);

    for (int c = 0; c < nchunks; ++c) {
      u32x4* bufc = buf + (c & 1) * kChunkVecs;
      // ---- stage xs for columns [c*1024, c*1024+1024) into LDS, B-operand order --------------
      for (int oo = tid >> 1; oo < CB * 16; oo += 128) {
        const int ch = tid & 1;
        const int qloc = oo >> 4, f = (oo & 15) >> 2, kg = oo & 3;
        const int kbase = (c * CB + qloc) * kBlockCols + f * 32 + kg * 8;
        _Float16 h[8][8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const int k = kbase + e;
          const float beta = (e >> 1) == 0 ? 1.f : (e >> 1) == 1 ? 0.5f : (e >> 1) == 2 ? 0.25f : 0.125f;
          const float rbeta = (float)(1 << (e >> 1));
          float vk = 0.f;
          if (k < p.K) vk = load_as_float(p.vin, (int64_t)b * p.vin_ld + k, p.vin_dt);
#pragma unroll
          for (int cc = 0; cc < 8; ++cc) {
            const int s = ch * 8 + cc;
            float ev = 0.f;
            if (k < p.K && s < p.l) ev = load_as_float(p.Ein, (int64_t)k * p.l + s, p.env_dt);
            const _Float16 hv = (_Float16)((ev * vk) * beta);
            h[e][cc] = hv;
            cs[cc] += (float)hv * rbeta;
          }
        }
#pragma unroll
        for (int cc = 0; cc < 8; ++cc) {
          half8 v;
#pragma unroll
          for (int e = 0; e < 8; ++e) v[e] = h[e][cc];
          bufc[(qloc * 4 + f) * 64 + kg * 16 + ch * 8 + cc] = __builtin_bit_cast(u32x4, v);
        }
      }
      __syncthreads();
      // ---- contract this chunk ---------------------------------------------------------------
#pragma unroll
      for (int gi = 0; gi < CB / 4; ++gi) {
        const int g = c * (CB / 4) + gi;
        if (g < ngroups) {
          u32x4 w[R];
#pragma unroll
          for (int r = 0; r < R; ++r) w[r] = wnext[r];
          if (g + 1 < ngroups) load_group(g + 1, wnext);
          const int nb = min(4, KB - 4 * g);
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            if (j < nb) {
#pragma unroll
              for (int f = 0; f < 4; ++f) {
                const half8 bop = __builtin_bit_cast(half8, bufc[((gi * 4 + j) * 4 + f) * 64 + lane]);
#pragma unroll
                for (int r = 0; r < R; ++r) {
                  if (r < nt) {
                    const uint32_t word = w[r][j];
                    const uint32_t src = (f < 2) ? word : (word >> 8);
                    acc[r][f & 1] =
                        __builtin_amdgcn_mfma_f32_16x16x32_f16(expand(src, f & 1), bop, acc[r][f & 1], 0, 0, 0);
                  }
                }
              }
            }
          }
        }
      }
    }

    // ---- column sums of xs: reduce over the threads that staged the same column half ----------
#pragma unroll
    for (int cc = 0; cc < 8; ++cc) {
      float v = cs[cc];
      v += __shfl_xor(v, 2);
      v += __shfl_xor(v, 4);
      v += __shfl_xor(v, 8);
      v += __shfl_xor(v, 16);
      v += __shfl_xor(v, 32);
      cs[cc] = v;
    }
    if (lane < 2) {
#pragma unroll
      for (int cc = 0; cc < 8; ++cc) red[wave * 16 + lane * 8 + cc] = cs[cc];
    }
    __syncthreads();
    const int s = lane & 15;
    const float colsum = (red[s] + red[16 + s]) + (red[32 + s] + red[48 + s]);

    // ---- fix-up, envelope accumulate, store ----------------------------------------------------
#pragma unroll
    for (int r = 0; r < R; ++r) {
      if (r < nt) {
        const int rowb = (tile0 + wave + 4 * r) * kTileRows + 4 * (lane >> 4);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int row = rowb + i;
          const float P = colsum - acc[r][0][i] * 33554432.f - acc[r][1][i] * 2097152.f;  // 2^25, 2^21
          float ev = 0.f;
          if (row < p.rows && s < p.l) ev = load_as_float(p.Eout, (int64_t)row * p.l + s, p.env_dt);
          float v = ev * P;
          v += __shfl_xor(v, 1);
          v += __shfl_xor(v, 2);
          v += __shfl_xor(v, 4);
          v += __shfl_xor(v, 8);
          if (s == 0 && row < p.rows) emit_result(p.out, (int64_t)b * p.out_ld + row, p.out_dt, v, p.flags);
        }
      }
    }
    __syncthreads();  // red and the chunk buffers are reused by the next token
  }
}

template <int R>
static int launch_generic_r(const StageProb* probs_dev, const WorkItem* items_dev, int nblocks, int tiles_per_item,
                    const StageProb* single, hipStream_t s) {
  static KernelSetup setup;
  if (int e = kernel_setup(setup, [] {
        return hipFuncSetAttribute(reinterpret_cast<const void*>(&stage_generic_kernel<R>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, kSmemBytes);
      }))
    return e;
  hipLaunchKernelGGL(stage_generic_kernel<R>, dim3((unsigned)nblocks), dim3(256), kSmemBytes, s, probs_dev, items_dev,
                     *single, tiles_per_item);
  return (int)hipGetLastError();
}

int launch_stage_generic(const StageProb* probs_dev, const WorkItem* items_dev, int nitems, int tiles_per_item,
                      const StageProb* single, hipStream_t s) {
  int nblocks = nitems;
  if (!probs_dev) nblocks = (single->ntiles + tiles_per_item - 1) / tiles_per_item;
  switch (tiles_per_item) {
    case 4: return launch_generic_r<1>(probs_dev, items_dev, nblocks, tiles_per_item, single, s);
    case 8: return launch_generic_r<2>(probs_dev, items_dev, nblocks, tiles_per_item, single, s);
    case 16: return launch_generic_r<4>(probs_dev, items_dev, nblocks, tiles_per_item, single, s);
    default: return (int)hipErrorInvalidValue;
  }
}

}  // namespace mdbf
