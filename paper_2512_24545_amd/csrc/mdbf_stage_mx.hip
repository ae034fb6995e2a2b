// Block-scaled (MX) matrix-core evaluation of one envelope-scaled binary product on gfx950.
//
//   out[r] = sum_c Eout[r,c] * P[r,c],     P[r,c] = sum_j S[r,j] * xs[j,c],   xs[j,c] = Ein[j,c] * vin[j]
//
// (paper Eq. "me-dbf-expand").  Same problem as the fp16 variant in mdbf_stage_mfma.hip, served by
// v_mfma_scale_f32_16x16x128_f8f6f4: one instruction contracts a whole 128-column block of a 16-row tile.
//
//  * A operand (signs) in fp4 (e2m1).  A lane's 32 sign bits of a block are one 32-bit word w; the four
//    operand registers are  w & 0x11111111, w & 0x22222222, w & 0x44444444, (w >> 1) & 0x44444444 :
//    every nibble is 0 or the single-bit pattern of 0.5, 1, 2, 2.  Five vector operations expand 32 signs
//    (the fp16 variant needs 17).  With bit t = 1 meaning -1, S = 1 - 2t, so P = colsum - 2 * sum t*xs.
//  * B operand (activations) in three fp6 (e2m3) limbs with one power-of-two scale per lane and block
//    (32 values): xs' = L1*2^E + L2*2^(E-4) + L3*2^(E-8) to about 2^-13 of the block maximum, where
//    xs' = xs / {0.5,1,2,2} undoes the value of the sign nibble.  Three MFMAs per tile and block, all into
//    one fp32 accumulator; the hardware applies the scales.
//  * The limbs are produced once per (problem, token) by mx_scale_in_kernel, in the order the workgroups
//    copy them to LDS; the main kernel does no arithmetic on activations.
//  * colsum[c] = sum_j xs[j,c] is taken over the quantised values by the scale-in kernel (exact in fp32 per
//    element, one partial sum per chunk and mode) and travels at the end of each chunk record.
//
// The persistent-workgroup skeleton (units, loads of the next unit issued a chunk ahead, no load inside a
// branch) is the one of the fp16 variant; a chunk is 6 blocks (768 columns) so that two workgroups fit a CU.
#include <type_traits>

#include "mdbf_internal.h"

namespace mdbf {
namespace mx {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

#define MDBF_GLOBAL __attribute__((address_space(1)))
typedef const MDBF_GLOBAL u32x4* g_u32x4_ptr;
typedef const MDBF_GLOBAL uint32_t* g_u32_ptr;
typedef const MDBF_GLOBAL uint16_t* g_u16_ptr;
typedef const MDBF_GLOBAL float* g_f32_ptr;

#ifdef MDBF_DBG_TIMING
__device__ unsigned long long g_dbg_time_mx[64 * 64];   // [block < 64][slot]
#define DBG_T(slot) do { if (dbg_unit == 2 && blockIdx.x < 64 && (threadIdx.x & 63) == 0 && (threadIdx.x >> 6) == 1 && (slot) < 64) \
    g_dbg_time_mx[blockIdx.x * 64 + (slot)] = __builtin_readcyclecounter(); } while (0)
#define DBG_UNIT_DECL int dbg_unit = 0
#define DBG_UNIT_NEXT ++dbg_unit
#else
#define DBG_T(slot) do {} while (0)
#define DBG_UNIT_DECL do {} while (0)
#define DBG_UNIT_NEXT do {} while (0)
#endif

constexpr int CBX = 6;                         // blocks per chunk
// per block in the activation stream: 3 limbs x (64 x 16 B + 64 x 8 B) + 64 x 4 B of scales
constexpr int kLimbA = 0;                      // byte offsets inside a block record
constexpr int kLimbBytes = 64 * 24;            // 1536: [64 x 16 B][64 x 8 B]
constexpr int kScaleOff = 3 * kLimbBytes;      // 4608
constexpr int kBlockBytes = kScaleOff + 256;   // 4864
constexpr int kBlockVecs = kBlockBytes / 16;   // 304
constexpr int kColsumOff = CBX * kBlockBytes;  // 16 fp32 column sums of the chunk close its record
constexpr int kChunkVecs = CBX * kBlockVecs + 4;           // 1828 (29248 B)
constexpr int kCopyPerThread = (kChunkVecs + 255) / 256;   // 8
constexpr int kBufVecs = kCopyPerThread * 256;             // LDS buffer of a chunk, padded so that copies need no mask
__host__ __device__ constexpr int eo_vecs(int R) { return R * 4 * 16 * 2 < 256 ? 256 : R * 4 * 16 * 2; }
__host__ __device__ constexpr int smem_bytes(int R) { return 2 * kBufVecs * 16 + eo_vecs(R) * 16; }

// ---------------------------------------------------------------------------------------------------
// fp6 e2m3: 1 sign, 2 exponent (bias 1), 3 mantissa bits: 0, 0.125 .. 0.875, 1 .. 1.875, 2 .. 3.75, 4 .. 7.5.
// v_cvt_scalef32_2xpk16_fp6_f32 converts 32 floats at once: divides by the power of two in the exponent
// field of `scale`, rounds to nearest even, saturates at +-7.5; element 2i of the result comes from the
// first source's element i, element 2i+1 from the second's; element j sits at bits [6j, 6j+6) -- the order
// the matrix-core instruction reads.  v_cvt_scalef32_pk32_f32_fp6 is the inverse (times the scale).
// ---------------------------------------------------------------------------------------------------
typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v32f __attribute__((ext_vector_type(32)));
typedef unsigned v6u __attribute__((ext_vector_type(6)));

__device__ __forceinline__ v6u fp6_encode32(const float (&v)[32], float scale) {
  v16f even, odd;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    even[i] = v[2 * i];
    odd[i] = v[2 * i + 1];
  }
  return __builtin_amdgcn_cvt_scalef32_2xpk16_fp6_f32(even, odd, scale);
}

// local column (0..127) of element j (0..31) of lane group kg: element j = 8v + i is nibble i of operand
// register v, i.e. bit 4i + v of the lane's sign word; the bit-to-column map is the packed layout's
__host__ __device__ constexpr int local_col_of_element(int j, int kg) {
  const int b = 4 * (j & 7) + (j >> 3);
  const int h = b >> 4, bb = b & 15;
  const int f = 2 * (bb >> 3) + ((bb >> 2) & 1), i = bb & 3;
  return f * 32 + kg * 8 + 2 * i + h;
}

// ---------------------------------------------------------------------------------------------------
// scale-in kernel: one workgroup per (problem, token, chunk), one wave per 128-column block.
//   1. the block's products Ein[k,c] * vin[k] (fp32; zero for k >= K) go to LDS, 128 x 16
//   2. lane (kg, n) gathers its 32 values in operand order, undoes the nibble values, takes the block
//      exponent E (largest magnitude <= 7.5 * 2^E) and peels three fp6 limbs at scales E, E-4, E-8;
//      every residual is exact in fp32
//   3. the chunk's column sums of the quantised values close the record
// ---------------------------------------------------------------------------------------------------
constexpr int kProdStride = 18;   // floats per LDS row: lane groups 8 rows apart land on disjoint banks

__global__ __launch_bounds__(64 * CBX) void mx_scale_in_kernel(const StageProb* __restrict__ probs, StageProb single) {
  __shared__ __attribute__((aligned(16))) float prod[CBX][128 * kProdStride];
  __shared__ float csum[CBX][16];
  StageProb p;
  if (probs) p = probs[blockIdx.y];
  else p = single;
  const int nch = (p.KB + CBX - 1) / CBX;
  const int unit = blockIdx.x;
  if (unit >= nch * p.T) return;
  const int b = unit / nch, c = unit - b * nch;
  const int tid = threadIdx.x, lane = tid & 63;
  const int qb = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int kg = lane >> 4, n = lane & 15;
  unsigned char* out_chunk = (unsigned char*)p.xs + ((size_t)b * nch + c) * (size_t)(kChunkVecs * 16);
  unsigned char* blk = out_chunk + (size_t)qb * kBlockBytes;
  const int k0 = (c * CBX + qb) * kBlockCols;
  float* pr = prod[qb];

  // ---- 1. products: lane handles rows lane/2 + 32 i, modes 8 (lane & 1) .. + 7.  All eight loads are
  //         issued before the first use (one memory round trip per workgroup).
  {
    int kc[4];
    bool in[4];
    u32x4 raw[4];
    float xk[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int k = k0 + (lane >> 1) + 32 * i;
      in[i] = k < p.K;
      kc[i] = min(k, p.K - 1);
      raw[i] = ((g_u32x4_ptr)p.Ein)[(size_t)kc[i] * 2 + (lane & 1)];
    }
    const int64_t xrow = (int64_t)b * p.vin_ld;
    if (p.vin_dt == MDBF_F32) {
#pragma unroll
      for (int i = 0; i < 4; ++i) xk[i] = ((g_f32_ptr)p.vin)[xrow + kc[i]];
    } else {
      uint16_t h[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) h[i] = ((g_u16_ptr)p.vin)[xrow + kc[i]];
#pragma unroll
      for (int i = 0; i < 4; ++i)
        xk[i] = (p.vin_dt == MDBF_F16) ? (float)__builtin_bit_cast(_Float16, h[i])
                                       : __builtin_bit_cast(float, (uint32_t)h[i] << 16);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t w[4] = {raw[i].x, raw[i].y, raw[i].z, raw[i].w};
      float* dst = pr + ((lane >> 1) + 32 * i) * kProdStride + (lane & 1) * 8;
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const float lo = (float)__builtin_bit_cast(_Float16, (uint16_t)(w[t] & 0xFFFFu));
        const float hi = (float)__builtin_bit_cast(_Float16, (uint16_t)(w[t] >> 16));
        dst[2 * t] = in[i] ? lo * xk[i] : 0.f;
        dst[2 * t + 1] = in[i] ? hi * xk[i] : 0.f;
      }
    }
  }
  __syncthreads();

  // ---- 2. gather in operand order, quantise
  float val[32];
  float m = 0.f;
#pragma unroll
  for (int j = 0; j < 32; ++j) {
    const float presc = (j < 8) ? 2.f : (j < 16 ? 1.f : 0.5f);   // undo the nibble values 0.5, 1, 2, 2
    val[j] = pr[(local_col_of_element(j, 0) + 8 * kg) * kProdStride + n] * presc;
    m = fmaxf(m, fabsf(val[j]));
  }
  int E = -100;
  if (m > 0.f) {
    int ex;
    const float fr = frexpf(m, &ex);          // m = fr * 2^ex, fr in [0.5, 1)
    E = (fr <= 0.9375f) ? ex - 3 : ex - 2;     // 7.5 = 0.9375 * 2^3
    E = max(E, -100);
  }
  E = min(E, 120);
  const float sc1 = __builtin_bit_cast(float, (uint32_t)(E + 127) << 23);
  const float sc2 = __builtin_bit_cast(float, (uint32_t)(E + 123) << 23);
  const float sc3 = __builtin_bit_cast(float, (uint32_t)(E + 119) << 23);
  const v6u l1 = fp6_encode32(val, sc1);
  const v32f b1 = __builtin_amdgcn_cvt_scalef32_pk32_f32_fp6(l1, sc1);
  float r[32];
#pragma unroll
  for (int j = 0; j < 32; ++j) r[j] = val[j] - b1[j];
  const v6u l2 = fp6_encode32(r, sc2);
  const v32f b2 = __builtin_amdgcn_cvt_scalef32_pk32_f32_fp6(l2, sc2);
#pragma unroll
  for (int j = 0; j < 32; ++j) r[j] -= b2[j];
  const v6u l3 = fp6_encode32(r, sc3);
  const v32f b3 = __builtin_amdgcn_cvt_scalef32_pk32_f32_fp6(l3, sc3);
  // quantised value = val - (last residual); back at the scale of xs, summed over the lane's 32 columns
  float part = 0.f;
#pragma unroll
  for (int j = 0; j < 32; ++j) {
    const float inv = (j < 8) ? 0.5f : (j < 16 ? 1.f : 2.f);
    part += (val[j] - (r[j] - b3[j])) * inv;
  }
  const v6u limb[3] = {l1, l2, l3};
#pragma unroll
  for (int L = 0; L < 3; ++L) {
    u32x4 a;
    a.x = limb[L][0]; a.y = limb[L][1]; a.z = limb[L][2]; a.w = limb[L][3];
    u32x2 bpart;
    bpart.x = limb[L][4]; bpart.y = limb[L][5];
    reinterpret_cast<u32x4*>(blk + L * kLimbBytes)[lane] = a;
    reinterpret_cast<u32x2*>(blk + L * kLimbBytes + 64 * 16)[lane] = bpart;
  }
  reinterpret_cast<uint32_t*>(blk + kScaleOff)[lane] =
      (uint32_t)(E + 127) | ((uint32_t)(E + 123) << 8) | ((uint32_t)(E + 119) << 16);

  // ---- 3. column sums of the chunk
  part += __shfl_xor(part, 16);
  part += __shfl_xor(part, 32);
  if (lane < 16) csum[qb][lane] = part;
  __syncthreads();
  if (tid < 16) {
    float t = 0.f;
#pragma unroll
    for (int w = 0; w < CBX; ++w) t += csum[w][tid];
    reinterpret_cast<float*>(out_chunk + kColsumOff)[tid] = t;
  }
}

// ---------------------------------------------------------------------------------------------------
// main kernel
// ---------------------------------------------------------------------------------------------------
struct BlockOps {
  u32x4 la[3];
  u32x2 lb[3];
  uint32_t sc;
};

__device__ __forceinline__ void load_block_ops(const unsigned char* __restrict__ blk, int lane, BlockOps& o) {
#pragma unroll
  for (int L = 0; L < 3; ++L) {
    o.la[L] = reinterpret_cast<const u32x4*>(blk + L * kLimbBytes)[lane];
    o.lb[L] = reinterpret_cast<const u32x2*>(blk + L * kLimbBytes + 64 * 16)[lane];
  }
  o.sc = reinterpret_cast<const uint32_t*>(blk + kScaleOff)[lane];
}

__device__ __forceinline__ v8i limb_operand(const BlockOps& o, int L) {
  const u32x4 a = o.la[L];
  const u32x2 b = o.lb[L];
  v8i r;
  r[0] = (int)a.x; r[1] = (int)a.y; r[2] = (int)a.z; r[3] = (int)a.w;
  r[4] = (int)b.x; r[5] = (int)b.y; r[6] = 0; r[7] = 0;
  return r;
}

__device__ __forceinline__ v8i sign_operand(uint32_t w) {
  v8i r;
  r[0] = (int)(w & 0x11111111u);
  r[1] = (int)(w & 0x22222222u);
  r[2] = (int)(w & 0x44444444u);
  r[3] = (int)((w >> 1) & 0x44444444u);
  r[4] = 0; r[5] = 0; r[6] = 0; r[7] = 0;
  return r;
}

__device__ __forceinline__ floatx4 mx_mfma(v8i a, v8i b, floatx4 c, int L, uint32_t sc) {
  // A: fp4 (format 4), scale 2^0; B: fp6 e2m3 (format 2), scale byte L of sc
  if (L == 0) return __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, b, c, 4, 2, 0, 0x7F7F7F7F, 0, (int)sc);
  if (L == 1) return __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, b, c, 4, 2, 0, 0x7F7F7F7F, 1, (int)sc);
  return __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, b, c, 4, 2, 0, 0x7F7F7F7F, 2, (int)sc);
}

template <int R>
__device__ __forceinline__ void contract_block(const BlockOps& o, const uint32_t (&word)[R], floatx4 (&acc)[R]) {
  v8i bl[3];
#pragma unroll
  for (int L = 0; L < 3; ++L) bl[L] = limb_operand(o, L);
  v8i a[R];
#pragma unroll
  for (int r = 0; r < R; ++r) a[r] = sign_operand(word[r]);
  // limb outermost: consecutive instructions write different accumulators
#pragma unroll
  for (int L = 0; L < 3; ++L)
#pragma unroll
    for (int r = 0; r < R; ++r) acc[r] = mx_mfma(a[r], bl[L], acc[r], L, o.sc);
}

__device__ __forceinline__ float row16_sum(float v) {
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, true));
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x4E, 0xF, 0xF, true));
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x141, 0xF, 0xF, true));
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x140, 0xF, 0xF, true));
  return v;
}

template <int R>
struct Unit {
  StageProb p;
  int tile0, ntl, b, item;
  const uint32_t* sbase[R];
  const u32x4* xs_tok;
};

template <int R>
__device__ __forceinline__ void finish_unit(Unit<R>& u, int wave) {
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int trel = min(wave + 4 * r, u.ntl - 1);
    u.sbase[r] = u.p.S + (size_t)(u.tile0 + trel) * (size_t)(u.p.KB * 64);
  }
  const int nch = (u.p.KB + CBX - 1) / CBX;
  u.xs_tok = (const u32x4*)u.p.xs + (size_t)u.b * (size_t)nch * (size_t)kChunkVecs;
}

__device__ __forceinline__ uint32_t fetch_desc(const WorkItem* __restrict__ items, int item, int lane) {
  return ((g_u32_ptr)(items + item))[lane & 31];
}

template <int R, bool BATCH>
__device__ __forceinline__ void make_unit(uint32_t desc, const StageProb& single, int tiles_per_item, int item,
                                          int wave, Unit<R>& u) {
  if (BATCH) {
    uint32_t d[28];
#pragma unroll
    for (int i = 0; i < 28; ++i) d[i] = __builtin_amdgcn_readlane(desc, i);
    auto ptr = [&](int i) { return (uint64_t)d[i] | ((uint64_t)d[i + 1] << 32); };
    u.p.S = (const uint32_t*)ptr(0);
    u.p.Ein = (const void*)ptr(2);
    u.p.Eout = (const void*)ptr(4);
    u.p.vin = (const void*)ptr(6);
    u.p.out = (void*)ptr(8);
    u.p.xs = (void*)ptr(10);
    u.p.vin_ld = (int64_t)ptr(12);
    u.p.out_ld = (int64_t)ptr(14);
    u.p.rows = (int)d[16];
    u.p.K = (int)d[17];
    u.p.l = (int)d[18];
    u.p.T = (int)d[19];
    u.p.KB = (int)d[20];
    u.p.ntiles = (int)d[21];
    u.p.env_dt = (int)d[22];
    u.p.vin_dt = (int)d[23];
    u.p.out_dt = (int)d[24];
    u.p.pad_ = 0;
    u.tile0 = (int)d[26];
    u.ntl = (int)d[27];
  } else {
    u.p = single;
    u.tile0 = item * tiles_per_item;
    u.ntl = min(tiles_per_item, single.ntiles - u.tile0);
  }
  u.item = item;
  u.b = 0;
  finish_unit<R>(u, wave);
}

template <int R>
__device__ __forceinline__ void settle(uint32_t (&wq)[R][CBX]) {
#pragma unroll
  for (int r = 0; r < R; ++r)
#pragma unroll
    for (int j = 0; j < CBX; ++j) asm volatile("" : "+v"(wq[r][j]));
}

template <int R, bool BATCH>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2)))
void stage_mx_kernel(const WorkItem* __restrict__ items, int nitems, StageProb single, int tiles_per_item) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  u32x4* buf = reinterpret_cast<u32x4*>(smem);
  u32x4* eo = reinterpret_cast<u32x4*>(smem + 2 * kBufVecs * 16);

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int kg = lane >> 4, n = lane & 15;

  int item, i_hi, stride;
  if ((gridDim.x & 7) == 0) {
    const int xcd = blockIdx.x & 7;
    const int i_lo = (int)(((long)nitems * xcd) >> 3);
    i_hi = (int)(((long)nitems * (xcd + 1)) >> 3);
    stride = gridDim.x >> 3;
    item = i_lo + (blockIdx.x >> 3);
  } else {
    i_hi = nitems;
    stride = gridDim.x;
    item = blockIdx.x;
  }
  if (item >= i_hi) return;

  Unit<R> u;
  {
    uint32_t desc0 = 0;
    if (BATCH) desc0 = fetch_desc(items, item, lane);
    make_unit<R, BATCH>(desc0, single, tiles_per_item, item, wave, u);
  }

  // ---- prologue: first sign words and first chunk of the first unit
  uint32_t wq[R][CBX];
#pragma unroll
  for (int r = 0; r < R; ++r)
#pragma unroll
    for (int j = 0; j < CBX; ++j) wq[r][j] = ((g_u32_ptr)(u.sbase[r] + j * 64))[lane];   // KB >= CBX
  u32x4 cp[kCopyPerThread];
  {
    g_u32x4_ptr src = (g_u32x4_ptr)u.xs_tok + tid;
#pragma unroll
    for (int i = 0; i < kCopyPerThread; ++i) cp[i] = src[min(256 * i, kChunkVecs - 1 - tid)];
#pragma unroll
    for (int i = 0; i < kCopyPerThread; ++i) buf[tid + 256 * i] = cp[i];
  }
  int par = 0;
  __syncthreads();

  DBG_UNIT_DECL;
  for (;;) {
    DBG_UNIT_NEXT;
    DBG_T(0);
    settle<R>(wq);
    const bool next_token = (u.b + 1 < u.p.T);
    const int ni = u.item + stride;
    const bool has_next = next_token || (ni < i_hi);
    uint32_t desc_next = 0;
    if (BATCH) desc_next = fetch_desc(items, min(ni, nitems - 1), lane);
    Unit<R> un = u;

    floatx4 acc[R];
    float colsum = 0.f;
#pragma unroll
    for (int r = 0; r < R; ++r) acc[r] = floatx4{0.f, 0.f, 0.f, 0.f};

    const int KB = u.p.KB;
    const int nchunks = (KB + CBX - 1) / CBX;
    uint32_t wnext[R][CBX];

    // ---- all chunks but the last
#pragma unroll 1
    for (int c = 0; c < nchunks - 1; ++c) {
#pragma unroll
      for (int j = 0; j < CBX; ++j) {
        const int qn = (c + 1) * CBX + j;
        const uint64_t off = (qn < KB) ? (uint64_t)qn * 256u : 0u;
#pragma unroll
        for (int r = 0; r < R; ++r) wnext[r][j] = ((g_u32_ptr)((uint64_t)u.sbase[r] + off))[lane];
      }
      {
        g_u32x4_ptr src = (g_u32x4_ptr)u.xs_tok + ((size_t)(c + 1) * kChunkVecs + tid);
#pragma unroll
        for (int i = 0; i < kCopyPerThread; ++i) cp[i] = src[min(256 * i, kChunkVecs - 1 - tid)];
      }
      DBG_T(1 + 4 * c);
      const unsigned char* bufc = reinterpret_cast<const unsigned char*>(buf + par * kBufVecs);
#pragma unroll
      for (int jj = 0; jj < CBX; ++jj) {
        uint32_t word[R];
#pragma unroll
        for (int r = 0; r < R; ++r) word[r] = wq[r][jj];
        BlockOps ops;
        load_block_ops(bufc + jj * kBlockBytes, lane, ops);
        contract_block<R>(ops, word, acc);
      }
      colsum += reinterpret_cast<const float*>(bufc + kColsumOff)[n];
      DBG_T(2 + 4 * c);
      {
        u32x4* dst = buf + (par ^ 1) * kBufVecs;
#pragma unroll
        for (int i = 0; i < kCopyPerThread; ++i) dst[tid + 256 * i] = cp[i];
      }
      DBG_T(3 + 4 * c);
      __syncthreads();
      DBG_T(4 + 4 * c);
      par ^= 1;
#pragma unroll
      for (int r = 0; r < R; ++r)
#pragma unroll
        for (int j = 0; j < CBX; ++j) wq[r][j] = wnext[r][j];
      settle<R>(wq);   // the wait for the prefetched words belongs here, after the chunk's contraction
    }

    // ---- the last chunk: the next unit's first chunk and this unit's Eout rows are requested up front
    {
      const int c = nchunks - 1;
      settle<R>(wq);
      asm volatile("" : "+v"(desc_next));
      if (next_token) {
        un.b = u.b + 1;
        finish_unit<R>(un, wave);
      } else if (has_next) {
        make_unit<R, BATCH>(desc_next, single, tiles_per_item, ni, wave, un);
      }
#pragma unroll
      for (int r = 0; r < R; ++r)
#pragma unroll
        for (int j = 0; j < CBX; ++j) wnext[r][j] = ((g_u32_ptr)(un.sbase[r] + j * 64))[lane];
      {
        g_u32x4_ptr src = (g_u32x4_ptr)un.xs_tok + tid;
#pragma unroll
        for (int i = 0; i < kCopyPerThread; ++i) cp[i] = src[min(256 * i, kChunkVecs - 1 - tid)];
      }
      u32x4 eoreg[eo_vecs(R) / 256];
#pragma unroll
      for (int t = 0; t < eo_vecs(R) / 256; ++t) {
        const int v = tid + 256 * t;
        const int row = min(u.tile0 * kTileRows + (v >> 1), u.p.rows - 1);
        eoreg[t] = ((g_u32x4_ptr)u.p.Eout)[(size_t)row * 2 + (v & 1)];
      }
      DBG_T(1 + 4 * c);
      const unsigned char* bufc = reinterpret_cast<const unsigned char*>(buf + par * kBufVecs);
#pragma unroll
      for (int jj = 0; jj < CBX; ++jj) {
        if (c * CBX + jj < KB) {
          uint32_t word[R];
#pragma unroll
          for (int r = 0; r < R; ++r) word[r] = wq[r][jj];
          BlockOps ops;
          load_block_ops(bufc + jj * kBlockBytes, lane, ops);
          contract_block<R>(ops, word, acc);
        }
      }
      colsum += reinterpret_cast<const float*>(bufc + kColsumOff)[n];
      DBG_T(2 + 4 * c);
#pragma unroll
      for (int t = 0; t < eo_vecs(R) / 256; ++t) eo[tid + 256 * t] = eoreg[t];
      {
        u32x4* dst = buf + (par ^ 1) * kBufVecs;
#pragma unroll
        for (int i = 0; i < kCopyPerThread; ++i) dst[tid + 256 * i] = cp[i];
      }
      DBG_T(3 + 4 * c);
      __syncthreads();
      DBG_T(4 + 4 * c);
      par ^= 1;
    }
    DBG_T(40);

    // ---- epilogue
    const _Float16* eoh = reinterpret_cast<const _Float16*>(eo);
    float res[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const int trel = min(wave + 4 * r, u.ntl - 1);
      float v[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float ev = (float)eoh[(trel * kTileRows + 4 * kg + i) * 16 + n];
        const float P = colsum - 2.f * acc[r][i];
        v[i] = row16_sum(ev * P);
      }
      const int sel = n & 3;
      res[r] = sel == 0 ? v[0] : sel == 1 ? v[1] : sel == 2 ? v[2] : v[3];
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const int row = (u.tile0 + wave + 4 * r) * kTileRows + 4 * kg + n;
      if ((wave + 4 * r) < u.ntl && n < 4 && row < u.p.rows)
        store_from_float(u.p.out, (int64_t)u.b * u.p.out_ld + row, u.p.out_dt, res[r]);
    }
    DBG_T(41);
    if (!has_next) break;
    // a one-chunk unit writes eo again before any other barrier: wait for the slowest reader
    if (nchunks == 1) __syncthreads();
    u = un;
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
      for (int j = 0; j < CBX; ++j) wq[r][j] = wnext[r][j];
  }
}

template <int R, bool BATCH>
static int launch_rb(const WorkItem* items_dev, int nitems, int tiles_per_item, const StageProb* single,
                     hipStream_t s) {
  static bool attr_set = false;
  static int max_wgs = 512;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&stage_mx_kernel<R, BATCH>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, smem_bytes(R));
    if (e != hipSuccess) return (int)e;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus > 0)
      max_wgs = 2 * cus;
    attr_set = true;
  }
  const int nwg = nitems < max_wgs ? nitems : max_wgs;
  hipLaunchKernelGGL((stage_mx_kernel<R, BATCH>), dim3((unsigned)nwg), dim3(256), smem_bytes(R), s, items_dev,
                     nitems, *single, tiles_per_item);
  return (int)hipGetLastError();
}

}  // namespace mx

#ifdef MDBF_DBG_TIMING
extern "C" int mdbf_dbg_read_mx(void* host, size_t bytes) {
  return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(mx::g_dbg_time_mx),
                                  bytes < sizeof(mx::g_dbg_time_mx) ? bytes : sizeof(mx::g_dbg_time_mx));
}
#endif

int launch_scale_in_mx(const StageProb* probs_dev, int count, int max_units, const StageProb* single, hipStream_t s) {
  hipLaunchKernelGGL(mx::mx_scale_in_kernel, dim3((unsigned)max_units, (unsigned)count), dim3(64 * mx::CBX), 0, s, probs_dev,
                     *single);
  return (int)hipGetLastError();
}

size_t xs_bytes_for_mx(int K, int T) {
  const int nch = (num_blocks(K) + mx::CBX - 1) / mx::CBX;
  return (size_t)T * (size_t)nch * (size_t)mx::kChunkVecs * 16u;
}

int mx_chunks(int KB) { return (KB + mx::CBX - 1) / mx::CBX; }

bool stage_is_mx(const StageProb& p) {
  return p.l == 16 && p.env_dt == MDBF_F16 && p.KB >= mx::CBX && p.xs != nullptr && p.T <= kMaxPreTokens;
}

int launch_stage_mx(const StageProb* probs_dev, const WorkItem* items_dev, int nitems, int tiles_per_item,
                    const StageProb* single, hipStream_t s) {
  if (!probs_dev) nitems = (single->ntiles + tiles_per_item - 1) / tiles_per_item;
  switch (tiles_per_item) {
    case 4: return probs_dev ? mx::launch_rb<1, true>(items_dev, nitems, tiles_per_item, single, s)
                             : mx::launch_rb<1, false>(items_dev, nitems, tiles_per_item, single, s);
    case 8: return probs_dev ? mx::launch_rb<2, true>(items_dev, nitems, tiles_per_item, single, s)
                             : mx::launch_rb<2, false>(items_dev, nitems, tiles_per_item, single, s);
    case 16: return probs_dev ? mx::launch_rb<4, true>(items_dev, nitems, tiles_per_item, single, s)
                              : mx::launch_rb<4, false>(items_dev, nitems, tiles_per_item, single, s);
    default: return (int)hipErrorInvalidValue;
  }
}

}  // namespace mdbf
