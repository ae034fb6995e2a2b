// Matrix-core evaluation of one envelope-scaled binary product on gfx950: the FAST variant
// (l == 16, fp16 envelopes, K >= 897 and a multiple of 8, 16-byte aligned activation rows).
//
//   out[r] = sum_c Eout[r,c] * P[r,c],     P[r,c] = sum_j S[r,j] * xs[j,c],   xs[j,c] = fp16(Ein[j,c] * vin[j])
//
// (paper Eq. "me-dbf-expand": per factor, l envelope-scaled copies of the shared sign basis).
// P is a skinny GEMM (rows x K) . (K x 16): exactly one 16x16x32 fp16 MFMA tile wide.
//
// Work decomposition: a unit of work is (up to 4*R row tiles of one problem, one token, the whole
// contraction).  Workgroups of four wavefronts are persistent: each walks a list of units, and the
// loads of the next unit (its first sign words, its first chunk of envelope rows) are issued while
// the current unit finishes, so that no unit starts or ends on an exposed memory latency.
// Wave w owns tiles w, w+4, ... of the unit.  The scaled activations xs are staged chunk by chunk
// (1024 columns) in LDS in the order the MFMA B operand wants them and shared by all tiles of the
// workgroup; sign words stream from HBM one chunk (1024 columns) ahead of their use.
//
// Sign expansion without shifts: with bit t=1 meaning -1,  S = 1 - 2t, hence
//      P[r,c] = colsum[c] - 2 * sum_j t[r,j] xs[j,c].
// The A operand of an MFMA step is  w & mask : the two selected bits of a word, read as two fp16
// values, are 0 or 2^(p-24) (p = bit position 0..7; fp16 denormals are honoured by the MFMA).  The
// staged activation of the entry at position p = 4c+i carries the factor 2^-i, so every product of
// class c (positions 4c..4c+3) is scaled by 2^(4c-24) exactly, and each class has its own fp32
// accumulator.  Bits 8..15 of each half word are brought down with one shift per word.
// colsum comes from the same MFMAs applied to a virtual row whose bits are all 1, so that it sees
// exactly the staged (rounded) values; wave w contracts MFMA step f == w of every block for it.
#include <type_traits>

#include "mdbf_internal.h"

namespace mdbf {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

typedef const MDBF_GLOBAL u32x4* g_u32x4_ptr;
typedef const MDBF_GLOBAL uint32_t* g_u32_ptr;
typedef const MDBF_GLOBAL floatx4* g_f32x4_ptr;
typedef const MDBF_GLOBAL _Float16* g_f16_ptr;
typedef const MDBF_GLOBAL uint16_t* g_u16_ptr;
typedef const MDBF_GLOBAL float* g_f32_ptr;

constexpr int CB = 8;                      // 128-column blocks per LDS chunk
constexpr int kChunkVecs = CB * 4 * 64;    // 16-byte vectors per chunk buffer (32 KB)
constexpr int kLoadSteps = 1;               // the next chunk's loads are issued during this many block steps (1, 2 or 4)
constexpr int kPrefetchBlocks = CB;        // sign words are loaded one chunk (8 blocks) ahead of their use
__host__ __device__ constexpr int eo_vecs(int R) { return R * 4 * 16 * 2 < 256 ? 256 : R * 4 * 16 * 2; }  // Eout rows of a unit, 16 B each, a multiple of the 256 threads
__host__ __device__ constexpr int fast_smem_bytes(int R) { return 2 * kChunkVecs * 16 + eo_vecs(R) * 16 + 4 * 16 * 4; }

__device__ __forceinline__ half8 expand(uint32_t src, int c) {
  // class c: bit positions 4c..4c+3 and the same 16 above
  const uint32_t m0 = 0x00010001u << (4 * c);
  u32x4 a;
  a.x = src & m0;
  a.y = src & (m0 << 1);
  a.z = src & (m0 << 2);
  a.w = src & (m0 << 3);
  return __builtin_bit_cast(half8, a);
}

// {fp16(lo16(e0) * x0), fp16(lo16(e1) * x1)} with one rounding each (mixed-precision fma)
__device__ __forceinline__ uint32_t mix_pair_lo(uint32_t e0, uint32_t e1, float x0, float x1) {
  uint32_t out;
  asm("v_fma_mixlo_f16 %0, %1, %2, 0 op_sel:[0,0,0] op_sel_hi:[1,0,0]" : "=v"(out) : "v"(e0), "v"(x0));
  asm("v_fma_mixhi_f16 %0, %1, %2, 0 op_sel:[0,0,0] op_sel_hi:[1,0,0]" : "+v"(out) : "v"(e1), "v"(x1));
  return out;
}
// the same for the upper halves of e0, e1
__device__ __forceinline__ uint32_t mix_pair_hi(uint32_t e0, uint32_t e1, float x0, float x1) {
  uint32_t out;
  asm("v_fma_mixlo_f16 %0, %1, %2, 0 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(out) : "v"(e0), "v"(x0));
  asm("v_fma_mixhi_f16 %0, %1, %2, 0 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "+v"(out) : "v"(e1), "v"(x1));
  return out;
}

// sum over the 16 lanes of a DPP row (result valid in every lane of the row)
__device__ __forceinline__ float row16_sum(float v) {
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, true));
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x4E, 0xF, 0xF, true));
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x141, 0xF, 0xF, true));
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x140, 0xF, 0xF, true));
  return v;
}

struct StageRegs {
  u32x4 e[8];    // 8 envelope rows of one column octet, 8 fp16 modes each
  u32x4 xr[2];   // the octet's 8 activations as loaded (xr[1] differs from xr[0] only for fp32)
  float vmask;   // 1 if the octet lies inside K, else 0
};

// Thread (oo = tid/2, ch = tid%2) stages the octet of columns `kcol..kcol+7` for modes 8ch..8ch+7.
// Octets at or beyond K read the (valid) first octet instead and get zero activations.  Only loads
// are issued here, with no branch around them; nothing waits for them until stage_store.  The loads
// come in four parts so that the caller can spread them over several block steps.
struct StageAddr {
  g_u32x4_ptr ep;                 // first envelope row of the octet, this thread's column half
  const char MDBF_GLOBAL* xb;     // first activation of the octet
  int x2off;                      // byte offset of the second activation vector (fp32 only, else 0)
};

__device__ __forceinline__ void stage_addr(const void* ein, int ch, const void* vin_row, int vin_dt, int kcol, int K,
                                           StageRegs& sr, StageAddr& sa) {
  const bool valid = kcol < K;
  const int kc = valid ? kcol : 0;
  sr.vmask = valid ? 1.f : 0.f;
  sa.ep = (g_u32x4_ptr)ein + ((size_t)kc * 2 + ch);
  const int esz_shift = (vin_dt == MDBF_F32) ? 2 : 1;
  sa.xb = (const char MDBF_GLOBAL*)vin_row + ((size_t)kc << esz_shift);
  sa.x2off = (vin_dt == MDBF_F32) ? 16 : 0;
}

__device__ __forceinline__ void stage_load_part(const StageAddr& sa, int part, StageRegs& sr) {
  sr.e[2 * part] = sa.ep[4 * part];
  sr.e[2 * part + 1] = sa.ep[4 * part + 2];
  if (part == 0) {
    sr.xr[0] = *(g_u32x4_ptr)sa.xb;
    sr.xr[1] = *(g_u32x4_ptr)(sa.xb + sa.x2off);
  }
}

__device__ __forceinline__ void stage_load(const void* ein, int ch, const void* vin_row, int vin_dt, int kcol, int K,
                                           StageRegs& sr) {
  StageAddr sa;
  stage_addr(ein, ch, vin_row, vin_dt, kcol, K, sr, sa);
#pragma unroll
  for (int part = 0; part < 4; ++part) stage_load_part(sa, part, sr);
}

// dst: the thread's 8 consecutive 16-byte slots (modes 8ch..8ch+7 of its octet); slot cc is stored at
// cc ^ sw so that the 64 lanes of one store instruction spread over all LDS banks.
__device__ __forceinline__ void stage_store(const StageRegs& sr, int vin_dt, u32x4* dst, int sw, float scale) {
  // activations as fp32, times 2^-(e/2) (the position factor of the sign expansion), times the K mask,
  // times the chunk's power-of-two scale (1 when the kernel stages for itself)
  float x[8];
  const u32x4 x0 = sr.xr[0], x1 = sr.xr[1];
  if (vin_dt == MDBF_F32) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const uint32_t bits = (e < 4) ? x0[e & 3] : x1[e & 3];
      x[e] = __builtin_bit_cast(float, bits);
    }
  } else if (vin_dt == MDBF_F16) {
    const half8 xh = __builtin_bit_cast(half8, x0);
#pragma unroll
    for (int e = 0; e < 8; ++e) x[e] = (float)xh[e];
  } else {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const uint32_t wd = x0[e >> 1];
      const uint32_t bits = (e & 1) ? (wd & 0xFFFF0000u) : (wd << 16);
      x[e] = __builtin_bit_cast(float, bits);
    }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) x[e] *= (sr.vmask * scale) * (1.0f / (float)(1 << (e >> 1)));
#pragma unroll
  for (int cc = 0; cc < 8; ++cc) {
    u32x4 v;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const u32x4 r0 = sr.e[2 * i], r1 = sr.e[2 * i + 1];
      const uint32_t a0 = r0[cc >> 1], a1 = r1[cc >> 1];
      const uint32_t pr = (cc & 1) ? mix_pair_hi(a0, a1, x[2 * i], x[2 * i + 1])
                                   : mix_pair_lo(a0, a1, x[2 * i], x[2 * i + 1]);
      v[i] = pr;
    }
    dst[cc ^ sw] = v;
  }
}

// 2^d for an integer -126 <= d <= 127
__device__ __forceinline__ float pow2i(int d) { return __builtin_bit_cast(float, (uint32_t)(127 + d) << 23); }

// Largest |Ein[k, c] * vin[k]| over the thread's octet of columns and its eight modes (0 outside K).
__device__ __forceinline__ float stage_absmax(const StageRegs& sr, int vin_dt) {
  float x[8];
  const u32x4 x0 = sr.xr[0], x1 = sr.xr[1];
  if (vin_dt == MDBF_F32) {
#pragma unroll
    for (int e = 0; e < 8; ++e) x[e] = __builtin_bit_cast(float, (e < 4) ? x0[e & 3] : x1[e & 3]);
  } else if (vin_dt == MDBF_F16) {
    const half8 xh = __builtin_bit_cast(half8, x0);
#pragma unroll
    for (int e = 0; e < 8; ++e) x[e] = (float)xh[e];
  } else {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const uint32_t wd = x0[e >> 1];
      x[e] = __builtin_bit_cast(float, (e & 1) ? (wd & 0xFFFF0000u) : (wd << 16));
    }
  }
  float m = 0.f;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    typedef _Float16 half2v __attribute__((ext_vector_type(2)));
    const u32x4 w = sr.e[e];
    const half2v a0 = __builtin_elementwise_abs(__builtin_bit_cast(half2v, w.x));
    const half2v a1 = __builtin_elementwise_abs(__builtin_bit_cast(half2v, w.y));
    const half2v a2 = __builtin_elementwise_abs(__builtin_bit_cast(half2v, w.z));
    const half2v a3 = __builtin_elementwise_abs(__builtin_bit_cast(half2v, w.w));
    const half2v mm = __builtin_elementwise_max(__builtin_elementwise_max(a0, a1), __builtin_elementwise_max(a2, a3));
    const float rm = fmaxf((float)mm.x, (float)mm.y);
    m = fmaxf(m, rm * fabsf(x[e]));
  }
  return m * sr.vmask;
}

// How a workgroup gets the scaled activations of a chunk into LDS.
//  PRE = false: computes them itself from Ein and vin (stage_addr / stage_load_part / stage_store).
//  PRE = true : the scale-in kernel has written them, in LDS order, to the problem's xs buffer; the
//               workgroup copies 32 KB per chunk (8 vectors per thread), no arithmetic.
template <bool PRE>
struct Stager;

template <>
struct Stager<false> {
  StageRegs sr;
  StageAddr sa;
  int vin_dt;
  __device__ __forceinline__ void addr(const void* ein, const void* vin_row, int dt, const u32x4* /*xs_tok*/, int chunk,
                                       int K, int ch, int st_col, int /*tid*/) {
    vin_dt = dt;
    stage_addr(ein, ch, vin_row, dt, chunk * (CB * kBlockCols) + st_col, K, sr, sa);
  }
  __device__ __forceinline__ void load_part(int part) { stage_load_part(sa, part, sr); }
  __device__ __forceinline__ void store(u32x4* bufbase, int st_vec, int st_sw, int /*tid*/) {
    stage_store(sr, vin_dt, bufbase + st_vec, st_sw, 1.0f);
  }
};

template <>
struct Stager<true> {
  u32x4 cp[8];
  g_u32x4_ptr src;
  __device__ __forceinline__ void addr(const void*, const void*, int, const u32x4* xs_tok, int chunk, int, int, int,
                                       int tid) {
    src = (g_u32x4_ptr)xs_tok + ((size_t)chunk * kChunkVecs + tid);
  }
  __device__ __forceinline__ void load_part(int part) {
    cp[2 * part] = src[(2 * part) * 256];
    cp[2 * part + 1] = src[(2 * part + 1) * 256];
  }
  __device__ __forceinline__ void store(u32x4* bufbase, int, int, int tid) {
#pragma unroll
    for (int i = 0; i < 8; ++i) bufbase[tid + 256 * i] = cp[i];
  }
};

// B operands of one block: the four MFMA steps plus this wave's share of the virtual row.
struct BlockOps {
  u32x4 v[5];
};

__device__ __forceinline__ void load_block_ops(const u32x4* __restrict__ blk, int rd_even, int rd_odd, int rd_virt,
                                               BlockOps& o) {
  o.v[0] = blk[rd_even];
  o.v[1] = blk[64 + rd_odd];
  o.v[2] = blk[128 + rd_even];
  o.v[3] = blk[192 + rd_odd];
  o.v[4] = blk[rd_virt];
}

template <int R>
__device__ __forceinline__ void contract_block(const BlockOps& o, const half8 avirt, const uint32_t (&word)[R],
                                               floatx4 (&acc)[R][2], floatx4& accv) {
  uint32_t hi[R];
#pragma unroll
  for (int r = 0; r < R; ++r) hi[r] = word[r] >> 8;
#pragma unroll
  for (int f = 0; f < 4; ++f) {
    const half8 bop = __builtin_bit_cast(half8, o.v[f]);
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const uint32_t src = (f < 2) ? word[r] : hi[r];
      acc[r][f & 1] = __builtin_amdgcn_mfma_f32_16x16x32_f16(expand(src, f & 1), bop, acc[r][f & 1], 0, 0, 0);
    }
  }
  accv = __builtin_amdgcn_mfma_f32_16x16x32_f16(avirt, __builtin_bit_cast(half8, o.v[4]), accv, 0, 0, 0);
}

// Makes the compiler wait, here, for the sign words that were loaded by an earlier loop iteration:
// across loop boundaries it cannot count which loads are still in flight and would otherwise wait
// for ALL outstanding loads at every later first use, including the ones just issued.
template <int R>
__device__ __forceinline__ void settle(uint32_t (&wq)[R][kPrefetchBlocks]) {
#pragma unroll
  for (int r = 0; r < R; ++r)
#pragma unroll
    for (int j = 0; j < kPrefetchBlocks; ++j) asm volatile("" : "+v"(wq[r][j]));
}

// Wave-uniform description of a unit.  sbase[r] is the first sign word of the r-th tile of this wave.
template <int R>
struct Unit {
  StageProb p;
  int tile0, ntl, b, item;
  uint32_t bstride;      // bytes between consecutive blocks of a tile (the unit lies inside one tile group)
  const uint32_t* sbase[R];
  const void* vin_row;
  const u32x4* xs_tok;   // pre-scaled activations of the unit's token (all chunks), or null
  const int* xs_exp;     // their power-of-two exponents, one per chunk (behind the activations of all tokens)
};

template <int R>
__device__ __forceinline__ void finish_unit(Unit<R>& u, int wave) {
  // Tiles of this wave: tile0 + wave + 4*r.  Tiles past the end of the unit are replaced by the unit's
  // last tile (their results are not stored), which keeps the contraction loop free of branches.
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int trel = min(wave + 4 * r, u.ntl - 1);
    u.sbase[r] = u.p.S + tile_base_words(u.tile0 + trel, u.p.KB);
  }
  u.bstride = (uint32_t)group_tiles(u.tile0, u.p.ntiles) * 256u;
  u.vin_row = (const char*)u.p.vin + (size_t)u.b * (size_t)u.p.vin_ld * (size_t)dtype_size(u.p.vin_dt);
  const int nch = (u.p.KB + CB - 1) / CB;
  u.xs_tok = (const u32x4*)u.p.xs + (size_t)u.b * (size_t)nch * (size_t)kChunkVecs;
  u.xs_exp = (const int*)((const u32x4*)u.p.xs + (size_t)u.p.T * (size_t)nch * (size_t)kChunkVecs) + (size_t)u.b * nch;
}

// In batch mode the 128-byte work item is fetched one dword per lane and broadcast to scalar registers
// later; a single call derives its units arithmetically.
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
    u.p.flags = (int)d[25];
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

template <int R, bool BATCH, bool PRE>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2)))
void stage_fast_kernel(const WorkItem* __restrict__ items, int nitems, StageProb single, int tiles_per_item) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  u32x4* buf = reinterpret_cast<u32x4*>(smem);
  u32x4* eo = reinterpret_cast<u32x4*>(smem + 2 * kChunkVecs * 16);
  float* red = reinterpret_cast<float*>(smem + 2 * kChunkVecs * 16 + eo_vecs(R) * 16);

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform, and known to be

  // ---- the units of this workgroup.  Workgroups are dealt round-robin to the 8 XCDs; each XCD gets a
  // contiguous range of items, walked by its workgroups side by side, so that the items of one problem
  // (which share Ein) meet in one L2 at about the same time.
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

  // staging role of this thread
  const int ch = tid & 1, oo = tid >> 1;
  const int st_q = oo >> 4, st_f = (oo & 15) >> 2, st_kg = oo & 3;
  const int st_col = st_q * kBlockCols + st_f * 32 + st_kg * 8;            // column inside a chunk
  const int st_vec = (st_q * 4 + st_f) * 64 + st_kg * 16 + ch * 8;         // first of its 8 LDS slots
  const int st_sw = (st_kg + 4 * (st_f & 1)) & 7;

  // B-operand read slots of this lane (same swizzle as the stores)
  const int kg = lane >> 4, n = lane & 15;
  const int rd_even = kg * 16 + ((n & 8) | ((n & 7) ^ (kg & 7)));
  const int rd_odd = kg * 16 + ((n & 8) | ((n & 7) ^ ((kg + 4) & 7)));
  // the virtual all-ones row: wave w contracts MFMA step f == w of every block (class w & 1)
  const int rd_virt = wave * 64 + ((wave & 1) ? rd_odd : rd_even);
  const half8 avirt = (wave & 1) ? expand(0xFFFFFFFFu, 1) : expand(0xFFFFFFFFu, 0);
  const float virt_scale = (wave & 1) ? 1048576.f : 16777216.f;  // 2^20 : 2^24

  Unit<R> u;
  {
    uint32_t desc0 = 0;
    if (BATCH) desc0 = fetch_desc(items, item, lane);
    make_unit<R, BATCH>(desc0, single, tiles_per_item, item, wave, u);
  }

  // ---- prologue: first sign words and first chunk of the first unit
  uint32_t wq[R][kPrefetchBlocks];
#pragma unroll
  for (int r = 0; r < R; ++r)
#pragma unroll
    for (int j = 0; j < kPrefetchBlocks; ++j)
      wq[r][j] = ((g_u32_ptr)((uint64_t)u.sbase[r] + (uint64_t)j * u.bstride))[lane];   // KB >= 8 for every fast problem
  Stager<PRE> stg;
  stg.addr(u.p.Ein, u.vin_row, u.p.vin_dt, u.xs_tok, 0, u.p.K, ch, st_col, tid);
#pragma unroll
  for (int part = 0; part < 4; ++part) stg.load_part(part);
  int par = 0;
  stg.store(buf, st_vec, st_sw, tid);
  __syncthreads();

  // Pre-scaled activations come with one power-of-two exponent per chunk (the scale-in kernel puts every
  // chunk's largest magnitude at 2^12): the accumulators are carried in the current chunk's scale and
  // brought to the next chunk's at the boundary; the result is scaled back at the end.
  int e_cur = PRE ? ((const MDBF_GLOBAL int*)u.xs_exp)[0] : 0;
  for (;;) {
    settle<R>(wq);
    // ---- which unit comes next: the next token of the same item, else this workgroup's next item,
    //      whose descriptor is requested now and only looked at when this unit's last chunk starts
    const bool next_token = (u.b + 1 < u.p.T);
    const int ni = u.item + stride;
    const bool has_next = next_token || (ni < i_hi);
    uint32_t desc_next = 0;
    if (BATCH) desc_next = fetch_desc(items, min(ni, nitems - 1), lane);
    Unit<R> un = u;

    floatx4 acc[R][2];
    floatx4 accv = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int r = 0; r < R; ++r) {
      acc[r][0] = floatx4{0.f, 0.f, 0.f, 0.f};
      acc[r][1] = floatx4{0.f, 0.f, 0.f, 0.f};
    }

    const int KB = u.p.KB;
    const int nchunks = (KB + CB - 1) / CB;
    int e_unit_next = 0;

    // ---- all chunks but the last.  The sign words and the envelope rows of the next chunk are requested
    //      up front, into registers of their own, and have the whole chunk to arrive; blocks that do
    //      not exist are replaced by a harmless reload of block 0 so that no branch surrounds a load.
    uint32_t wnext[R][kPrefetchBlocks];
#pragma unroll 1
    for (int c = 0; c < nchunks - 1; ++c) {
      const int e_nx = PRE ? ((const MDBF_GLOBAL int*)u.xs_exp)[c + 1] : 0;
      stg.addr(u.p.Ein, u.vin_row, u.p.vin_dt, u.xs_tok, c + 1, u.p.K, ch, st_col, tid);
      const u32x4* bufc = buf + par * kChunkVecs;
#pragma unroll
      for (int jj = 0; jj < CB; ++jj) {
        if (jj < kLoadSteps) {
          // a share of the next chunk's loads per step: they are all several steps old when the chunk
          // ends, and they do not arrive at the memory pipeline in one burst
#pragma unroll
          for (int j = (CB / kLoadSteps) * jj; j < (CB / kLoadSteps) * (jj + 1); ++j) {
            const int qn = (c + 1) * CB + j;
            const uint64_t off = (qn < KB) ? (uint64_t)qn * u.bstride : 0u;
#pragma unroll
            for (int r = 0; r < R; ++r) wnext[r][j] = ((g_u32_ptr)((uint64_t)u.sbase[r] + off))[lane];
          }
#pragma unroll
          for (int part = (4 / kLoadSteps) * jj; part < (4 / kLoadSteps) * (jj + 1); ++part) stg.load_part(part);
        }
        uint32_t word[R];
#pragma unroll
        for (int r = 0; r < R; ++r) word[r] = wq[r][jj];
        BlockOps ops;
        load_block_ops(bufc + jj * 256, rd_even, rd_odd, rd_virt, ops);
        contract_block<R>(ops, avirt, word, acc, accv);
      }
      stg.store(buf + (par ^ 1) * kChunkVecs, st_vec, st_sw, tid);
      __syncthreads();
      par ^= 1;
#pragma unroll
      for (int r = 0; r < R; ++r)
#pragma unroll
        for (int j = 0; j < kPrefetchBlocks; ++j) wq[r][j] = wnext[r][j];
      if (PRE) {
        const float f = pow2i(max(-126, min(127, e_nx - e_cur)));
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            acc[r][0][i] *= f;
            acc[r][1][i] *= f;
          }
#pragma unroll
        for (int i = 0; i < 4; ++i) accv[i] *= f;
        e_cur = e_nx;
      }
    }

    // ---- the last chunk.  All loads of the next unit (its first chunk of sign words and of envelope
    //      rows) and this unit's Eout rows are issued up front, into registers of their own, so that
    //      they have a whole chunk of contraction time to arrive.
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
      stg.addr(un.p.Ein, un.vin_row, un.p.vin_dt, un.xs_tok, 0, un.p.K, ch, st_col, tid);
      e_unit_next = PRE ? ((const MDBF_GLOBAL int*)un.xs_exp)[0] : 0;
      u32x4 eoreg[eo_vecs(R) / 256];
#pragma unroll
      for (int t = 0; t < eo_vecs(R) / 256; ++t) {
        const int v = tid + 256 * t;
        const int row = min(u.tile0 * kTileRows + (v >> 1), u.p.rows - 1);
        eoreg[t] = ((g_u32x4_ptr)u.p.Eout)[(size_t)row * 2 + (v & 1)];
      }
      const u32x4* bufc = buf + par * kChunkVecs;
#pragma unroll
      for (int jj = 0; jj < CB; ++jj) {
        if (jj < kLoadSteps) {
#pragma unroll
          for (int j = (CB / kLoadSteps) * jj; j < (CB / kLoadSteps) * (jj + 1); ++j)
#pragma unroll
            for (int r = 0; r < R; ++r) wnext[r][j] = ((g_u32_ptr)((uint64_t)un.sbase[r] + (uint64_t)j * un.bstride))[lane];
#pragma unroll
          for (int part = (4 / kLoadSteps) * jj; part < (4 / kLoadSteps) * (jj + 1); ++part) stg.load_part(part);
        }
        if (c * CB + jj < KB) {
          uint32_t word[R];
#pragma unroll
          for (int r = 0; r < R; ++r) word[r] = wq[r][jj];
          BlockOps ops;
          load_block_ops(bufc + jj * 256, rd_even, rd_odd, rd_virt, ops);
          contract_block<R>(ops, avirt, word, acc, accv);
        }
      }
      red[wave * 16 + n] = accv[0] * virt_scale;   // all output rows of the virtual tile are equal
#pragma unroll
      for (int t = 0; t < eo_vecs(R) / 256; ++t) eo[tid + 256 * t] = eoreg[t];
      stg.store(buf + (par ^ 1) * kChunkVecs, st_vec, st_sw, tid);
      __syncthreads();
      par ^= 1;
    }

    // ---- epilogue: column sums, fix-up, envelope accumulate, store --------------------------------
    const float colsum = (red[n] + red[16 + n]) + (red[32 + n] + red[48 + n]);
    const _Float16* eoh = reinterpret_cast<const _Float16*>(eo);
    const float unscale = PRE ? pow2i(-e_cur) : 1.f;
    float res[R];   // lane (kg, n < 4) ends up with the result of row 4*kg + n of tile r
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const int trel = min(wave + 4 * r, u.ntl - 1);
      float v[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float ev = (float)eoh[(trel * kTileRows + 4 * kg + i) * 16 + n];
        const float P = colsum - acc[r][0][i] * 33554432.f - acc[r][1][i] * 2097152.f;  // 2^25, 2^21
        v[i] = row16_sum(ev * P);
      }
      const int sel = n & 3;
      res[r] = (sel == 0 ? v[0] : sel == 1 ? v[1] : sel == 2 ? v[2] : v[3]) * unscale;
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const int row = (u.tile0 + wave + 4 * r) * kTileRows + 4 * kg + n;
      if ((wave + 4 * r) < u.ntl && n < 4 && row < u.p.rows)
        emit_result(u.p.out, (int64_t)u.b * u.p.out_ld + row, u.p.out_dt, res[r], u.p.flags);
    }
    e_cur = e_unit_next;
    if (!has_next) break;
    // a one-chunk unit writes red / eo again before any other barrier: wait for the slowest reader
    if (nchunks == 1) __syncthreads();
    u = un;
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
      for (int j = 0; j < kPrefetchBlocks; ++j) wq[r][j] = wnext[r][j];
  }
}

template <int R, bool BATCH, bool PRE>
static int launch_rbp(const WorkItem* items_dev, int nitems, int tiles_per_item, const StageProb* single,
                      hipStream_t s) {
  static KernelSetup setup;
  if (int e = kernel_setup(setup, [] {
        return hipFuncSetAttribute(reinterpret_cast<const void*>(&stage_fast_kernel<R, BATCH, PRE>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, fast_smem_bytes(R));
      }))
    return e;
  const int max_wgs = 2 * compute_units();   // two workgroups of four waves per compute unit
  const int nwg = nitems < max_wgs ? nitems : max_wgs;
  hipLaunchKernelGGL((stage_fast_kernel<R, BATCH, PRE>), dim3((unsigned)nwg), dim3(256), fast_smem_bytes(R), s,
                     items_dev, nitems, *single, tiles_per_item);
  return (int)hipGetLastError();
}

template <int R>
static int launch_r(const StageProb* probs_dev, const WorkItem* items_dev, int nitems, int tiles_per_item,
                    const StageProb* single, bool pre, hipStream_t s) {
  if (probs_dev) {
    if (pre) return launch_rbp<R, true, true>(items_dev, nitems, tiles_per_item, single, s);
    return launch_rbp<R, true, false>(items_dev, nitems, tiles_per_item, single, s);
  }
  if (pre) return launch_rbp<R, false, true>(items_dev, nitems, tiles_per_item, single, s);
  return launch_rbp<R, false, false>(items_dev, nitems, tiles_per_item, single, s);
}

// ---- scale-in kernel: one workgroup per (problem, token, chunk) -------------------------------------
__global__ __launch_bounds__(256) void scale_in_kernel(const StageProb* __restrict__ probs, StageProb single) {
  StageProb p;
  if (probs) p = probs[blockIdx.y];
  else p = single;
  const int nch = (p.KB + CB - 1) / CB;
  const int unit = blockIdx.x;
  if (unit >= nch * p.T) return;
  const int b = unit / nch, c = unit - b * nch;
  const int tid = threadIdx.x;
  const int ch = tid & 1, oo = tid >> 1;
  const int st_q = oo >> 4, st_f = (oo & 15) >> 2, st_kg = oo & 3;
  const int st_col = st_q * kBlockCols + st_f * 32 + st_kg * 8;
  const int st_vec = (st_q * 4 + st_f) * 64 + st_kg * 16 + ch * 8;
  const int st_sw = (st_kg + 4 * (st_f & 1)) & 7;
  const void* vin_row = (const char*)p.vin + (size_t)b * (size_t)p.vin_ld * (size_t)dtype_size(p.vin_dt);
  StageRegs sr;
  stage_load(p.Ein, ch, vin_row, p.vin_dt, c * (CB * kBlockCols) + st_col, p.K, sr);
  // the chunk's largest magnitude goes to [2^12, 2^13): the smallest position factor (1/8) still leaves
  // three decades of normal fp16 numbers below it, the largest stays a factor 8 under fp16's overflow
  __shared__ float wmax[4];
  float m = stage_absmax(sr, p.vin_dt);
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
  if ((tid & 63) == 0) wmax[tid >> 6] = m;
  __syncthreads();
  m = fmaxf(fmaxf(wmax[0], wmax[1]), fmaxf(wmax[2], wmax[3]));
  int e = 0;
  if (m > 0.f && m < 3.0e38f) {
    int ex;
    (void)frexpf(m, &ex);                     // m = fr * 2^ex, fr in [0.5, 1)
    e = min(max(13 - ex, -100), 100);
  }
  u32x4* dst = (u32x4*)p.xs + ((size_t)b * nch + c) * (size_t)kChunkVecs + st_vec;
  stage_store(sr, p.vin_dt, dst, st_sw, pow2i(e));
  if (tid == 0) ((MDBF_GLOBAL int*)((u32x4*)p.xs + (size_t)p.T * nch * (size_t)kChunkVecs))[(size_t)b * nch + c] = e;
}

int launch_scale_in(const StageProb* probs_dev, int count, int max_units, const StageProb* single, hipStream_t s) {
  hipLaunchKernelGGL(scale_in_kernel, dim3((unsigned)max_units, (unsigned)count), dim3(256), 0, s, probs_dev, *single);
  return (int)hipGetLastError();
}

size_t xs_bytes_for(int K, int T) {
  const int nch = (num_blocks(K) + CB - 1) / CB;
  // the staged chunks of every token, then one exponent per (token, chunk)
  return (size_t)T * (size_t)nch * (size_t)kChunkVecs * 16u + (((size_t)T * (size_t)nch * 4u + 15u) & ~(size_t)15u);
}

bool stage_is_fast(const StageProb& p) {
  if (p.l != 16 || p.env_dt != MDBF_F16 || (p.K & 7) != 0 || p.KB < kPrefetchBlocks) return false;
  const int64_t row_bytes = p.vin_ld * (int64_t)dtype_size(p.vin_dt);
  return (row_bytes & 15) == 0;
}

int mfma_tiles_per_item(long total_tiles) {
  // aim at >= 2 workgroups per compute unit (256 CUs) before growing the per-wave tile count
  long want = total_tiles / 512;
  int tpi = 4;
  while (tpi < 16 && tpi < want) tpi *= 2;
  return tpi;
}

int launch_stage_mfma(const StageProb* probs_dev, const WorkItem* items_dev, int nitems, int tiles_per_item,
                      const StageProb* single, bool pre, hipStream_t s) {
  if (!probs_dev) nitems = (single->ntiles + tiles_per_item - 1) / tiles_per_item;
  switch (tiles_per_item) {
    case 4: return launch_r<1>(probs_dev, items_dev, nitems, tiles_per_item, single, pre, s);
    case 8: return launch_r<2>(probs_dev, items_dev, nitems, tiles_per_item, single, pre, s);
    case 16: return launch_r<4>(probs_dev, items_dev, nitems, tiles_per_item, single, pre, s);
    default: return (int)hipErrorInvalidValue;
  }
}

}  // namespace mdbf
