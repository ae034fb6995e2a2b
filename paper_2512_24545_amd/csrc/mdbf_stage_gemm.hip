// Many-token evaluation of one envelope-scaled binary product on gfx950, in reconstruct order.
//
//   out[b, r] = sum_j W[r, j] * vin[b, j],     W[r, j] = S[r, j] * E[r, j],     E = Eout * Ein^T  (rank l)
//
// The same product as the other stage kernels (paper Eq. "me-dbf-basis": the factor is the sign matrix
// modulated by a rank-l envelope), but evaluated as a dense GEMM against the reconstructed factor instead
// of l scaled binary products: (l + T) multiply-adds per sign entry instead of l * T.  Nothing dense ever
// reaches memory: a wave rebuilds its 16 x 128 piece of E with eight small matrix-core products
// (contraction over the l modes), flips signs with the packed bits, rounds to fp16 and holds the piece in
// registers as the B operand of the token product; the activations go through LDS, shared by the waves.
//
//  * workgroup: 4 waves; wave w owns R row tiles (16 rows each); the workgroup owns 16 * TB tokens
//  * per 128-column block: E piece per tile = 2 x v_mfma_f32_16x16x16_f16 per 32 columns.  The products'
//    row index is chosen so that lane (r, g) receives columns 32f + 8g + 0..7 of row r: exactly the columns
//    whose signs sit in the lane's packed word, and exactly the B-operand slot of v_mfma_f32_16x16x32_f16
//    for contraction step f.  No cross-lane movement between reconstruction and use.
//  * token product: for every 16-token slab, 4 contraction steps; A operand = 8 consecutive fp16 activations
//    read from LDS (rows swizzled by 16-byte chunks against bank conflicts)
// Arithmetic: envelopes and activations rounded to fp16 on load, E accumulated in fp32 and rounded to fp16
// once, token product accumulated in fp32.  Values beyond the fp16 range overflow.
#include "mdbf_internal.h"

namespace mdbf {
namespace gemm {

typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kWaves = 4;
constexpr int kDies = 8;                    // accelerator dies (XCDs); workgroup i is placed on die i mod 8
constexpr int kEinBufBytes = 128 * 32;      // 128 columns x 16 modes fp16
// LDS of a workgroup with TB slabs of 16 tokens: two buffers of (16 TB tokens x 128 columns fp16) + envelope rows
__host__ __device__ constexpr int vin_buf_bytes(int TB) { return 16 * TB * 256; }
__host__ __device__ constexpr int smem_bytes(int TB) { return 2 * (vin_buf_bytes(TB) + kEinBufBytes); }
// waves per SIMD the register budget is cut for: the small shapes live on occupancy (their blocks are short
// dependent chains), the big one on registers
__host__ __device__ constexpr int min_waves(int TB) { return TB >= 4 ? 2 : (TB == 2 ? 3 : 4); }

// Envelope rows of a block in LDS: 128 columns x 16 modes fp16 (32 bytes a column).  A reconstruction
// operand read touches columns 8a + b (+4), a, b = 0..3, eight bytes (four modes) per lane: in column order
// the four values of `a` would land on the same banks.  Column bits 2 and 3 trade places in the row index,
// and the 16-byte halves of a row trade places for columns with bit 4 set: the 32 lanes served together
// then cover every bank once.
__host__ __device__ constexpr int ein_row(int col) { return (col & ~12) | ((col & 4) << 1) | ((col & 8) >> 1); }

__device__ __forceinline__ uint32_t pack_half2(float lo, float hi) {
  half2v h;
  h.x = (_Float16)lo;
  h.y = (_Float16)hi;
  return __builtin_bit_cast(uint32_t, h);
}

// eight consecutive elements p[idx0 .. idx0+7] as fp16 pairs; elements at or past `nvalid` read as zero
__device__ __forceinline__ u32x4 load8_as_half(const void* p, int64_t idx0, int nvalid, int dt) {
  u32x4 out = {0u, 0u, 0u, 0u};
  if (nvalid <= 0) return out;
  const int es = dtype_size(dt);
  const uintptr_t addr = (uintptr_t)p + (uintptr_t)idx0 * (uintptr_t)es;
  if (nvalid >= 8 && (addr & 15u) == 0) {
    if (dt == MDBF_F16) return *(const MDBF_GLOBAL u32x4*)addr;
    if (dt == MDBF_BF16) {
      const u32x4 raw = *(const MDBF_GLOBAL u32x4*)addr;
      const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
      uint32_t o[4];
#pragma unroll
      for (int i = 0; i < 4; ++i)
        o[i] = pack_half2(__builtin_bit_cast(float, w[i] << 16), __builtin_bit_cast(float, w[i] & 0xFFFF0000u));
      return u32x4{o[0], o[1], o[2], o[3]};
    }
    const floatx4 a = *(const MDBF_GLOBAL floatx4*)addr;
    const floatx4 b = *(const MDBF_GLOBAL floatx4*)(addr + 16);
    return u32x4{pack_half2(a.x, a.y), pack_half2(a.z, a.w), pack_half2(b.x, b.y), pack_half2(b.z, b.w)};
  }
  float v[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) v[i] = (i < nvalid) ? load_as_float(p, idx0 + i, dt) : 0.f;
  return u32x4{pack_half2(v[0], v[1]), pack_half2(v[2], v[3]), pack_half2(v[4], v[5]), pack_half2(v[6], v[7])};
}

// eight consecutive elements of known type, 16-byte aligned, no bounds to respect; fp16 pairs
template <int DT>
__device__ __forceinline__ u32x4 load8_vec(const void* p, int64_t idx0) {
  if (DT == MDBF_F16) return ((const MDBF_GLOBAL u32x4*)((const _Float16*)p + idx0))[0];
  if (DT == MDBF_BF16) {
    const u32x4 raw = ((const MDBF_GLOBAL u32x4*)((const uint16_t*)p + idx0))[0];
    const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
    uint32_t o[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
      o[i] = pack_half2(__builtin_bit_cast(float, w[i] << 16), __builtin_bit_cast(float, w[i] & 0xFFFF0000u));
    return u32x4{o[0], o[1], o[2], o[3]};
  }
  const floatx4 a = ((const MDBF_GLOBAL floatx4*)((const float*)p + idx0))[0];
  const floatx4 b = ((const MDBF_GLOBAL floatx4*)((const float*)p + idx0))[1];
  return u32x4{pack_half2(a.x, a.y), pack_half2(a.z, a.w), pack_half2(b.x, b.y), pack_half2(b.z, b.w)};
}

// R row tiles per wave, TB slabs of 16 tokens per workgroup.  MODE 0..2: the common case -- fp16 envelopes of
// rank 16 or 8, activations of type MODE with 16-byte aligned rows and K a multiple of 8: every load is a full
// vector, issued without a branch (addresses are clamped, values past the end replaced by zero).  MODE 3:
// any types, ranks and alignments, element by element.
// BATCH: the rows come from a plan's work items instead of the single problem.
constexpr int kGeneric = 3;
constexpr int kPlanR = 2;   // row tiles per wave in a plan's work items
template <int R, int TB, int MODE, bool BATCH>
__global__ __launch_bounds__(64 * kWaves, min_waves(TB))
void stage_gemm_kernel(const WorkItem* __restrict__ items, StageProb single) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  // the rows of this workgroup: a work item of a plan (at most kWaves * R row tiles of one problem), or
  // the blockIdx.x-th run of kWaves * R tiles of the single problem
  StageProb p;
  int item_tile0, item_end, slab_group;
  if (BATCH) {
    const WorkItem& w = items[blockIdx.x];   // uniform address: scalar loads
    p = w.p;
    item_tile0 = w.tile0;
    item_end = w.tile0 + w.ntiles;
    slab_group = blockIdx.y;
  } else {
    // One-dimensional grid.  Workgroups go to the chip's eight dies in turn (id mod 8), each die with an L2
    // of its own; the (token slab group, row group) pairs, token-major, are dealt out in eight contiguous
    // runs, one per die: the workgroups that read the same activations share an L2.
    p = single;
    const int row_groups = (p.ntiles + kWaves * R - 1) / (kWaves * R);
    const int slab_groups = (p.T + 16 * TB - 1) / (16 * TB);
    const int total = row_groups * slab_groups;
    const int per_die = (total + kDies - 1) / kDies;
    const int unit = (blockIdx.x % kDies) * per_die + blockIdx.x / kDies;
    if (unit >= total) return;
    slab_group = unit / row_groups;
    item_tile0 = (unit - slab_group * row_groups) * (kWaves * R);
    item_end = min(item_tile0 + kWaves * R, p.ntiles);
  }
  unsigned char* vin_buf = smem;                               // [2][16*TB tokens][16 chunks of 16 B], swizzled
  constexpr int kVinBufBytes = vin_buf_bytes(TB);
  unsigned char* ein_buf = smem + 2 * kVinBufBytes;            // [2][128 columns][16 modes]
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int r16 = lane & 15, g = lane >> 4;
  const int tile0 = item_tile0 + wave * R;                     // first row tile of this wave
  const int tok0 = slab_group * (16 * TB);
  if (tok0 >= p.T) return;                                     // a plan's grid covers its longest problem
  const int KB = p.KB;

  // ---- per-unit operands: Eout rows of the wave's tiles (B operand of the reconstruction), 4 modes per lane
  half4 eo_op[R];
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int row = (tile0 + r) * kTileRows + r16;
    float v[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const int mode = 4 * g + t;
      v[t] = (row < p.rows && mode < p.l) ? load_as_float(p.Eout, (int64_t)row * p.l + mode, p.env_dt) : 0.f;
    }
    eo_op[r] = half4{(_Float16)v[0], (_Float16)v[1], (_Float16)v[2], (_Float16)v[3]};
  }
  // sign words: tiles past the end read the last tile (their rows are never stored)
  const MDBF_GLOBAL uint32_t* sbase[R];
  size_t sstride[R];
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int t = min(tile0 + r, item_end - 1);
    sbase[r] = (const MDBF_GLOBAL uint32_t*)p.S + tile_base_words(t, KB) + lane;
    sstride[r] = (size_t)group_tiles(t, p.ntiles) * 64u;
  }

  floatx4 acc[TB][R];
#pragma unroll
  for (int tb = 0; tb < TB; ++tb)
#pragma unroll
    for (int r = 0; r < R; ++r) acc[tb][r] = floatx4{0.f, 0.f, 0.f, 0.f};

  // ---- staging of one block.  Envelope rows and sign words go through registers.  fp16 activations
  //      (kDma) go from global memory straight into LDS, 16 bytes per lane and 1 KB (four token rows) per
  //      instruction; the row swizzle is applied on the global side (a lane fetches the chunk that belongs at
  //      its LDS slot).  Other types are converted in registers on the way.  Values past the end: tokens past
  //      T are never stored; columns past K meet zeroed envelope rows (kDma) or are zeroed themselves.
  constexpr bool kDma = (MODE == MDBF_F16);
  constexpr int kVinChunks = (16 * TB * 16) / (64 * kWaves);   // 16-byte chunks per thread: TB
  u32x4 vin_reg[kDma ? 1 : kVinChunks];
  u32x4 ein_reg;
  uint32_t sw_next[R];
  auto dma_block = [&](int q, int buf) {
#pragma unroll
    for (int i = 0; i < kVinChunks; ++i) {
      const int id = tid + 64 * kWaves * i;
      const int tok = id >> 4, c = (id & 15) ^ (tok & 15);
      const int col = min(q * kBlockCols + c * 8, p.K - 8);
      const int b = min(tok0 + tok, p.T - 1);
      const MDBF_GLOBAL _Float16* src = (const MDBF_GLOBAL _Float16*)p.vin + ((int64_t)b * p.vin_ld + col);
      unsigned char* dst = vin_buf + buf * kVinBufBytes + (wave * 64 + 64 * kWaves * i) * 16;   // wave-uniform
      __builtin_amdgcn_global_load_lds((const MDBF_GLOBAL void*)src, (MDBF_LDS void*)dst, 16, 0, 0);
    }
  };
  auto fetch_block = [&](int q) {
    if (!kDma) {
#pragma unroll
      for (int i = 0; i < kVinChunks; ++i) {
        const int id = tid + 64 * kWaves * i;
        const int tok = id >> 4, c = id & 15;
        const int col = q * kBlockCols + c * 8;
        const int b = tok0 + tok;
        if (MODE == kGeneric) {
          const int nvalid = (b < p.T) ? (p.K - col) : 0;
          vin_reg[i] = load8_as_half(p.vin, (int64_t)min(b, p.T - 1) * p.vin_ld + col, nvalid, p.vin_dt);
        } else {
          const u32x4 v = load8_vec<MODE>(p.vin, (int64_t)min(b, p.T - 1) * p.vin_ld + min(col, p.K - 8));
          const bool ok = (b < p.T) && (col < p.K);
          vin_reg[i] = u32x4{ok ? v.x : 0u, ok ? v.y : 0u, ok ? v.z : 0u, ok ? v.w : 0u};
        }
      }
    }
    if (MODE != kGeneric) {
      const int col = q * kBlockCols + (tid >> 1);
      // rank 8: a row is one 16-byte vector; the half that would hold modes 8..15 becomes zero
      const int hl = p.l >> 3;
      const bool has_modes = (tid & 1) < hl;
      const u32x4 v = ((const MDBF_GLOBAL u32x4*)p.Ein)[(size_t)min(col, p.K - 1) * hl + (has_modes ? (tid & 1) : 0)];
      const bool ok = (col < p.K) && has_modes;
      ein_reg = u32x4{ok ? v.x : 0u, ok ? v.y : 0u, ok ? v.z : 0u, ok ? v.w : 0u};
    } else {
      const int colr = tid >> 1, half = tid & 1;
      const int col = q * kBlockCols + colr;
      float v[8];
#pragma unroll
      for (int t = 0; t < 8; ++t) {
        const int mode = half * 8 + t;
        v[t] = (col < p.K && mode < p.l) ? load_as_float(p.Ein, (int64_t)col * p.l + mode, p.env_dt) : 0.f;
      }
      ein_reg = u32x4{pack_half2(v[0], v[1]), pack_half2(v[2], v[3]), pack_half2(v[4], v[5]), pack_half2(v[6], v[7])};
    }
#pragma unroll
    for (int r = 0; r < R; ++r) sw_next[r] = sbase[r][(size_t)min(q, KB - 1) * sstride[r]];
  };
  auto stash_block = [&](int buf) {
    if (!kDma) {
#pragma unroll
      for (int i = 0; i < kVinChunks; ++i) {
        const int id = tid + 64 * kWaves * i;
        const int tok = id >> 4, c = id & 15;
        *reinterpret_cast<u32x4*>(vin_buf + buf * kVinBufBytes + tok * 256 + ((c ^ (tok & 15)) << 4)) = vin_reg[i];
      }
    }
    *reinterpret_cast<u32x4*>(ein_buf + buf * kEinBufBytes + ein_row(tid >> 1) * 32 +
                              (((tid & 1) ^ ((tid >> 5) & 1)) << 4)) = ein_reg;
  };

  // Register staging runs two blocks ahead (a block is requested at the end of one iteration and parked at
  // the end of the next).  Direct staging runs one block ahead: block q + 1 is requested right after the
  // barrier that opens iteration q, into the buffer iteration q - 1 has just released, and every wave waits
  // for its own requests before it reaches the next barrier.
  uint32_t sw[R];
  if (kDma) dma_block(0, 0);
  fetch_block(0);
  stash_block(0);
#pragma unroll
  for (int r = 0; r < R; ++r) sw[r] = sw_next[r];
  if (kDma) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  else fetch_block(min(1, KB - 1));

#pragma unroll 1
  for (int q = 0; q < KB; ++q) {
    const int cur = q & 1;
    __syncthreads();
    if (kDma) {
      dma_block(min(q + 1, KB - 1), cur ^ 1);
      fetch_block(min(q + 1, KB - 1));
    }

    // ---- per contraction step f (32 columns): rebuild the wave's pieces of W, wop[r] = B operand of the
    //      token product, then run the step over all token slabs.  The steps are independent of each other,
    //      which lets the rebuild of one step overlap the matrix-core work of the previous one.
    const unsigned char* ein = ein_buf + cur * kEinBufBytes;
    const unsigned char* vin = vin_buf + cur * kVinBufBytes;
#pragma unroll
    for (int f = 0; f < 4; ++f) {
      // A operands of the two reconstruction products: rows mi -> columns 32f + 8(mi/4) + mi%4 (+4)
      const int col0 = 32 * f + 8 * (r16 >> 2) + (r16 & 3);
      const int eoff = ein_row(col0) * 32 + ((g ^ ((r16 >> 2) & 2)) << 3);
      const half4 ea0 = *reinterpret_cast<const half4*>(ein + eoff);
      const half4 ea1 = *reinterpret_cast<const half4*>(ein + eoff + (ein_row(4) - ein_row(0)) * 32);
      half8 wop[R];
#pragma unroll
      for (int r = 0; r < R; ++r) {
        const floatx4 z4 = {0.f, 0.f, 0.f, 0.f};
        const floatx4 e0 = __builtin_amdgcn_mfma_f32_16x16x16f16(ea0, eo_op[r], z4, 0, 0, 0);
        const floatx4 e1 = __builtin_amdgcn_mfma_f32_16x16x16f16(ea1, eo_op[r], z4, 0, 0, 0);
        // lane (r16, g) now holds E[row r16][32f + 8g + e], e = 0..3 in e0 and 4..7 in e1.  The packed word
        // keeps the signs of columns e = 2i and 2i+1 at bits p and p + 16, p = 8(f/2) + 4(f%2) + i.
        const int pbase = 8 * (f >> 1) + 4 * (f & 1);
        uint32_t w4[4];
        w4[0] = pack_half2(e0[0], e0[1]) ^ ((sw[r] << (15 - (pbase + 0))) & 0x80008000u);
        w4[1] = pack_half2(e0[2], e0[3]) ^ ((sw[r] << (15 - (pbase + 1))) & 0x80008000u);
        w4[2] = pack_half2(e1[0], e1[1]) ^ ((sw[r] << (15 - (pbase + 2))) & 0x80008000u);
        w4[3] = pack_half2(e1[2], e1[3]) ^ ((sw[r] << (15 - (pbase + 3))) & 0x80008000u);
        wop[r] = __builtin_bit_cast(half8, u32x4{w4[0], w4[1], w4[2], w4[3]});
      }
      // the step's A operands (one per token slab) are all requested before the first product
      const int c = f * 4 + g;
      half8 a[TB];
#pragma unroll
      for (int tb = 0; tb < TB; ++tb) {
        const int tok = tb * 16 + r16;
        a[tb] = *reinterpret_cast<const half8*>(vin + tok * 256 + ((c ^ (tok & 15)) << 4));
      }
#pragma unroll
      for (int tb = 0; tb < TB; ++tb)
#pragma unroll
        for (int r = 0; r < R; ++r)
          acc[tb][r] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[tb], wop[r], acc[tb][r], 0, 0, 0);
    }

    // park the next block's register-staged parts and (register staging) request the one after
    // (past the end the last block is requested again: no branch around the loads)
    stash_block(cur ^ 1);
#pragma unroll
    for (int r = 0; r < R; ++r) sw[r] = sw_next[r];
    if (kDma) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    else fetch_block(min(q + 2, KB - 1));
  }

  // ---- store: lane (r16, g) holds out[token 16 tb + 4g + i][row r16 of tile r]
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int row = (tile0 + r) * kTileRows + r16;
    if (tile0 + r < item_end && row < p.rows) {
#pragma unroll
      for (int tb = 0; tb < TB; ++tb)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int b = tok0 + tb * 16 + 4 * g + i;
          if (b < p.T) emit_result(p.out, (int64_t)b * p.out_ld + row, p.out_dt, acc[tb][r][i], p.flags);
        }
    }
  }
}

// ---------------------------------------------------------------------------------------------------
// One short problem by itself (at most 16 tokens, the vector-load modes): the launch above would give each
// wave one row tile and the whole contraction dimension, a chain of KB dependent steps on a quarter of the
// device.  Here a workgroup owns ONE row tile and its four waves split the column blocks (wave w takes blocks
// 4 i + w); an iteration stages four blocks, two iterations ahead; the four partial results meet in LDS and
// are added in wave order (the same order every time).
// ---------------------------------------------------------------------------------------------------
constexpr int kSplitVinBytes = kWaves * 16 * 256;     // four blocks x 16 tokens x 128 columns fp16
constexpr int kSplitEinBytes = kWaves * kEinBufBytes;
constexpr int kSplitSmem = 2 * (kSplitVinBytes + kSplitEinBytes);

template <int MODE, int R>
__global__ __launch_bounds__(64 * kWaves, 2)
void stage_gemm_split_kernel(StageProb p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  unsigned char* vin_buf = smem;                               // [2][4 blocks][16 tokens][16 chunks], swizzled
  unsigned char* ein_buf = smem + 2 * kSplitVinBytes;          // [2][4 blocks][128 columns][16 modes]
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int r16 = lane & 15, g = lane >> 4;
  const int tile0 = blockIdx.x * R;                            // this workgroup's R consecutive row tiles
  const int KB = p.KB;
  const int iters = (KB + kWaves - 1) / kWaves;

  // Eout row of this lane's tile row, 4 modes per lane (B operand of the reconstruction)
  half4 eo_op[R];
  const MDBF_GLOBAL uint32_t* sbase[R];
  size_t sstride[R];
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int row = (tile0 + r) * kTileRows + r16;
    float v[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const int mode = 4 * g + t;
      v[t] = (row < p.rows && mode < p.l) ? load_as_float(p.Eout, (int64_t)row * p.l + mode, p.env_dt) : 0.f;
    }
    eo_op[r] = half4{(_Float16)v[0], (_Float16)v[1], (_Float16)v[2], (_Float16)v[3]};
    const int t = min(tile0 + r, p.ntiles - 1);               // a tile past the end repeats the last (never stored)
    sbase[r] = (const MDBF_GLOBAL uint32_t*)p.S + tile_base_words(t, KB) + lane;
    sstride[r] = (size_t)group_tiles(t, p.ntiles) * 64u;
  }

  // staging of the four blocks of iteration `it`: thread -> (token, chunk) of every block, and (column, half)
  // of every block's envelope rows.  Columns past K (also whole blocks past KB) get zero envelope rows and
  // zero activations; tokens past T are never stored.
  // (values past the end are replaced by zero when a block is parked, not when it is requested: a select
  // right after the load would make the wave wait for the load there)
  u32x4 vin_reg[kWaves], ein_reg[kWaves];
  uint32_t live = 0;                 // bits j: activations of block j hold real data; bits 8 + j: envelope rows
  uint32_t sw_next[R];
  const int st_tok = tid >> 4, st_c = tid & 15;
  const int hl = p.l >> 3;
  const bool has_modes = (tid & 1) < hl;
  auto fetch = [&](int it) {
    uint32_t lv = 0;
#pragma unroll
    for (int j = 0; j < kWaves; ++j) {
      const int q = it * kWaves + j;
      const int col = q * kBlockCols + st_c * 8;
      vin_reg[j] = load8_vec<MODE>(p.vin, (int64_t)min(st_tok, p.T - 1) * p.vin_ld + min(col, p.K - 8));
      lv |= ((st_tok < p.T) && (col < p.K)) ? (1u << j) : 0u;
      const int ecol = q * kBlockCols + (tid >> 1);
      ein_reg[j] = ((const MDBF_GLOBAL u32x4*)p.Ein)[(size_t)min(ecol, p.K - 1) * hl + (has_modes ? (tid & 1) : 0)];
      lv |= ((ecol < p.K) && has_modes) ? (256u << j) : 0u;
    }
    live = lv;
#pragma unroll
    for (int r = 0; r < R; ++r) sw_next[r] = sbase[r][(size_t)min(it * kWaves + wave, KB - 1) * sstride[r]];
  };
  auto stash = [&](int buf) {
    const u32x4 zero = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int j = 0; j < kWaves; ++j) {
      *reinterpret_cast<u32x4*>(vin_buf + buf * kSplitVinBytes + j * (16 * 256) + st_tok * 256 +
                                ((st_c ^ (st_tok & 15)) << 4)) = ((live >> j) & 1u) ? vin_reg[j] : zero;
      *reinterpret_cast<u32x4*>(ein_buf + buf * kSplitEinBytes + j * kEinBufBytes + ein_row(tid >> 1) * 32 +
                                (((tid & 1) ^ ((tid >> 5) & 1)) << 4)) = ((live >> (8 + j)) & 1u) ? ein_reg[j] : zero;
    }
  };

  fetch(0);
  stash(0);
  uint32_t sw[R];
  floatx4 acc[R];
#pragma unroll
  for (int r = 0; r < R; ++r) {
    sw[r] = sw_next[r];
    acc[r] = floatx4{0.f, 0.f, 0.f, 0.f};
  }
  fetch(min(1, iters - 1));

#pragma unroll 1
  for (int it = 0; it < iters; ++it) {
    const int cur = it & 1;
    __syncthreads();
    const unsigned char* ein = ein_buf + cur * kSplitEinBytes + wave * kEinBufBytes;
    const unsigned char* vin = vin_buf + cur * kSplitVinBytes + wave * (16 * 256);
#pragma unroll
    for (int f = 0; f < 4; ++f) {
      const int col0 = 32 * f + 8 * (r16 >> 2) + (r16 & 3);
      const int eoff = ein_row(col0) * 32 + ((g ^ ((r16 >> 2) & 2)) << 3);
      const half4 ea0 = *reinterpret_cast<const half4*>(ein + eoff);
      const half4 ea1 = *reinterpret_cast<const half4*>(ein + eoff + (ein_row(4) - ein_row(0)) * 32);
      const int c = f * 4 + g;
      const half8 a = *reinterpret_cast<const half8*>(vin + r16 * 256 + ((c ^ r16) << 4));
      const int pbase = 8 * (f >> 1) + 4 * (f & 1);
#pragma unroll
      for (int r = 0; r < R; ++r) {
        const floatx4 z4 = {0.f, 0.f, 0.f, 0.f};
        const floatx4 e0 = __builtin_amdgcn_mfma_f32_16x16x16f16(ea0, eo_op[r], z4, 0, 0, 0);
        const floatx4 e1 = __builtin_amdgcn_mfma_f32_16x16x16f16(ea1, eo_op[r], z4, 0, 0, 0);
        uint32_t w4[4];
        w4[0] = pack_half2(e0[0], e0[1]) ^ ((sw[r] << (15 - (pbase + 0))) & 0x80008000u);
        w4[1] = pack_half2(e0[2], e0[3]) ^ ((sw[r] << (15 - (pbase + 1))) & 0x80008000u);
        w4[2] = pack_half2(e1[0], e1[1]) ^ ((sw[r] << (15 - (pbase + 2))) & 0x80008000u);
        w4[3] = pack_half2(e1[2], e1[3]) ^ ((sw[r] << (15 - (pbase + 3))) & 0x80008000u);
        const half8 wop = __builtin_bit_cast(half8, u32x4{w4[0], w4[1], w4[2], w4[3]});
        acc[r] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, wop, acc[r], 0, 0, 0);
      }
    }
    stash(cur ^ 1);
#pragma unroll
    for (int r = 0; r < R; ++r) sw[r] = sw_next[r];
    fetch(min(it + 2, iters - 1));
  }

  // ---- the four partial results: through LDS, added in wave order by wave 0
  __syncthreads();                                             // every wave is done with the staging buffers
  floatx4* red = reinterpret_cast<floatx4*>(smem);              // [R][4 waves][64 lanes]
#pragma unroll
  for (int r = 0; r < R; ++r) red[(r * kWaves + wave) * 64 + lane] = acc[r];
  __syncthreads();
  if (wave < R) {                                              // wave r adds up and stores tile r
    floatx4 sum = red[(wave * kWaves) * 64 + lane];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) {
      const floatx4 t = red[(wave * kWaves + w) * 64 + lane];
      sum[0] += t[0]; sum[1] += t[1]; sum[2] += t[2]; sum[3] += t[3];
    }
    const int row = (tile0 + wave) * kTileRows + r16;
    if (tile0 + wave < p.ntiles && row < p.rows) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int b = 4 * g + i;
        if (b < p.T) emit_result(p.out, (int64_t)b * p.out_ld + row, p.out_dt, sum[i], p.flags);
      }
    }
  }
}

// R row tiles per workgroup (wave r stores tile r): more tiles mean fewer re-reads of the envelope rows and
// activations (every workgroup reads all of them) but longer chains and fewer workgroups.
template <int MODE, int R>
static int launch_split_r(const StageProb* p, hipStream_t s) {
  static_assert(R >= 1 && R <= kWaves, "wave r stores tile r");
  static KernelSetup setup;
  if (int e = kernel_setup(setup, [] {
        return hipFuncSetAttribute(reinterpret_cast<const void*>(&stage_gemm_split_kernel<MODE, R>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, kSplitSmem);
      }))
    return e;
  hipLaunchKernelGGL((stage_gemm_split_kernel<MODE, R>), dim3((unsigned)((p->ntiles + R - 1) / R)),
                     dim3(64 * kWaves), kSplitSmem, s, *p);
  return (int)hipGetLastError();
}

// one tile per workgroup as long as the device holds all workgroups at once (two per compute unit)
template <int MODE>
static int launch_split(const StageProb* p, hipStream_t s) {
  if (p->ntiles > 2 * compute_units()) return launch_split_r<MODE, 2>(p, s);
  return launch_split_r<MODE, 1>(p, s);
}

// items_dev null: the single problem *p.  Else nitems work items of a plan, `p` describing the launch:
// p->T = the longest token count among the problems.
template <int R, int TB, int MODE, bool BATCH>
static int launch_rtmb(const WorkItem* items_dev, int nitems, const StageProb* p, hipStream_t s) {
  static KernelSetup setup;
  if (int e = kernel_setup(setup, [] {
        return hipFuncSetAttribute(reinterpret_cast<const void*>(&stage_gemm_kernel<R, TB, MODE, BATCH>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, smem_bytes(TB));
      }))
    return e;
  const int rows_per_wg = kWaves * R;   // tiles
  unsigned gx = BATCH ? (unsigned)nitems : (unsigned)((p->ntiles + rows_per_wg - 1) / rows_per_wg);
  unsigned gy = (unsigned)((p->T + 16 * TB - 1) / (16 * TB));
  if (!BATCH) {
    const unsigned total = gx * gy;
    gx = kDies * ((total + kDies - 1) / kDies);
    gy = 1;
  }
  hipLaunchKernelGGL((stage_gemm_kernel<R, TB, MODE, BATCH>), dim3(gx, gy), dim3(64 * kWaves), smem_bytes(TB), s,
                     items_dev, *p);
  return (int)hipGetLastError();
}

template <int R, int TB, int MODE>
static int launch_rtm(const WorkItem* items_dev, int nitems, const StageProb* p, hipStream_t s) {
  if (items_dev) {
    // plans: items of kPlanR tiles per wave, short token slabs
    if constexpr (R == kPlanR && TB <= 4) return launch_rtmb<R, TB, MODE, true>(items_dev, nitems, p, s);
    return (int)hipErrorInvalidValue;
  } else {
    if constexpr (R == 1 || TB >= 6) return launch_rtmb<R, TB, MODE, false>(nullptr, 0, p, s);
    return (int)hipErrorInvalidValue;
  }
}

template <int R, int TB>
static int launch_rt(const WorkItem* items_dev, int nitems, int mode, const StageProb* p, hipStream_t s) {
  if (mode == kGeneric) return launch_rtm<R, TB, kGeneric>(items_dev, nitems, p, s);
  if (mode == MDBF_F16) return launch_rtm<R, TB, MDBF_F16>(items_dev, nitems, p, s);
  if (mode == MDBF_BF16) return launch_rtm<R, TB, MDBF_BF16>(items_dev, nitems, p, s);
  return launch_rtm<R, TB, MDBF_F32>(items_dev, nitems, p, s);
}

}  // namespace gemm

// Token slabs per workgroup for a long single problem (two row tiles per wave).  A workgroup's cost per
// column block is a fixed part (rebuilding its piece of the factor) plus a part per slab; the launch takes as
// long as the busiest compute unit, which holds ceil(workgroups / units) of them.  Fewer slabs per workgroup
// make more, lighter workgroups: worth it when that evens out the last round (166 row tiles x 2048 tokens:
// 336 workgroups of 8 slabs leave most units with one workgroup and some with two; 462 of 6 slabs fill them).
static int long_problem_slabs(const StageProb& p) {
  const int cus = compute_units();
  const int row_groups = (p.ntiles + 2 * gemm::kWaves - 1) / (2 * gemm::kWaves);
  int best = 8;
  double best_cost = 0.0;
  for (int tb = 8; tb >= 6; --tb) {
    const int64_t wgs = (int64_t)row_groups * ((p.T + 16 * tb - 1) / (16 * tb));
    const double cost = (double)((wgs + cus - 1) / cus) * (4.8 + tb);   // fixed part ~ 4.8 slabs' worth
    if (tb == 8 || cost < best_cost) { best = tb; best_cost = cost; }
  }
  return best;
}
bool stage_is_gemm(const StageProb& p) { return p.l >= 1 && p.l <= 16; }

int gemm_load_mode(const StageProb& p) {
  const int es = dtype_size(p.vin_dt);
  const bool fast = p.env_dt == MDBF_F16 && (p.l == 16 || p.l == 8) && (p.K & 7) == 0 && p.K >= 8 &&
                    (((uintptr_t)p.vin | (uintptr_t)p.Ein) & 15u) == 0 && ((p.vin_ld * es) & 15) == 0;
  return fast ? p.vin_dt : gemm::kGeneric;
}

int gemm_tiles_per_item() { return gemm::kWaves * gemm::kPlanR; }
int gemm_plan_max_tokens() { return 64; }   // plans with longer problems launch the single-problem kernel per problem

int launch_stage_gemm(const WorkItem* items_dev, int nitems, int mode, const StageProb* p, hipStream_t s) {
  if (items_dev) {
    if (p->T > 32) return gemm::launch_rt<gemm::kPlanR, 4>(items_dev, nitems, mode, p, s);
    if (p->T > 16) return gemm::launch_rt<gemm::kPlanR, 2>(items_dev, nitems, mode, p, s);
    return gemm::launch_rt<gemm::kPlanR, 1>(items_dev, nitems, mode, p, s);
  }
  mode = gemm_load_mode(*p);
  if (p->T > 64) {
    switch (long_problem_slabs(*p)) {
      case 6: return gemm::launch_rt<2, 6>(nullptr, 0, mode, p, s);
      case 7: return gemm::launch_rt<2, 7>(nullptr, 0, mode, p, s);
      default: return gemm::launch_rt<2, 8>(nullptr, 0, mode, p, s);
    }
  }
  if (p->T > 32) return gemm::launch_rt<1, 4>(nullptr, 0, mode, p, s);
  if (p->T > 16) return gemm::launch_rt<1, 2>(nullptr, 0, mode, p, s);
  if (mode == MDBF_F16) return gemm::launch_split<MDBF_F16>(p, s);
  if (mode == MDBF_BF16) return gemm::launch_split<MDBF_BF16>(p, s);
  if (mode == MDBF_F32) return gemm::launch_split<MDBF_F32>(p, s);
  return gemm::launch_rt<1, 1>(nullptr, 0, mode, p, s);
}

}  // namespace mdbf
