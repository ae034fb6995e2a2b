// Matrix-core evaluation of one envelope-scaled binary product on gfx950: the FAST variant
// (l == 16, fp16 envelopes, K a multiple of 8, 16-byte aligned activation rows).
//
//   out[r] = sum_c Eout[r,c] * P[r,c],     P[r,c] = sum_j S[r,j] * xs[j,c],   xs[j,c] = fp16(Ein[j,c] * vin[j])
//
// (paper Eq. "me-dbf-expand": per factor, l envelope-scaled copies of the shared sign basis).
// P is a skinny GEMM (rows x K) . (K x 16): exactly one 16x16x32 fp16 MFMA tile wide.
//
// Work decomposition: a workgroup of four wavefronts owns up to 4*R row tiles (16 rows each) of
// one problem and the whole contraction; wave w owns tiles w, w+4, ...  The scaled activations xs
// are staged chunk by chunk (1024 columns) in LDS in the order the MFMA B operand wants them and
// shared by all tiles of the workgroup; sign words stream from HBM with 128-bit loads, one group
// (512 columns) ahead of their use; the envelope rows of the next chunk are in flight while the
// current chunk is contracted.
//
// Sign expansion without shifts: with bit t=1 meaning -1,  S = 1 - 2t, hence
//      P[r,c] = colsum[c] - 2 * sum_j t[r,j] xs[j,c].
// The A operand of an MFMA step is  w & mask : the two selected bits of a word, read as two fp16
// values, are 0 or 2^(p-24) (p = bit position 0..7; fp16 denormals are honoured by the MFMA).  The
// staged activation of the entry at position p = 4c+i carries the factor 2^-i, so every product of
// class c (positions 4c..4c+3) is scaled by 2^(4c-24) exactly, and each class has its own fp32
// accumulator.  Bits 8..15 of each half word are brought down with one shift per word.
// colsum comes from the same MFMAs applied to a virtual row whose bits are all 1, so that it sees
// exactly the staged (rounded) values; the four waves share that work block by block.
#include "mdbf_internal.h"

namespace mdbf {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

#define MDBF_GLOBAL __attribute__((address_space(1)))
typedef const MDBF_GLOBAL u32x4* g_u32x4_ptr;
typedef const MDBF_GLOBAL uint32_t* g_u32_ptr;
typedef const MDBF_GLOBAL floatx4* g_f32x4_ptr;
typedef const MDBF_GLOBAL _Float16* g_f16_ptr;
typedef const MDBF_GLOBAL uint16_t* g_u16_ptr;
typedef const MDBF_GLOBAL float* g_f32_ptr;

#ifdef MDBF_DBG_TIMING
__device__ unsigned long long g_dbg_time[64 * 64];   // [block < 64][slot]
#define DBG_T(slot) do { if (blockIdx.x < 64 && (threadIdx.x & 63) == 0 && (threadIdx.x >> 6) == 1) \
    g_dbg_time[blockIdx.x * 64 + (slot)] = __builtin_readcyclecounter(); } while (0)
#else
#define DBG_T(slot) do {} while (0)
#endif

constexpr int CB = 8;                      // 128-column blocks per LDS chunk
constexpr int kChunkVecs = CB * 4 * 64;    // 16-byte vectors per chunk buffer (32 KB)
constexpr int kFastSmemBytes = 2 * kChunkVecs * 16 + 4 * 16 * 4;

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
  u32x4 e[8];   // 8 envelope rows of one column octet, 8 fp16 modes each
  float x[8];   // the octet's 8 activations, already multiplied by 2^-(e/2)
};

// Thread (oo = tid/2, ch = tid%2) stages the octet of columns `kcol..kcol+7` for modes 8ch..8ch+7.
// Octets at or beyond K read the (valid) first octet instead and get zero activations: no branch.
__device__ __forceinline__ void stage_load(g_u32x4_ptr ein_thr, const void* vin_row, int vin_dt, int kcol, int K,
                                           StageRegs& sr) {
  const bool valid = kcol < K;
  const int kc = valid ? kcol : 0;
  g_u32x4_ptr ep = ein_thr + (size_t)kc * 2;
#pragma unroll
  for (int e = 0; e < 8; ++e) sr.e[e] = ep[2 * e];
  if (vin_dt == MDBF_F32) {
    g_f32x4_ptr xp = (g_f32x4_ptr)((g_f32_ptr)vin_row + kc);
    const floatx4 x0 = xp[0], x1 = xp[1];
    sr.x[0] = x0.x; sr.x[1] = x0.y; sr.x[2] = x0.z * 0.5f; sr.x[3] = x0.w * 0.5f;
    sr.x[4] = x1.x * 0.25f; sr.x[5] = x1.y * 0.25f; sr.x[6] = x1.z * 0.125f; sr.x[7] = x1.w * 0.125f;
  } else if (vin_dt == MDBF_F16) {
    const u32x4 xb = *(g_u32x4_ptr)((g_f16_ptr)vin_row + kc);
    const half8 xh = __builtin_bit_cast(half8, xb);
#pragma unroll
    for (int e = 0; e < 8; ++e) sr.x[e] = (float)xh[e] * (1.0f / (float)(1 << (e >> 1)));
  } else {
    const u32x4 xb = *(g_u32x4_ptr)((g_u16_ptr)vin_row + kc);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const uint32_t wd = xb[e >> 1];
      const uint32_t bits = (e & 1) ? (wd & 0xFFFF0000u) : (wd << 16);
      sr.x[e] = __builtin_bit_cast(float, bits) * (1.0f / (float)(1 << (e >> 1)));
    }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) sr.x[e] = valid ? sr.x[e] : 0.f;
}

// dst: the thread's 8 consecutive 16-byte slots (modes 8ch..8ch+7 of its octet); slot cc is stored at
// cc ^ sw so that the 64 lanes of one store instruction spread over all LDS banks.
__device__ __forceinline__ void stage_store(const StageRegs& sr, u32x4* dst, int sw) {
#pragma unroll
  for (int cc = 0; cc < 8; ++cc) {
    u32x4 v;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const u32x4 r0 = sr.e[2 * i], r1 = sr.e[2 * i + 1];
      const uint32_t a0 = r0[cc >> 1], a1 = r1[cc >> 1];
      const uint32_t pr = (cc & 1) ? mix_pair_hi(a0, a1, sr.x[2 * i], sr.x[2 * i + 1])
                                   : mix_pair_lo(a0, a1, sr.x[2 * i], sr.x[2 * i + 1]);
      v[i] = pr;
    }
    dst[cc ^ sw] = v;
  }
}

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

template <int R>
__device__ __forceinline__ void run_item(const StageProb& p, const int tile0, const int ntl, u32x4* buf, float* red) {
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform, and known to be
  const int KB = p.KB, NG = KB >> 2, TB = KB & 3;
  const int nchunks = (KB + CB - 1) / CB;

  // Tiles of this wave: tile0 + wave + 4*r.  Tiles past the end of the item are replaced by the
  // item's last tile (their results are not stored), which keeps the contraction loop branch-free.
  int trel[R];
#pragma unroll
  for (int r = 0; r < R; ++r) trel[r] = min(wave + 4 * r, ntl - 1);
  g_u32x4_ptr sp[R];
  g_u32_ptr stail[R];
#pragma unroll
  for (int r = 0; r < R; ++r) {
    sp[r] = (g_u32x4_ptr)p.S + (size_t)(tile0 + trel[r]) * (size_t)(KB * 16) + lane;
    stail[r] = (g_u32_ptr)p.S + (size_t)(tile0 + trel[r]) * (size_t)(KB * 64) + (size_t)NG * 256 + lane;
  }

  // staging role of this thread
  const int ch = tid & 1, oo = tid >> 1;
  const int st_q = oo >> 4, st_f = (oo & 15) >> 2, st_kg = oo & 3;
  const int st_col = st_q * kBlockCols + st_f * 32 + st_kg * 8;            // column inside a chunk
  const int st_vec = (st_q * 4 + st_f) * 64 + st_kg * 16 + ch * 8;         // first of its 8 LDS slots
  const int st_sw = (st_kg + 4 * (st_f & 1)) & 7;
  g_u32x4_ptr ein_thr = (g_u32x4_ptr)p.Ein + ch;

  // B-operand read slots of this lane (same swizzle as the stores)
  const int kg = lane >> 4, n = lane & 15;
  const int rd_even = kg * 16 + ((n & 8) | ((n & 7) ^ (kg & 7)));
  const int rd_odd = kg * 16 + ((n & 8) | ((n & 7) ^ ((kg + 4) & 7)));
  // the virtual all-ones row: wave w contracts MFMA step f == w of every block (class w & 1)
  const int rd_virt = wave * 64 + ((wave & 1) ? rd_odd : rd_even);
  const half8 avirt = (wave & 1) ? expand(0xFFFFFFFFu, 1) : expand(0xFFFFFFFFu, 0);
  const float virt_scale = (wave & 1) ? 1048576.f : 16777216.f;  // 2^20 : 2^24

  for (int b = 0; b < p.T; ++b) {
    const void* vin_row = (const char*)p.vin + (size_t)b * (size_t)p.vin_ld * (size_t)dtype_size(p.vin_dt);
    floatx4 acc[R][2];
    floatx4 accv = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int r = 0; r < R; ++r) {
      acc[r][0] = floatx4{0.f, 0.f, 0.f, 0.f};
      acc[r][1] = floatx4{0.f, 0.f, 0.f, 0.f};
    }

    u32x4 wn[R];
#pragma unroll
    for (int r = 0; r < R; ++r) wn[r] = u32x4{0u, 0u, 0u, 0u};
    if (NG > 0) {
#pragma unroll
      for (int r = 0; r < R; ++r) wn[r] = sp[r][0];
    }

    StageRegs sr;
    DBG_T(0);
    stage_load(ein_thr, vin_row, p.vin_dt, st_col, p.K, sr);
    stage_store(sr, buf + st_vec, st_sw);
    DBG_T(1);
    __syncthreads();
    DBG_T(2);

#pragma unroll 1
    for (int c = 0; c < nchunks; ++c) {
      const u32x4* bufc = buf + (c & 1) * kChunkVecs;
      const bool more = (c + 1 < nchunks);
      DBG_T(3 + 4 * c);
#ifndef MDBF_DBG_NOSTAGE
      if (more) stage_load(ein_thr, vin_row, p.vin_dt, (c + 1) * (CB * kBlockCols) + st_col, p.K, sr);
#endif
      // ---- full groups of this chunk; B operands are read from LDS one block ahead ---------------
#pragma unroll
      for (int gi = 0; gi < CB / 4; ++gi) {
        const int g = c * (CB / 4) + gi;
        if (g < NG) {
          u32x4 w[R];
#pragma unroll
          for (int r = 0; r < R; ++r) w[r] = wn[r];
#ifndef MDBF_DBG_NOSIGNLOAD
          if (g + 1 < NG) {
#pragma unroll
            for (int r = 0; r < R; ++r) wn[r] = sp[r][(g + 1) * 64];
          }
#endif
          BlockOps ops[4];
          load_block_ops(bufc + (gi * 4) * 256, rd_even, rd_odd, rd_virt, ops[0]);
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            uint32_t word[R];
#pragma unroll
            for (int r = 0; r < R; ++r) {
              const u32x4 t = w[r];
              word[r] = t[j];
            }
            if (j < 3) load_block_ops(bufc + (gi * 4 + j + 1) * 256, rd_even, rd_odd, rd_virt, ops[j + 1]);
            __builtin_amdgcn_sched_barrier(0);  // keep the LDS reads of the next block ahead of this block's MFMAs
            contract_block<R>(ops[j], avirt, word, acc, accv);
          }
        }
      }
      // ---- the 1..3 tail blocks (stored block-major) live in the last chunk ---------------------
      if (TB != 0 && c == nchunks - 1) {
#pragma unroll 1
        for (int tb = 0; tb < TB; ++tb) {
          const int q = 4 * NG + tb;
          uint32_t word[R];
#pragma unroll
          for (int r = 0; r < R; ++r) word[r] = stail[r][tb * 64];
          BlockOps ops;
          load_block_ops(bufc + (q - c * CB) * 256, rd_even, rd_odd, rd_virt, ops);
          contract_block<R>(ops, avirt, word, acc, accv);
        }
      }
      DBG_T(4 + 4 * c);
#ifndef MDBF_DBG_NOSTAGE
      if (more) stage_store(sr, buf + ((c + 1) & 1) * kChunkVecs + st_vec, st_sw);
#endif
      DBG_T(5 + 4 * c);
      __syncthreads();
      DBG_T(6 + 4 * c);
    }
    DBG_T(40);

    // ---- column sums of xs from the virtual all-ones row (all its output rows are equal) --------
    if (lane < 16) red[wave * 16 + lane] = accv[0] * virt_scale;
    __syncthreads();
    const float colsum = (red[n] + red[16 + n]) + (red[32 + n] + red[48 + n]);

    // ---- fix-up, envelope accumulate, store ----------------------------------------------------
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const bool tile_ok = (wave + 4 * r) < ntl;
      const int rowb = (tile0 + trel[r]) * kTileRows + 4 * kg;
      float ev[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int row = min(rowb + i, p.rows - 1);
        ev[i] = (float)((g_f16_ptr)p.Eout)[(size_t)row * 16 + n];
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int row = rowb + i;
        const float P = colsum - acc[r][0][i] * 33554432.f - acc[r][1][i] * 2097152.f;  // 2^25, 2^21
        const float v = row16_sum(ev[i] * P);
        if (tile_ok && n == 0 && row < p.rows) store_from_float(p.out, (int64_t)b * p.out_ld + row, p.out_dt, v);
      }
    }
    DBG_T(41);
    __syncthreads();  // red and the chunk buffers are reused by the next token
  }
}

template <int R>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2)))
void stage_fast_kernel(const StageProb* __restrict__ probs, const WorkItem* __restrict__ items, StageProb single,
                       int tiles_per_item) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  u32x4* buf = reinterpret_cast<u32x4*>(smem);
  float* red = reinterpret_cast<float*>(smem + 2 * kChunkVecs * 16);

  // Blocks are dealt round-robin to the 8 XCDs; give each XCD a contiguous run of work items so that
  // the items of one problem (which share Ein) meet in one L2.
  const int nb = gridDim.x, bx = blockIdx.x;
  const int xcd = bx & 7;
  const int item = xcd * (nb >> 3) + min(xcd, nb & 7) + (bx >> 3);

  StageProb p;
  int tile0, ntl;
  if (probs) {
    const WorkItem it = items[item];
    p = probs[it.prob];
    tile0 = it.tile0;
    ntl = it.ntiles;
  } else {
    p = single;
    tile0 = item * tiles_per_item;
    ntl = min(tiles_per_item, single.ntiles - tile0);
  }
  run_item<R>(p, tile0, ntl, buf, red);
}

template <int R>
static int launch_r(const StageProb* probs_dev, const WorkItem* items_dev, int nblocks, int tiles_per_item,
                    const StageProb* single, hipStream_t s) {
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&stage_fast_kernel<R>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kFastSmemBytes);
    if (e != hipSuccess) return (int)e;
    attr_set = true;
  }
  hipLaunchKernelGGL(stage_fast_kernel<R>, dim3((unsigned)nblocks), dim3(256), kFastSmemBytes, s, probs_dev,
                     items_dev, *single, tiles_per_item);
  return (int)hipGetLastError();
}

#ifdef MDBF_DBG_TIMING
extern "C" int mdbf_dbg_read(void* host, size_t bytes) {
  return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(g_dbg_time), bytes < sizeof(g_dbg_time) ? bytes : sizeof(g_dbg_time));
}
#endif

bool stage_is_fast(const StageProb& p) {
  if (p.l != 16 || p.env_dt != MDBF_F16 || (p.K & 7) != 0) return false;
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
                      const StageProb* single, hipStream_t s) {
  int nblocks = nitems;
  if (!probs_dev) nblocks = (single->ntiles + tiles_per_item - 1) / tiles_per_item;
  switch (tiles_per_item) {
    case 4: return launch_r<1>(probs_dev, items_dev, nblocks, tiles_per_item, single, s);
    case 8: return launch_r<2>(probs_dev, items_dev, nblocks, tiles_per_item, single, s);
    case 16: return launch_r<4>(probs_dev, items_dev, nblocks, tiles_per_item, single, s);
    default: return (int)hipErrorInvalidValue;
  }
}

}  // namespace mdbf
