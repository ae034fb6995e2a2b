// Internal declarations of libmdbf (HIP side only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>

#include "mdbf.h"

// Every pointer the kernels receive is device global memory.  Saying so in the pointer type makes the
// compiler emit global_* instead of flat_* accesses: a flat access also counts against the LDS counter, so
// a wait for an LDS read would wait for every global load in flight as well.
#define MDBF_GLOBAL __attribute__((address_space(1)))
#define MDBF_LDS __attribute__((address_space(3)))

namespace mdbf {

// ---------------------------------------------------------------------------------------
// Packed sign layout (one bit per entry, bit 1 <=> -1).
//
// A sign matrix S (rows x K, contracted along K) is cut into row tiles of 16 rows and column
// blocks of 128 entries.  One (tile, block) is 64 32-bit words, one per wavefront lane:
//   lane = kg*16 + r       r  = row inside the tile (0..15), kg = 8-column group (0..3)
//   local column kl (0..127) of the block:  f = kl/32 (which of the block's four 32-deep
//   matrix-core steps), kg = (kl%32)/8, e = kl%8, i = e/2, h = e%2
//   bit index inside the word = 8*(f/2) + 4*(f%2) + i + 16*h
// so that, with u = w >> 8*(f/2), the word  u & ((1<<(4c+i)) | (1<<(4c+i+16))),  c = f%2,
// viewed as two fp16 values, holds the entries (e = 2i, 2i+1) as {0 or 2^(4c+i-24)}: the
// operand of one matrix-core step costs one AND per register and no shift.
// Row tiles are stored in groups of 64 consecutive tiles (the last group holds what is left).  Inside a
// group the order is block-major: all tiles' words of block 0, then of block 1, ...  so that a workgroup
// that contracts a range of a group's tiles reads one contiguous run per block, and consecutive blocks
// follow each other (long sequential runs; a tile-major order puts a power-of-two stride between tiles for
// power-of-two K, which aliases HBM channels):
//   word offset of (tile t, block q, lane L), KB = blocks per row, g0 = 64*(t/64), Gt = min(64, tiles - g0):
//       (g0*KB + q*Gt + (t - g0))*64 + L
// Padding rows/columns hold bit 0.
// ---------------------------------------------------------------------------------------
constexpr int kTileRows = 16;
constexpr int kBlockCols = 128;

__host__ __device__ inline int num_tiles(int rows) { return (rows + kTileRows - 1) / kTileRows; }
__host__ __device__ inline int num_blocks(int cols) { return (cols + kBlockCols - 1) / kBlockCols; }
__host__ __device__ inline size_t packed_words(int rows, int cols) {
  return (size_t)num_tiles(rows) * (size_t)num_blocks(cols) * 64u;
}
constexpr int kGroupTiles = 64;
// tiles in the group that holds `tile`
__host__ __device__ inline int group_tiles(int tile, int ntiles) {
  const int g0 = tile & ~(kGroupTiles - 1);
  return ntiles - g0 < kGroupTiles ? ntiles - g0 : kGroupTiles;
}
// word offset of (tile, block 0, lane 0); consecutive blocks of the tile are group_tiles()*64 words apart
__host__ __device__ inline size_t tile_base_words(int tile, int KB) {
  const int g0 = tile & ~(kGroupTiles - 1);
  return ((size_t)g0 * (size_t)KB + (size_t)(tile - g0)) * 64u;
}
__host__ __device__ inline size_t word_offset(int tile, int q, int lane, int KB, int ntiles) {
  return tile_base_words(tile, KB) + (size_t)q * (size_t)group_tiles(tile, ntiles) * 64u + (size_t)lane;
}
// bit index of local column kl (0..127) inside its lane's word, and the lane's 8-column group
__host__ __device__ inline int bit_of_local_col(int kl) {
  const int f = kl >> 5, e = kl & 7, i = e >> 1, h = e & 1;
  return 8 * (f >> 1) + 4 * (f & 1) + i + 16 * h;
}
__host__ __device__ inline int kgroup_of_local_col(int kl) { return (kl & 31) >> 3; }

// ---------------------------------------------------------------------------------------
// One envelope-scaled binary product ("stage"):
//   out[b, r] = sum_c Eout[r,c] * ( sum_j S[r,j] * Ein[j,c] * vin[b,j] )      r < rows, b < T
// Stage 1 of a layer: S=SB, Ein=B, vin=X, Eout=G, out=z (fp32 workspace).
// Stage 2 of a layer: S=SA, Ein=Q, vin=z, Eout=A, out=Y.
// ---------------------------------------------------------------------------------------
struct StageProb {
  const uint32_t* S;
  const void* Ein;
  const void* Eout;
  const void* vin;
  void* out;
  void* xs;            // pre-scaled activations in B-operand order (T x chunks x 32 KB), or null
  int64_t vin_ld, out_ld;
  int32_t rows, K, l, T;
  int32_t KB, ntiles;
  int32_t env_dt, vin_dt, out_dt;
  int32_t flags;       // kStageAccumulate
};
constexpr int32_t kStageAccumulate = 1;   // out += result instead of out = result

// A unit of work of the stage kernels: row tiles [tile0, tile0+ntiles) of problem `prob`, with a copy
// of the problem so that one 128-byte read describes the whole item.
struct alignas(128) WorkItem {
  StageProb p;
  int32_t tile0, ntiles, prob, pad_;
};
static_assert(sizeof(StageProb) == 104, "StageProb layout is read dword by dword on the device");
static_assert(sizeof(WorkItem) == 128, "WorkItem must be 128 bytes");

// Plan of a batched forward (host and device copies are byte-identical).
struct PlanHeader {
  uint32_t magic;
  int32_t count;              // layers
  int32_t nitems[2];          // work items of stage 1 / stage 2
  int32_t tiles_per_item[2];  // upper bound of WorkItem::ntiles, per stage
  int32_t precise;            // all layers use the fp32 path
  int32_t fast[2];            // every problem of the stage qualifies for the fast matrix-core variant
  int32_t pre[2];             // ... and has a buffer for pre-scaled activations (written by the scale-in kernel)
  int32_t max_units[2];       // largest tokens x chunks of a problem of the stage (grid of the scale-in kernel)
  int32_t mx[2];              // every problem of the stage qualifies for the block-scaled variant and has this
                              // envelope rank (16 or 8); 0: the stage runs another variant
  int32_t gemm;               // every layer has kGemmMinTokensPlan tokens or more: many-token variant
  int32_t gemm_mode[2];       // its load mode per stage
  int32_t max_tokens;         // longest token count among the layers
  int32_t max_units_mx[2];    // grid of that variant's scale-in kernel
  uint64_t probs_off[2];      // byte offsets of StageProb[count] for stage 1 / 2
  uint64_t items_off[2];      // byte offsets of WorkItem[nitems[s]]
  uint64_t total_bytes;
  int32_t fuse2;              // both stages run the block-scaled variant at one rank: the first stage's launch
                              // writes the second stage's activation records (no scale-in launch for stage 2)
  int32_t pad_;
};
constexpr uint32_t kPlanMagic = 0x4D444246u;  // "MDBF"

// One-time set-up of a kernel per device (raising its dynamic LDS limit): thread-safe, and the outcome of
// the one attempt is what every later call on that device reports.
constexpr int kMaxDevices = 64;
struct KernelSetup {
  std::once_flag once[kMaxDevices];
  int err[kMaxDevices];
};
template <class F>
inline int kernel_setup(KernelSetup& k, F&& fn) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return (int)e;
  if (dev < 0 || dev >= kMaxDevices) return (int)hipErrorInvalidDevice;
  std::call_once(k.once[dev], [&] { k.err[dev] = (int)fn(); });
  return k.err[dev];
}

// launchers (defined in the kernel translation units); return hipError_t as int
int launch_pack(const int8_t* signs, int rows, int cols, int64_t ld, uint32_t* packed, hipStream_t s);
int launch_unpack(const uint32_t* packed, int rows, int cols, int8_t* signs, int64_t ld, hipStream_t s);
int launch_pad_envelope(const void* src, int rows, int l, void* dst, int l_to, int es, hipStream_t s);
int launch_stream_read(const void* src, size_t bytes, uint32_t* sink, int sink_words, hipStream_t s);
int launch_stage_precise(const StageProb* probs_dev, const WorkItem* items_dev, int nitems,
                         const StageProb* single, hipStream_t s);
// pre: the problems' xs buffers hold the pre-scaled activations (launch_scale_in ran before)
int launch_stage_mfma(const StageProb* probs_dev, const WorkItem* items_dev, int nitems, int tiles_per_item,
                      const StageProb* single, bool pre, hipStream_t s);
int launch_stage_generic(const StageProb* probs_dev, const WorkItem* items_dev, int nitems, int tiles_per_item,
                         const StageProb* single, hipStream_t s);
// scale-in kernel: writes xs = fp16(Ein * vin) of every (problem, token, 1024-column chunk) to p.xs in the
// order the matrix-core kernel copies it to LDS (paper Eq. "me-dbf-expand", the D_b / D_q factors)
int launch_scale_in(const StageProb* probs_dev, int count, int max_units, const StageProb* single, hipStream_t s);
// bytes of one problem's xs buffer
size_t xs_bytes_for(int K, int T);
// Block-scaled (MX) variant of the matrix-core kernel: signs as fp4, activations as three fp6 limbs with a
// power-of-two scale per 32 values, written by its own scale-in kernel into the same xs buffer.
size_t xs_bytes_for_mx(int K, int T);
int mx_item_tiles();                         // row tiles per work item of this variant at most (64)
// row tiles per work item (64, 56 or 48) for a launch over problems of ntiles[i] row tiles, kb[i] blocks
int mx_pick_item_tiles(int count, const int* ntiles, const int* kb);
int mx_max_workgroups();                     // workgroups of this variant the current device holds at once
bool stage_is_mx(const StageProb& p);        // l == 16 or 8, fp16 envelopes, an xs buffer, few tokens
// max_units: largest tokens x blocks of a problem of the launch
int launch_scale_in_mx(const StageProb* probs_dev, int count, int max_units, const StageProb* single,
                       hipStream_t s);
// items_dev null: one problem (`single`), items are cut on the fly
// single->l = the envelope rank of the launch (16 or 8; a plan's problems all have the same); with items_dev,
// single->ntiles = the row tiles per work item the plan was cut with (mx_pick_item_tiles)
// next_probs_dev (plans only, or null): the problems of the factor that follows, indexed like this launch's
// (WorkItem::prob); with it the launch writes that factor's activation records itself (no scale-in launch
// for it) and does not store its own results.  Needs that factor to be served by this variant too.
int launch_stage_mx(const WorkItem* items_dev, int nitems, const StageProb* single, const StageProb* next_probs_dev,
                    hipStream_t s);
// Split variant of the block-scaled kernel for one small problem with one token: workgroup (g, s) takes row
// tiles 8g .. 8g + 7 and `bs` blocks of the contraction dimension and builds its activation records itself;
// the partial sums of the nsplit workgroups of a tile group are added in a fixed order, by the reader
// (part_in of the next launch) or by the last workgroup of the group to finish (counters).
struct SplitGeom {
  int bs, nsplit, ngroup;
};
SplitGeom split_geom(int ntiles, int KB);    // host arithmetic only: the same on every machine
bool stage_is_split(const StageProb& p);     // l == 16 or 8, fp16 envelopes, one token
// part_in (or null: p->vin): nsplit_in vectors part_in_ld apart whose sum is the activation vector.
// part_out: g.nsplit vectors part_out_ld apart (unused when g.nsplit == 1: the result goes to p->out).
// counters (or null): g.ngroup zeroed words; with them the launch itself stores the sums to p->out.
// clear (or null): nclear words this launch sets to zero.
int launch_stage_mx_split(const StageProb* p, const SplitGeom& g, const float* part_in, int nsplit_in,
                          int64_t part_in_ld, float* part_out, int64_t part_out_ld, uint32_t* counters,
                          uint32_t* clear, int nclear, hipStream_t s);
constexpr int kMaxPreTokens = 16;   // token counts up to this use the scale-in kernel
// true if the fast matrix-core variant can run the problem (l == 16, fp16 envelopes, K % 8 == 0,
// 16-byte aligned activation rows); otherwise the general variant is used
bool stage_is_fast(const StageProb& p);
// tiles per work item the matrix-core kernel wants for a problem with `ntiles` row tiles when
// `total_tiles` tiles are in flight in the same launch
int mfma_tiles_per_item(long total_tiles);

// Many-token variant: the product as a dense GEMM against the factor rebuilt on the fly (any l <= 16, any
// dtypes and shapes); one launch per problem, grid = row blocks x token blocks.
// Token counts from which the many-token variant is taken: a single call (one layer cannot fill the device
// with the streaming kernels, the rebuild costs the same for 1 to 16 tokens), and a plan (the streaming
// kernels read the signs once per token; the rebuild pays off from a few tokens on).
constexpr int kGemmMinTokensSingle = 2;
constexpr int kGemmMinTokensPlan = 4;
bool stage_is_gemm(const StageProb& p);
// how the kernel may load the problem's operands: a dtype code (vector loads of that activation type, fp16
// rank-16 envelopes, aligned rows) or 3 (element by element); a plan takes 3 unless all problems agree
int gemm_load_mode(const StageProb& p);
// compute units of the current device (cached after the first call; 256 if the query fails)
int compute_units();
int gemm_tiles_per_item();
int gemm_plan_max_tokens();
// items_dev null: the single problem *p (mode ignored).  Else the work items of a plan (at most
// gemm_plan_max_tokens() tokens per problem); p->T = the longest token count among its problems, mode as above.
int launch_stage_gemm(const WorkItem* items_dev, int nitems, int mode, const StageProb* p, hipStream_t s);

// MSVID_l (sign mask + truncated SVD of |Z| by block subspace iteration), csrc/mdbf_msvid.hip
int msvid_block(int l);                                  // columns of the iteration's block: l plus oversampling
size_t msvid_ws_bytes(int rows, int cols, int l);
int launch_msvid(const float* Z, int rows, int cols, int64_t ld, int l, int iters, const float* X0, int8_t* S, float* A,
                 float* Q, float* sigma, void* ws, hipStream_t s);

// dtype helpers (device)
__device__ inline float load_as_float(const void* p, int64_t idx, int dt) {
  if (dt == MDBF_F32) return ((const MDBF_GLOBAL float*)p)[idx];
  if (dt == MDBF_F16) return (float)((const MDBF_GLOBAL _Float16*)p)[idx];
  uint32_t u = ((uint32_t)((const MDBF_GLOBAL uint16_t*)p)[idx]) << 16;
  return __builtin_bit_cast(float, u);
}
__device__ inline uint16_t float_to_bf16_rne(float f) {
  uint32_t u = __builtin_bit_cast(uint32_t, f);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x40u);  // NaN
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
__device__ inline void store_from_float(void* p, int64_t idx, int dt, float v) {
  if (dt == MDBF_F32) ((MDBF_GLOBAL float*)p)[idx] = v;
  else if (dt == MDBF_F16) ((MDBF_GLOBAL _Float16*)p)[idx] = (_Float16)v;
  else ((MDBF_GLOBAL uint16_t*)p)[idx] = float_to_bf16_rne(v);
}
// the store of a stage's result: plain, or added to what `p[idx]` holds (kStageAccumulate)
__device__ inline void emit_result(void* p, int64_t idx, int dt, float v, int flags) {
  if (flags & kStageAccumulate) v += load_as_float(p, idx, dt);
  store_from_float(p, idx, dt, v);
}
__host__ __device__ inline int dtype_size(int dt) { return dt == MDBF_F32 ? 4 : 2; }

}  // namespace mdbf
