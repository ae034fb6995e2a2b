// C ABI of libmdbf: argument validation, storage accounting, plans and kernel dispatch.
// Every argument check happens before the first HIP call.
#include <math.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <atomic>
#include <vector>

#include "mdbf_internal.h"

using namespace mdbf;

namespace {

thread_local char g_hip_err[256] = "";

int hip_fail(int e) {
  if (e == 0) return MDBF_OK;
  snprintf(g_hip_err, sizeof(g_hip_err), "%s", hipGetErrorString((hipError_t)e));
  return MDBF_EHIP;
}

bool valid_dtype(int d) { return d == MDBF_F16 || d == MDBF_BF16 || d == MDBF_F32; }
bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
int kpad_of(int k) { return (k + 7) & ~7; }  // z rows stay 32-byte aligned

int check_desc(const mdbf_desc_t* d) {
  if (!d) return MDBF_EINVAL;
  if (d->m <= 0 || d->n <= 0 || d->k <= 0) return MDBF_EINVAL;
  if (d->l < 1 || d->l > MDBF_MAX_L) return MDBF_EINVAL;
  if (!valid_dtype(d->x_dtype) || !valid_dtype(d->env_dtype) || !valid_dtype(d->y_dtype)) return MDBF_EDTYPE;
  if (d->flags & ~(MDBF_FLAG_PRECISE | MDBF_FLAG_BLOCK_SCALED | MDBF_FLAG_ACCUMULATE | MDBF_FLAG_FP16_STAGED))
    return MDBF_EUNSUPPORTED;
  if ((d->flags & MDBF_FLAG_BLOCK_SCALED) && (d->flags & MDBF_FLAG_FP16_STAGED)) return MDBF_EINVAL;
  return MDBF_OK;
}

size_t z_bytes(const mdbf_desc_t* d, int T) { return align_up((size_t)T * (size_t)kpad_of(d->k) * 4u, 256); }

// Buffers for the pre-scaled activations of the two stages (only for small token counts and the
// fp16-envelope cases of rank 16 or 8 the matrix-core kernels serve; zero otherwise).
bool wants_xs(const mdbf_desc_t* d, int T) {
  return T <= kMaxPreTokens && (d->l == 16 || d->l == 8) && d->env_dtype == MDBF_F16 &&
         !(d->flags & MDBF_FLAG_PRECISE);
}
size_t xs_need(int K, int T) {
  const size_t a = xs_bytes_for(K, T), b = xs_bytes_for_mx(K, T);
  return align_up(a > b ? a : b, 256);
}
size_t xs1_bytes(const mdbf_desc_t* d, int T) { return wants_xs(d, T) ? xs_need(d->n, T) : 0; }
size_t xs2_bytes(const mdbf_desc_t* d, int T) { return wants_xs(d, T) ? xs_need(d->k, T) : 0; }

// The block-scaled variant is the default where it applies; MDBF_FLAG_FP16_STAGED in the descriptor keeps a
// layer (and with it the plan it sits in) on the fp16-staged variants.
bool use_mx(const StageProb& p, uint32_t flags) { return !(flags & MDBF_FLAG_FP16_STAGED) && stage_is_mx(p); }
// The block-scaled kernel walks the contraction dimension in stages of fixed latency and shares one copy of
// the activation stream among 64 row tiles: it pays off when the launch has enough row tiles to give every
// workgroup slot of the device an item.  Smaller launches (a single layer) go to the fp16 variant, whose
// items are 4 to 16 tiles.
bool mx_worthwhile(long launch_tiles) {
  return launch_tiles >= (long)mx_item_tiles() * (long)mx_max_workgroups();
}
size_t plan_layer_ws_bytes(const mdbf_desc_t* d, int T) { return z_bytes(d, T) + xs1_bytes(d, T) + xs2_bytes(d, T); }

// A single call with one token splits the contraction of each factor across workgroups (split_geom); its
// partial sums and the completion counters of the second factor lie behind the plan-style workspace.
bool wants_split(const mdbf_desc_t* d, int T) {
  return T == 1 && (d->l == 16 || d->l == 8) && d->env_dtype == MDBF_F16 &&
         !(d->flags & (MDBF_FLAG_PRECISE | MDBF_FLAG_FP16_STAGED));
}
struct SplitLayout {
  SplitGeom g[2];
  int64_t ld[2];                 // floats between the partial vectors of factor 1 / 2
  size_t part_off[2], ctr_off, bytes;   // offsets from the start of the split region
};
SplitLayout split_layout(const mdbf_desc_t* d) {
  SplitLayout L;
  L.g[0] = split_geom(num_tiles(d->k), num_blocks(d->n));
  L.g[1] = split_geom(num_tiles(d->m), num_blocks(d->k));
  L.ld[0] = (int64_t)align_up((size_t)d->k, 64);
  L.ld[1] = (int64_t)align_up((size_t)d->m, 64);
  L.part_off[0] = 0;
  L.part_off[1] = align_up((size_t)L.g[0].nsplit * (size_t)L.ld[0] * 4u, 256);
  L.ctr_off = L.part_off[1] + align_up((size_t)L.g[1].nsplit * (size_t)L.ld[1] * 4u, 256);
  L.bytes = L.ctr_off + align_up((size_t)L.g[1].ngroup * 4u, 256);
  return L;
}
size_t layer_ws_bytes(const mdbf_desc_t* d, int T) {
  return plan_layer_ws_bytes(d, T) + (wants_split(d, T) ? split_layout(d).bytes : 0);
}

int check_layer(const mdbf_desc_t* d, const void* SA, const void* SB, const mdbf_env_t* env, const void* X,
                int64_t ldx, void* Y, int64_t ldy, int T) {
  int st = check_desc(d);
  if (st) return st;
  if (!SA || !SB || !env || !X || !Y) return MDBF_EINVAL;
  if (!env->A_dev || !env->Q_dev || !env->G_dev || !env->B_dev) return MDBF_EINVAL;
  if (T < 1) return MDBF_EINVAL;
  if (ldx < d->n || ldy < d->m) return MDBF_EINVAL;
  if (!aligned16(SA) || !aligned16(SB) || !aligned16(X) || !aligned16(Y) || !aligned16(env->A_dev) ||
      !aligned16(env->Q_dev) || !aligned16(env->G_dev) || !aligned16(env->B_dev))
    return MDBF_EALIGN;
  return MDBF_OK;
}

// the two stage problems of one layer (paper Eq. "me-dbf-expand": V first, then U)
void make_stages(const mdbf_desc_t* d, const void* SA, const void* SB, const mdbf_env_t* env, const void* X,
                 int64_t ldx, void* Y, int64_t ldy, int T, void* ws, StageProb out[2]) {
  void* z = ws;
  unsigned char* xs1 = (unsigned char*)ws + z_bytes(d, T);
  unsigned char* xs2 = xs1 + xs1_bytes(d, T);
  StageProb s1;
  memset(&s1, 0, sizeof(s1));
  s1.S = (const uint32_t*)SB;
  s1.Ein = env->B_dev;
  s1.Eout = env->G_dev;
  s1.vin = X;
  s1.out = z;
  s1.xs = xs1_bytes(d, T) ? xs1 : nullptr;
  s1.vin_ld = ldx;
  s1.out_ld = kpad_of(d->k);
  s1.rows = d->k;
  s1.K = d->n;
  s1.l = d->l;
  s1.T = T;
  s1.KB = num_blocks(d->n);
  s1.ntiles = num_tiles(d->k);
  s1.env_dt = d->env_dtype;
  s1.vin_dt = d->x_dtype;
  s1.out_dt = MDBF_F32;
  StageProb s2;
  memset(&s2, 0, sizeof(s2));
  s2.S = (const uint32_t*)SA;
  s2.Ein = env->Q_dev;
  s2.Eout = env->A_dev;
  s2.vin = z;
  s2.out = Y;
  s2.xs = xs2_bytes(d, T) ? xs2 : nullptr;
  s2.vin_ld = kpad_of(d->k);
  s2.out_ld = ldy;
  s2.rows = d->m;
  s2.K = d->k;
  s2.l = d->l;
  s2.T = T;
  s2.KB = num_blocks(d->k);
  s2.ntiles = num_tiles(d->m);
  s2.env_dt = d->env_dtype;
  s2.vin_dt = MDBF_F32;
  s2.out_dt = d->y_dtype;
  s2.flags = (d->flags & MDBF_FLAG_ACCUMULATE) ? kStageAccumulate : 0;
  out[0] = s1;
  out[1] = s2;
}

// The many-token kernel rounds its activations to fp16 as it loads them.  When it runs both factors, the
// first one stores z in fp16 right away: the same values reach the second product (one rounding, to nearest
// even, either way), with half the bytes to move and no conversion on the way in.
void half_intermediate(StageProb sp[2]) {
  sp[0].out_dt = MDBF_F16;
  sp[1].vin_dt = MDBF_F16;
}

}  // namespace

int mdbf::compute_units() {
  // one slot per device, filled by the first successful query (an atomic: any thread may be the first)
  static std::atomic<int> cached[kMaxDevices];
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return 256;
  const int have = cached[dev].load(std::memory_order_relaxed);
  if (have > 0) return have;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
    return 256;   // not cached: the next call asks again
  cached[dev].store(cus, std::memory_order_relaxed);
  return cus;
}

extern "C" {

double mdbf_bpw(int m, int n, int k, int l, int env_bits, int merge_inner) {
  if (m <= 0 || n <= 0 || k <= 0 || l < 1 || env_bits < 1) return -1.0;
  if (merge_inner && l != 1) return -1.0;
  const double sign_bits = ((double)m + (double)n) * (double)k;
  const double real_entries = merge_inner ? ((double)m + n + k) : (double)l * ((double)m + n + 2.0 * k);
  return (sign_bits + (double)env_bits * real_entries) / ((double)m * (double)n);
}

int mdbf_rank_for_budget(int m, int n, int l, double bpw, int env_bits, int multiple) {
  if (m <= 0 || n <= 0 || l < 1 || env_bits < 1 || !(bpw > 0.0)) return MDBF_EINVAL;
  const double mn = (double)m * (double)n, s = (double)m + (double)n;
  const double k_real = (bpw * mn - (double)env_bits * l * s) / (s + 2.0 * env_bits * l);
  if (k_real < 0.0) return 0;
  if (multiple <= 1) {
    long k = (long)floor(k_real + 1e-9);
    while (k > 0 && mdbf_bpw(m, n, (int)k, l, env_bits, 0) > bpw + 1e-12) --k;
    while (mdbf_bpw(m, n, (int)k + 1, l, env_bits, 0) <= bpw + 1e-12) ++k;
    return (int)k;
  }
  return (int)(multiple * floor(k_real / multiple + 0.5));
}

int mdbf_packed_bytes(int rows, int cols, size_t* bytes_out) {
  if (!bytes_out || rows <= 0 || cols <= 0) return MDBF_EINVAL;
  *bytes_out = packed_words(rows, cols) * 4u;
  return MDBF_OK;
}

int mdbf_pack(const int8_t* signs_dev, int rows, int cols, int64_t ld, void* packed_dev, size_t packed_bytes,
              void* stream) {
  if (!signs_dev || !packed_dev || rows <= 0 || cols <= 0 || ld < cols) return MDBF_EINVAL;
  if (!aligned16(packed_dev)) return MDBF_EALIGN;
  if (packed_bytes < packed_words(rows, cols) * 4u) return MDBF_EWORKSPACE;
  return hip_fail(launch_pack(signs_dev, rows, cols, ld, (uint32_t*)packed_dev, (hipStream_t)stream));
}

int mdbf_unpack(const void* packed_dev, int rows, int cols, int8_t* signs_dev, int64_t ld, void* stream) {
  if (!signs_dev || !packed_dev || rows <= 0 || cols <= 0 || ld < cols) return MDBF_EINVAL;
  if (!aligned16(packed_dev)) return MDBF_EALIGN;
  return hip_fail(launch_unpack((const uint32_t*)packed_dev, rows, cols, signs_dev, ld, (hipStream_t)stream));
}

int mdbf_pad_envelope(const void* env_dev, int rows, int l, int dtype, void* out_dev, int l_to, void* stream) {
  if (!env_dev || !out_dev || rows <= 0 || l < 1 || l_to < l || l_to > MDBF_MAX_L) return MDBF_EINVAL;
  if (!valid_dtype(dtype)) return MDBF_EDTYPE;
  if (!aligned16(env_dev) || !aligned16(out_dev)) return MDBF_EALIGN;
  return hip_fail(launch_pad_envelope(env_dev, rows, l, out_dev, l_to, dtype_size(dtype), (hipStream_t)stream));
}

int mdbf_stream_read(const void* src_dev, size_t bytes, uint32_t* sink_dev, int sink_words, void* stream) {
  if (!src_dev || !sink_dev || bytes == 0 || (bytes & 15) != 0) return MDBF_EINVAL;
  if (sink_words < 4 || sink_words > (1 << 20) || (sink_words & 3) != 0) return MDBF_EINVAL;
  if (!aligned16(src_dev) || !aligned16(sink_dev)) return MDBF_EALIGN;
  return hip_fail(launch_stream_read(src_dev, bytes, sink_dev, sink_words, (hipStream_t)stream));
}

int mdbf_workspace_bytes(const mdbf_desc_t* desc, int T, size_t* bytes_out) {
  int st = check_desc(desc);
  if (st) return st;
  if (!bytes_out || T < 1) return MDBF_EINVAL;
  *bytes_out = layer_ws_bytes(desc, T);
  return MDBF_OK;
}

int mdbf_forward(const mdbf_desc_t* desc, const void* SA_packed_dev, const void* SB_packed_dev,
                 const mdbf_env_t* env, const void* X_dev, int64_t ldx, void* Y_dev, int64_t ldy, int T,
                 void* workspace_dev, size_t workspace_bytes, void* stream) {
  int st = check_layer(desc, SA_packed_dev, SB_packed_dev, env, X_dev, ldx, Y_dev, ldy, T);
  if (st) return st;
  if (!workspace_dev) return MDBF_EINVAL;
  if (!aligned16(workspace_dev)) return MDBF_EALIGN;
  if (workspace_bytes < layer_ws_bytes(desc, T)) return MDBF_EWORKSPACE;
  StageProb sp[2];
  make_stages(desc, SA_packed_dev, SB_packed_dev, env, X_dev, ldx, Y_dev, ldy, T, workspace_dev, sp);
  hipStream_t s = (hipStream_t)stream;
  if (wants_split(desc, T) && stage_is_split(sp[0]) && stage_is_split(sp[1])) {
    // two launches, no scale-in launch: the second factor's workgroups add up the first factor's partial sums
    const SplitLayout L = split_layout(desc);
    unsigned char* base = (unsigned char*)workspace_dev + plan_layer_ws_bytes(desc, T);
    float* part1 = (float*)(base + L.part_off[0]);
    float* part2 = (float*)(base + L.part_off[1]);
    uint32_t* ctr = (uint32_t*)(base + L.ctr_off);
    const bool direct1 = L.g[0].nsplit == 1;         // then z itself is written and read
    int e = launch_stage_mx_split(&sp[0], L.g[0], nullptr, 0, 0, part1, L.ld[0], nullptr, ctr, L.g[1].ngroup, s);
    if (e) return hip_fail(e);
    e = launch_stage_mx_split(&sp[1], L.g[1], direct1 ? nullptr : part1, direct1 ? 0 : L.g[0].nsplit, L.ld[0], part2,
                              L.ld[1], ctr, nullptr, 0, s);
    return hip_fail(e);
  }
  {
    bool both_gemm = !(desc->flags & MDBF_FLAG_PRECISE) && T >= kGemmMinTokensSingle;
    for (int i = 0; i < 2; ++i)
      both_gemm = both_gemm && stage_is_gemm(sp[i]) && !((desc->flags & MDBF_FLAG_BLOCK_SCALED) && use_mx(sp[i], desc->flags));
    if (both_gemm) half_intermediate(sp);
  }
  for (int i = 0; i < 2; ++i) {
    int e;
    const bool forced_mx = (desc->flags & MDBF_FLAG_BLOCK_SCALED) && use_mx(sp[i], desc->flags);
    if (desc->flags & MDBF_FLAG_PRECISE)
      e = launch_stage_precise(nullptr, nullptr, 0, &sp[i], s);
    else if (!forced_mx && T >= kGemmMinTokensSingle && stage_is_gemm(sp[i]))
      e = launch_stage_gemm(nullptr, 0, 0, &sp[i], s);
    else if (forced_mx || (use_mx(sp[i], desc->flags) && (mx_worthwhile(sp[i].ntiles) || !stage_is_fast(sp[i])))) {
      // (a small launch the fp16 variant cannot take -- rank 8 -- is still better off here than in the
      // element-wise kernel)
      e = launch_scale_in_mx(nullptr, 1, T * sp[i].KB, &sp[i], s);
      if (e) return hip_fail(e);
      e = launch_stage_mx(nullptr, 0, &sp[i], nullptr, s);
    }
    else if (stage_is_fast(sp[i])) {
      const bool pre = sp[i].xs != nullptr;
      if (pre) {
        const int units = T * ((sp[i].KB + 7) / 8);
        e = launch_scale_in(nullptr, 1, units, &sp[i], s);
        if (e) return hip_fail(e);
      }
      e = launch_stage_mfma(nullptr, nullptr, 0, mfma_tiles_per_item(sp[i].ntiles), &sp[i], pre, s);
    }
    else
      e = launch_stage_generic(nullptr, nullptr, 0, mfma_tiles_per_item(sp[i].ntiles), &sp[i], s);
    if (e) return hip_fail(e);
  }
  return MDBF_OK;
}

// ---- scratch memory of mdbf_forward_static: one array per device, owned by the loaded code object.  In host
// code the array's name is only a handle for hipGetSymbolAddress; the device address is looked up once per
// device (with that device current) and kept.
}  // extern "C"
static __device__ __align__(256) unsigned char scratch[MDBF_STATIC_SCRATCH_BYTES];
namespace {
constexpr size_t kStaticScratchBytes = MDBF_STATIC_SCRATCH_BYTES;
struct ScratchSlots {
  std::once_flag once[kMaxDevices];
  void* ptr[kMaxDevices];
  int err[kMaxDevices];
};
ScratchSlots g_scratch;
// device address of the current device's copy of `scratch`; returns a hipError_t as int
int static_scratch(void** out) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return (int)e;
  if (dev < 0 || dev >= kMaxDevices) return (int)hipErrorInvalidDevice;
  std::call_once(g_scratch.once[dev], [&] {
    void* p = nullptr;
    hipError_t r = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    g_scratch.ptr[dev] = (r == hipSuccess) ? p : nullptr;
    g_scratch.err[dev] = (int)r;
  });
  if (g_scratch.err[dev]) return g_scratch.err[dev];
  if (!g_scratch.ptr[dev]) return (int)hipErrorInvalidSymbol;
  *out = g_scratch.ptr[dev];
  return 0;
}
}  // namespace
extern "C" {

int mdbf_forward_static(const mdbf_desc_t* desc, const void* SA_packed_dev, const void* SB_packed_dev,
                        const mdbf_env_t* env, const void* X_dev, int64_t ldx, void* Y_dev, int64_t ldy, int T,
                        void* stream) {
  int st = check_layer(desc, SA_packed_dev, SB_packed_dev, env, X_dev, ldx, Y_dev, ldy, T);
  if (st) return st;
  if (layer_ws_bytes(desc, T) > kStaticScratchBytes) return MDBF_EWORKSPACE;
  void* ws = nullptr;
  int e = static_scratch(&ws);
  if (e) return hip_fail(e);
  // Nothing in the scratch has to start at zero: every byte a kernel of the call reads (z, the scaled
  // activations' records) is written earlier in the same call.
  return mdbf_forward(desc, SA_packed_dev, SB_packed_dev, env, X_dev, ldx, Y_dev, ldy, T, ws, kStaticScratchBytes,
                      stream);
}

// Work items of a stage of the block-scaled kernel, reordered for its static schedule.  The kernel's
// workgroups (nwg of them; groups of nwg / 8 per XCD when nwg is a multiple of 8) walk a contiguous slice
// [lo, hi) of the table: workgroup j of the slice takes entries lo + j, lo + j + stride, ..., so the first
// (hi - lo) mod stride workgroups take one entry more than the others.  An item costs its stage count
// (tokens x (ceil(KB / 2) + 1)), whatever its tile count; with problems of different contraction lengths in
// one plan the slice's workgroups would end at very different times.  Within each slice: items in
// descending cost (ties keep their order), each to the workgroup with the least cost so far among those
// with a free entry (ties: the one with fewer entries in all, then the lowest index), so that the costliest
// items land where fewer items go.  Slices whose items all cost the same keep their order.
// A stage of the block-scaled kernel whose items all cost the same and do not fill a whole number of rounds
// of the device's workgroups (1344 items on 256 workgroups: 5.25 rounds) ends with a round in which most
// workgroups idle.  The items of that last, partial round are cut into pieces of fewer row tiles (multiples
// of the 8 tiles a contraction wave owns), as many as give every workgroup one piece: a piece's stages are
// shorter than a full item's (fewer waves contract, on separate SIMDs), so the last round is.  The pieces are
// dealt to the ends of the eight per-XCD slices the kernel walks.  Returns the new number of items
// (at most `cap`, the room of the table).
static int split_last_round(std::vector<WorkItem>& items, int max_wgs, size_t cap) {
  const int n = (int)items.size();
  if (n <= max_wgs || (max_wgs & 7) != 0) return n;
  const int r = n % max_wgs;
  if (r == 0 || 2 * r > max_wgs) return n;
  const long c0 = (long)items[0].p.T * ((items[0].p.KB + 1) / 2 + 1);
  for (const WorkItem& w : items)
    if ((long)w.p.T * ((w.p.KB + 1) / 2 + 1) != c0) return n;
  int pieces = max_wgs / r;
  if (pieces > 8) pieces = 8;
  std::vector<WorkItem> full(items.begin(), items.end() - r), small;
  for (int i = n - r; i < n; ++i) {
    const WorkItem& w = items[(size_t)i];
    const int per = ((w.ntiles + pieces - 1) / pieces + 7) & ~7;     // tiles per piece: whole contraction waves
    for (int t = 0; t < w.ntiles; t += per) {
      WorkItem q = w;
      q.tile0 = w.tile0 + t;
      q.ntiles = w.ntiles - t < per ? w.ntiles - t : per;
      small.push_back(q);
    }
  }
  if (full.size() + small.size() > cap) return n;
  items.clear();
  for (int x = 0; x < 8; ++x) {
    items.insert(items.end(), full.begin() + (long)full.size() * x / 8, full.begin() + (long)full.size() * (x + 1) / 8);
    items.insert(items.end(), small.begin() + (long)small.size() * x / 8, small.begin() + (long)small.size() * (x + 1) / 8);
  }
  return (int)items.size();
}

static void balance_mx_items(WorkItem* items, int n, int max_wgs) {
  const int nwg = n < max_wgs ? n : max_wgs;
  const int slices = (nwg & 7) == 0 ? 8 : 1;
  const int stride = nwg / slices;
  if (stride < 1) return;
  std::vector<WorkItem> sorted;
  std::vector<long> load((size_t)stride);
  std::vector<int> cap((size_t)stride), used((size_t)stride);
  auto cost = [](const WorkItem& w) { return (long)w.p.T * ((w.p.KB + 1) / 2 + 1); };
  for (int x = 0; x < slices; ++x) {
    const int lo = (int)(((long)n * x) / slices), hi = (int)(((long)n * (x + 1)) / slices);
    const int cnt = hi - lo;
    if (cnt < 2) continue;
    sorted.assign(items + lo, items + hi);
    std::stable_sort(sorted.begin(), sorted.end(),
                     [&](const WorkItem& a, const WorkItem& b) { return cost(a) > cost(b); });
    if (cost(sorted.front()) == cost(sorted.back())) continue;
    for (int j = 0; j < stride; ++j) {
      cap[(size_t)j] = (cnt - j + stride - 1) / stride;   // entries lo + j + k * stride below hi
      used[(size_t)j] = 0;
      load[(size_t)j] = 0;
    }
    for (int i = 0; i < cnt; ++i) {
      int best = -1;
      for (int j = 0; j < stride; ++j) {
        if (used[(size_t)j] >= cap[(size_t)j]) continue;
        if (best < 0 || load[(size_t)j] < load[(size_t)best] ||
            (load[(size_t)j] == load[(size_t)best] && cap[(size_t)j] < cap[(size_t)best]))
          best = j;
      }
      items[lo + best + used[(size_t)best] * stride] = sorted[(size_t)i];
      ++used[(size_t)best];
      load[(size_t)best] += cost(sorted[(size_t)i]);
    }
  }
}

static int batch_layout(int count, const mdbf_layer_t* layers, PlanHeader* h, size_t* ws_bytes) {
  if (count < 1 || !layers) return MDBF_EINVAL;
  long tiles[2] = {0, 0};
  size_t ws = 0;
  int precise = 0;
  for (int i = 0; i < count; ++i) {
    const mdbf_layer_t* L = &layers[i];
    int st = check_layer(&L->desc, L->SA_packed_dev, L->SB_packed_dev, &L->env, L->X_dev, L->ldx, L->Y_dev,
                         L->ldy, L->T);
    if (st) return st;
    precise += (L->desc.flags & MDBF_FLAG_PRECISE) ? 1 : 0;
    tiles[0] += num_tiles(L->desc.k);
    tiles[1] += num_tiles(L->desc.m);
    ws += plan_layer_ws_bytes(&L->desc, L->T);
  }
  if (precise != 0 && precise != count) return MDBF_EUNSUPPORTED;  // all or none
  memset(h, 0, sizeof(*h));
  h->magic = kPlanMagic;
  h->count = count;
  h->precise = precise ? 1 : 0;
  // a stage whose problems all qualify for the block-scaled variant is cut into that variant's items
  int mx[2] = {1, 1};
  int all_fast[2] = {1, 1};
  for (int i = 0; i < count; ++i) {
    const mdbf_layer_t* L = &layers[i];
    StageProb sp[2];
    make_stages(&L->desc, L->SA_packed_dev, L->SB_packed_dev, &L->env, L->X_dev, L->ldx, L->Y_dev, L->ldy, L->T,
                (void*)(uintptr_t)256, sp);   // placeholder workspace: only the predicates are wanted
    for (int s = 0; s < 2; ++s) {
      // one envelope rank per launch of the block-scaled kernel
      if (!use_mx(sp[s], L->desc.flags) || (mx[s] != 1 && mx[s] != sp[s].l)) mx[s] = 0;
      else mx[s] = sp[s].l;
      if (!stage_is_fast(sp[s])) all_fast[s] = 0;
    }
  }
  int forced = 0, many = 0;
  for (int i = 0; i < count; ++i) {
    forced += (layers[i].desc.flags & MDBF_FLAG_BLOCK_SCALED) ? 1 : 0;
    many += (layers[i].T >= kGemmMinTokensPlan) ? 1 : 0;
    if (layers[i].T > h->max_tokens) h->max_tokens = layers[i].T;
  }
  h->gemm = (many == count && !precise && forced != count) ? 1 : 0;
  for (int s = 0; s < 2; ++s)
    if (h->gemm || (forced != count && !mx_worthwhile(tiles[s]) && all_fast[s])) mx[s] = 0;
  // otherwise one tile count per work item for both stages keeps one kernel instantiation per plan
  const int tpi_fp16 = mfma_tiles_per_item(tiles[0] < tiles[1] ? tiles[0] : tiles[1]);
  long nitems[2] = {0, 0};
  for (int s = 0; s < 2; ++s) {
    h->mx[s] = mx[s];
    int tpi_mx = mx_item_tiles();
    if (mx[s] && !h->gemm) {
      std::vector<int> nt(count), kb(count);
      for (int i = 0; i < count; ++i) {
        nt[i] = num_tiles(s == 0 ? layers[i].desc.k : layers[i].desc.m);
        kb[i] = num_blocks(s == 0 ? layers[i].desc.n : layers[i].desc.k) * layers[i].T;
      }
      tpi_mx = mx_pick_item_tiles(count, nt.data(), kb.data());
    }
    h->tiles_per_item[s] = h->gemm ? gemm_tiles_per_item() : mx[s] ? tpi_mx : tpi_fp16;
  }
  h->fuse2 = (!precise && !h->gemm && h->mx[0] != 0 && h->mx[0] == h->mx[1]) ? 1 : 0;
  for (int i = 0; i < count; ++i) {
    nitems[0] += (num_tiles(layers[i].desc.k) + h->tiles_per_item[0] - 1) / h->tiles_per_item[0];
    nitems[1] += (num_tiles(layers[i].desc.m) + h->tiles_per_item[1] - 1) / h->tiles_per_item[1];
  }
  if (nitems[0] + mx_max_workgroups() > 65535 || nitems[1] + mx_max_workgroups() > 65535) return MDBF_EUNSUPPORTED;
  h->nitems[0] = (int)nitems[0];
  h->nitems[1] = (int)nitems[1];
  size_t off = align_up(sizeof(PlanHeader), 256);
  for (int s = 0; s < 2; ++s) {
    h->probs_off[s] = off;
    off = align_up(off + (size_t)count * sizeof(StageProb), 256);
  }
  for (int s = 0; s < 2; ++s) {
    h->items_off[s] = off;
    // (room for the pieces the last round of a block-scaled stage may be cut into: at most one per workgroup)
    const size_t room = (size_t)nitems[s] + (h->mx[s] ? (size_t)mx_max_workgroups() : 0u);
    off = align_up(off + room * sizeof(WorkItem), 256);
  }
  h->total_bytes = off;
  *ws_bytes = ws;
  return MDBF_OK;
}

int mdbf_batch_plan_bytes(int count, const mdbf_layer_t* layers, size_t* plan_bytes_out,
                          size_t* workspace_bytes_out) {
  if (!plan_bytes_out || !workspace_bytes_out) return MDBF_EINVAL;
  PlanHeader h;
  size_t ws;
  int st = batch_layout(count, layers, &h, &ws);
  if (st) return st;
  *plan_bytes_out = (size_t)h.total_bytes;
  *workspace_bytes_out = ws;
  return MDBF_OK;
}

int mdbf_batch_plan_build(int count, const mdbf_layer_t* layers, void* workspace_dev, size_t workspace_bytes,
                          void* plan_host, size_t plan_bytes) {
  if (!plan_host || !workspace_dev) return MDBF_EINVAL;
  if (!aligned16(workspace_dev)) return MDBF_EALIGN;
  PlanHeader h;
  size_t ws;
  int st = batch_layout(count, layers, &h, &ws);
  if (st) return st;
  if (plan_bytes < h.total_bytes || workspace_bytes < ws) return MDBF_EWORKSPACE;
  // The tables are built in properly aligned host vectors and copied into the caller's buffer byte by byte:
  // plan_host needs no particular alignment.
  std::vector<StageProb> probs[2];
  std::vector<WorkItem> items[2];
  for (int s = 0; s < 2; ++s) {
    probs[s].resize((size_t)count);
    items[s].resize((size_t)h.nitems[s]);
  }
  size_t zoff = 0;
  int ni[2] = {0, 0};
  int fast[2] = {1, 1};
  int pre[2] = {1, 1};
  int max_units[2] = {1, 1};
  int max_units_mx[2] = {1, 1};
  int gmode[2] = {-1, -1};
  for (int i = 0; i < count; ++i) {
    const mdbf_layer_t* L = &layers[i];
    StageProb sp[2];
    make_stages(&L->desc, L->SA_packed_dev, L->SB_packed_dev, &L->env, L->X_dev, L->ldx, L->Y_dev, L->ldy, L->T,
                (unsigned char*)workspace_dev + zoff, sp);
    if (h.gemm) half_intermediate(sp);
    zoff += plan_layer_ws_bytes(&L->desc, L->T);
    for (int s = 0; s < 2; ++s) {
      probs[s][(size_t)i] = sp[s];
      if (!stage_is_fast(sp[s])) fast[s] = 0;
      const int gm = gemm_load_mode(sp[s]);
      gmode[s] = (gmode[s] == -1 || gmode[s] == gm) ? gm : 3;
      if (!sp[s].xs) pre[s] = 0;
      const int units = sp[s].T * ((sp[s].KB + 7) / 8);
      if (units > max_units[s]) max_units[s] = units;
      const int tpi = h.tiles_per_item[s];
      const int units_mx = sp[s].T * sp[s].KB;
      if (units_mx > max_units_mx[s]) max_units_mx[s] = units_mx;
      for (int t0 = 0; t0 < sp[s].ntiles; t0 += tpi) {
        WorkItem w;
        memset(&w, 0, sizeof(w));
        w.p = sp[s];
        w.prob = i;
        w.tile0 = t0;
        w.ntiles = sp[s].ntiles - t0 < tpi ? sp[s].ntiles - t0 : tpi;
        w.pad_ = 0;
        items[s][(size_t)ni[s]++] = w;
      }
    }
  }
  for (int s = 0; s < 2; ++s)
    if (h.mx[s] && !h.precise && !h.gemm) {
      balance_mx_items(items[s].data(), ni[s], mx_max_workgroups());
      ni[s] = split_last_round(items[s], mx_max_workgroups(), items[s].size() + (size_t)mx_max_workgroups());
      h.nitems[s] = ni[s];
    }
  h.fast[0] = fast[0];
  h.fast[1] = fast[1];
  h.pre[0] = fast[0] && pre[0];
  h.pre[1] = fast[1] && pre[1];
  h.max_units[0] = max_units[0];
  h.max_units[1] = max_units[1];
  for (int s = 0; s < 2; ++s) {
    h.max_units_mx[s] = max_units_mx[s];
    h.gemm_mode[s] = gmode[s];
  }
  unsigned char* base = (unsigned char*)plan_host;
  memset(base, 0, (size_t)h.total_bytes);
  for (int s = 0; s < 2; ++s) {
    memcpy(base + h.probs_off[s], probs[s].data(), probs[s].size() * sizeof(StageProb));
    memcpy(base + h.items_off[s], items[s].data(), items[s].size() * sizeof(WorkItem));
  }
  memcpy(base, &h, sizeof(h));
  return MDBF_OK;
}

int mdbf_forward_batch(const void* plan_host, const void* plan_dev, size_t plan_bytes, void* stream) {
  return mdbf_forward_batch_part(plan_host, plan_dev, plan_bytes, 3, 3, stream);
}

int mdbf_forward_batch_part(const void* plan_host, const void* plan_dev, size_t plan_bytes, int stages,
                            int kernels, void* stream) {
  if (!plan_host || !plan_dev) return MDBF_EINVAL;
  if (stages < 1 || stages > 3 || kernels < 1 || kernels > 3) return MDBF_EINVAL;
  if (!aligned16(plan_dev)) return MDBF_EALIGN;
  PlanHeader h;
  if (plan_bytes < sizeof(PlanHeader)) return MDBF_EWORKSPACE;
  memcpy(&h, plan_host, sizeof(h));
  if (h.magic != kPlanMagic || h.count < 1 || h.total_bytes > plan_bytes) return MDBF_EINVAL;
  const unsigned char* dev = (const unsigned char*)plan_dev;
  hipStream_t s = (hipStream_t)stream;
  if (h.gemm && h.max_tokens > gemm_plan_max_tokens()) {
    // long problems: each fills the device by itself; one launch per problem and stage, from the host copy
    const unsigned char* host = (const unsigned char*)plan_host;
    for (int i = 0; i < h.count; ++i)
      for (int st = 0; st < 2; ++st) {
        if (!(stages & (1 << st)) || !(kernels & 2)) continue;
        StageProb one;   // plan_host may have any alignment
        memcpy(&one, host + h.probs_off[st] + (size_t)i * sizeof(StageProb), sizeof(one));
        int e = launch_stage_gemm(nullptr, 0, 0, &one, s);
        if (e) return hip_fail(e);
      }
    return MDBF_OK;
  }
  if (h.gemm) {
    for (int st = 0; st < 2; ++st) {
      if (!(stages & (1 << st)) || !(kernels & 2)) continue;
      StageProb launch;
      memset(&launch, 0, sizeof(launch));
      launch.T = h.max_tokens;
      int e = launch_stage_gemm((const WorkItem*)(dev + h.items_off[st]), h.nitems[st], h.gemm_mode[st], &launch, s);
      if (e) return hip_fail(e);
    }
    return MDBF_OK;
  }
  for (int st = 0; st < 2; ++st) {
    const StageProb* probs = (const StageProb*)(dev + h.probs_off[st]);
    const WorkItem* items = (const WorkItem*)(dev + h.items_off[st]);
    StageProb dummy;
    memset(&dummy, 0, sizeof(dummy));
    dummy.ntiles = h.tiles_per_item[st];
    if (!(stages & (1 << st))) continue;
    const bool pre_k = (kernels & 1) != 0, main_k = (kernels & 2) != 0;
    int e = 0;
    if (h.precise) {
      if (main_k) e = launch_stage_precise(probs, items, h.nitems[st], &dummy, s);
    } else if (h.mx[st]) {
      dummy.l = h.mx[st];
      // (fused plans: the first stage's product launch has written this stage's records)
      if (pre_k && !(st == 1 && h.fuse2)) e = launch_scale_in_mx(probs, h.count, h.max_units_mx[st], &dummy, s);
      if (e) return hip_fail(e);
      const StageProb* next = (st == 0 && h.fuse2) ? (const StageProb*)(dev + h.probs_off[1]) : nullptr;
      if (main_k) e = launch_stage_mx(items, h.nitems[st], &dummy, next, s);
    } else if (h.fast[st]) {
      if (h.pre[st] && pre_k) e = launch_scale_in(probs, h.count, h.max_units[st], &dummy, s);
      if (e) return hip_fail(e);
      if (main_k) e = launch_stage_mfma(probs, items, h.nitems[st], h.tiles_per_item[st], &dummy, h.pre[st] != 0, s);
    } else if (main_k) {
      e = launch_stage_generic(probs, items, h.nitems[st], h.tiles_per_item[st], &dummy, s);
    }
    if (e) return hip_fail(e);
  }
  return MDBF_OK;
}

const char* mdbf_batch_plan_kernel(const void* plan_host, size_t plan_bytes, int stage) {
  if (!plan_host || plan_bytes < sizeof(PlanHeader) || stage < 1 || stage > 2) return "";
  PlanHeader h;
  memcpy(&h, plan_host, sizeof(h));
  if (h.magic != kPlanMagic) return "";
  const int st = stage - 1;
  if (h.precise) return "stage_precise_kernel";
  if (h.gemm) return "stage_gemm_kernel";
  if (h.mx[st]) return "stage_mx_kernel";
  if (h.fast[st]) return "stage_fast_kernel";
  return "stage_generic_kernel";
}

int mdbf_batch_plan_launches(const void* plan_host, size_t plan_bytes) {
  if (!plan_host || plan_bytes < sizeof(PlanHeader)) return MDBF_EINVAL;
  PlanHeader h;
  memcpy(&h, plan_host, sizeof(h));
  if (h.magic != kPlanMagic || h.count < 1) return MDBF_EINVAL;
  if (h.gemm) return h.max_tokens > gemm_plan_max_tokens() ? 2 * h.count : 2;
  if (h.precise) return 2;
  int n = 0;
  for (int st = 0; st < 2; ++st) {
    if (h.mx[st]) n += (st == 1 && h.fuse2) ? 1 : 2;
    else if (h.fast[st]) n += h.pre[st] ? 2 : 1;
    else n += 1;
  }
  return n;
}

int mdbf_msvid_block(int l) {
  if (l < 1 || l > MDBF_MAX_L) return MDBF_EINVAL;
  return msvid_block(l);
}

static int check_msvid_shape(int rows, int cols, int l) {
  if (rows <= 0 || cols <= 0 || l < 1 || l > MDBF_MAX_L) return MDBF_EINVAL;
  const int b = msvid_block(l);
  if (b > rows || b > cols) return MDBF_EUNSUPPORTED;
  return MDBF_OK;
}

int mdbf_msvid_workspace_bytes(int rows, int cols, int l, size_t* bytes_out) {
  if (!bytes_out) return MDBF_EINVAL;
  int st = check_msvid_shape(rows, cols, l);
  if (st) return st;
  *bytes_out = msvid_ws_bytes(rows, cols, l);
  return MDBF_OK;
}

int mdbf_msvid(const float* Z_dev, int rows, int cols, int64_t ld, int l, int iters, const float* X0_dev,
               int8_t* S_dev, float* A_dev, float* Q_dev, float* sigma_dev, void* workspace_dev,
               size_t workspace_bytes, void* stream) {
  int st = check_msvid_shape(rows, cols, l);
  if (st) return st;
  if (!Z_dev || !X0_dev || !S_dev || !A_dev || !Q_dev || !sigma_dev || !workspace_dev) return MDBF_EINVAL;
  if (ld < cols || iters < 0 || iters > 64) return MDBF_EINVAL;
  if (!aligned16(Z_dev) || !aligned16(X0_dev) || !aligned16(S_dev) || !aligned16(A_dev) || !aligned16(Q_dev) ||
      !aligned16(sigma_dev) || !aligned16(workspace_dev))
    return MDBF_EALIGN;
  if (workspace_bytes < msvid_ws_bytes(rows, cols, l)) return MDBF_EWORKSPACE;
  return hip_fail(launch_msvid(Z_dev, rows, cols, ld, l, iters, X0_dev, S_dev, A_dev, Q_dev, sigma_dev, workspace_dev,
                               (hipStream_t)stream));
}

const char* mdbf_strerror(int status) {
  switch (status) {
    case MDBF_OK: return "ok";
    case MDBF_EINVAL: return "invalid argument";
    case MDBF_EALIGN: return "device pointer not 16-byte aligned";
    case MDBF_EDTYPE: return "unknown dtype";
    case MDBF_EWORKSPACE: return "buffer too small";
    case MDBF_EUNSUPPORTED: return "unsupported request";
    case MDBF_EHIP: return "HIP call failed";
    default: return "unknown status";
  }
}

const char* mdbf_last_hip_error(void) { return g_hip_err; }

int mdbf_version(void) { return MDBF_VERSION; }

}  // extern "C"
