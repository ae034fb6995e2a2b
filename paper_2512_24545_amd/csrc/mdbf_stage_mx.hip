// Block-scaled (MX) matrix-core evaluation of one envelope-scaled binary product on gfx950.
//
//   out[r] = sum_c Eout[r,c] * P[r,c],     P[r,c] = sum_j S[r,j] * xs[j,c],   xs[j,c] = Ein[j,c] * vin[j]
//
// (paper Eq. "me-dbf-expand").  Same problem as the fp16 variant in mdbf_stage_mfma.hip, served by
// v_mfma_scale_f32_16x16x128_f8f6f4: one instruction contracts a whole 128-column block of a 16-row tile.
//
//  * A operand (signs) in fp4 (e2m1).  A lane's 32 sign bits of a block are one 32-bit word w; the four
//    operand registers are  w & 0x11111111, w & 0x22222222, w & 0x44444444, (w & 0x88888888) | 0x22222222 :
//    in the first three every nibble is 0 or the single-bit pattern of 0.5, 1, 2; in the fourth the bit is the
//    fp4 sign of a 1.0, i.e. the sign S itself.  Four vector operations expand 32 signs (the fp16 variant
//    needs 17).  With bit t = 1 meaning -1, S = 1 - 2t: over the first three registers' columns
//    P = colsum - 2 * sum t*xs; the fourth register's columns carry -xs/2, so that the same -2 * acc adds
//    their sum S*xs.
//  * B operand (activations) in three fp6 (e2m3) limbs with one power-of-two scale per lane and block
//    (32 values): xs' = L1*2^E + L2*2^(E-4) + L3*2^(E-8) to about 2^-13 of the block maximum, where
//    xs' = xs / {0.5,1,2,-2} undoes the value of the sign nibble.  Three MFMAs per tile and block, all into
//    one fp32 accumulator; the hardware applies the scales.
//  * The limbs are produced once per (problem, token) by mx_scale_in_kernel as a stream of 5120-byte block
//    records; the main kernel does no arithmetic on activations.
//  * colsum[c] = sum_j xs[j,c] over the columns of the first three operand registers is taken over the
//    quantised values by the scale-in kernel (exact in fp32 per element, one partial sum per block and
//    mode) and travels inside each block record.
//
// The main kernel is split by role.  A workgroup has eight contraction waves (eight row tiles each) and two
// loader waves.  The loaders move sign words, activation records and envelope rows from global memory
// straight into a ring of three LDS stages (global_load_lds: no registers, and no waiting on their own
// loads beyond the stage that is due) and run two stages ahead; the contraction waves read everything
// from LDS and issue no global loads in their loop, so a saturated memory pipeline stalls only the
// loaders.  One barrier per stage hands a filled stage to the contraction waves and a drained one back.
#include "mdbf_internal.h"

namespace mdbf {
namespace mx {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

typedef const MDBF_GLOBAL u32x4* g_u32x4_ptr;
typedef const MDBF_GLOBAL uint32_t* g_u32_ptr;
typedef const MDBF_GLOBAL uint16_t* g_u16_ptr;
typedef const MDBF_GLOBAL float* g_f32_ptr;

// ---- activation stream: one record per 128-column block
constexpr int kLimbBytes = 64 * 24;            // 1536: [64 lanes x 16 B][64 lanes x 8 B]
constexpr int kScaleOff = 3 * kLimbBytes;      // 4608: 64 x 4 B, scale bytes of the three limbs
constexpr int kColsumOff = kScaleOff + 256;    // 4864: 16 fp32 column sums of the block
constexpr int kBlockBytes = 5120;              // padded to a multiple of 1 KB (one loader instruction)

// ---- main kernel geometry.  R = row tiles per contraction wave: 8, or fewer when that leaves fewer unused
// tile slots (a factor of 166 row tiles is three items of 56 tiles, not 64 + 64 + 38)
constexpr int kComputeWaves = 8;
constexpr int kMaxR = 8;
constexpr int SB = 2;                                  // blocks per stage
constexpr int kStages = 3;                             // ring depth
constexpr int kStageXs = SB * kBlockBytes;
constexpr int kXsInstr = kStageXs / 1024;              // loader instructions (64 lanes x 16 B each)
constexpr int kLoaderWaves = 2;                        // a wave keeps at most 63 loads in flight
constexpr int kThreads = 64 * (kComputeWaves + kLoaderWaves);
template <int R>
struct Geo {
  static constexpr int kItemTiles = kComputeWaves * R;          // row tiles per work item
  static constexpr int kStageSigns = kItemTiles * SB * 256;     // [block][tile][64 words]
  static constexpr int kStageBytes = kStageXs + kStageSigns;
  static constexpr int kEoBytes = kItemTiles * kTileRows * 32;  // envelope rows of an item (fp16, 16 modes)
  static constexpr int kSignInstr = kStageSigns / 1024;
  static constexpr int kEoInstr = kEoBytes / 1024;
  static constexpr int kSmemBytes = kStages * kStageBytes;
  static constexpr int kZBytes = kItemTiles * kTileRows * 4;      // fused launches: the item's results, behind the ring
  static constexpr int kSignInstrPerBlock = kItemTiles / 4 / kLoaderWaves;   // per loader wave
  static_assert(kItemTiles % 4 == 0, "a loader instruction carries four whole tiles");
  static_assert(kEoBytes <= kStageBytes, "the envelope rows travel in a stage of their own");
  static_assert((160 * 1024) / kSmemBytes == 1, "one workgroup of this kernel per compute unit");
  static_assert(kXsInstr % kLoaderWaves == 0 && kSignInstr % kLoaderWaves == 0 && kEoInstr % kLoaderWaves == 0,
                "the loader waves split every stage evenly");
  static_assert(2 * (kXsInstr + kSignInstr) / kLoaderWaves <= 63, "two stages in flight must fit the counter");
};
constexpr int kWgsPerCu = 1;                           // workgroups of the main kernel a compute unit holds

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
  // The result must not share registers with the sources: with a destination inside the second source's
  // range the instruction gave wrong limbs (seen in a build whose register allocation produced that
  // overlap; the compiler's builtin does not exclude it).  Hence the instruction is written out with an
  // early-clobber result; the idle cycle after it covers the wait a conversion's result may need before
  // an ordinary vector instruction reads it, which the compiler cannot add around opaque text.
  v6u out;
  asm("v_cvt_scalef32_2xpk16_fp6_f32 %0, %1, %2, %3\n\ts_nop 1" : "=&v"(out) : "v"(even), "v"(odd), "v"(scale));
  return out;
}

// the inverse (32 floats from one limb), with the same precaution
__device__ __forceinline__ v32f fp6_decode32(v6u limb, float scale) {
  v32f out;
  asm("v_cvt_scalef32_pk32_f32_fp6 %0, %1, %2\n\ts_nop 1" : "=&v"(out) : "v"(limb), "v"(scale));
  return out;
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
// scale-in kernel: one record per (problem, token, 128-column block); a wave builds `per_wave` consecutive
// records of a problem, fetching the inputs of the next one before it works on the current one.
//   1. the block's products Ein[k,c] * vin[k] (fp32; zero for k >= K) go to LDS, 128 x 16
//   2. lane (kg, n) gathers its 32 values in operand order, undoes the nibble values, takes the block
//      exponent E (largest magnitude <= 7.5 * 2^E) and peels three fp6 limbs at scales E, E-4, E-8;
//      every residual is exact in fp32
//   3. the block's column sums of the quantised values close the record
// ---------------------------------------------------------------------------------------------------
constexpr int kProdStride = 18;   // floats per LDS row: lane groups 8 rows apart land on disjoint banks
constexpr int kPrepWaves = 4;
constexpr int kPrepMaxPerWave = 4;

// inputs of one record as they come from memory: lane handles rows lane/2 + 32 i, modes 8 (lane & 1) .. + 7
struct PrepInput {
  u32x4 raw[4];      // eight envelope entries (fp16) per row
  uint32_t xbits[4]; // the row's activation: fp32 bits, or fp16 / bf16 bits in the low half
};

__device__ __forceinline__ PrepInput prep_load(const StageProb& p, int unit, int lane) {
  const int b = unit / p.KB, q = unit - b * p.KB;
  // rank 8: a row of the envelope factor is one 16-byte vector; the lanes of modes 8..15 read it too
  // and contribute zeros (the matrix-core tile is 16 modes wide whatever the rank)
  const int hl = p.l >> 3;                    // 16-byte vectors per envelope row: 2 or 1
  const bool has_modes = (lane & 1) < hl;
  const int64_t xrow = (int64_t)b * p.vin_ld;
  PrepInput in;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int kc = min(q * kBlockCols + (lane >> 1) + 32 * i, p.K - 1);
    in.raw[i] = ((g_u32x4_ptr)p.Ein)[(size_t)kc * hl + (has_modes ? (lane & 1) : 0)];
    in.xbits[i] = (p.vin_dt == MDBF_F32) ? ((g_u32_ptr)p.vin)[xrow + kc] : (uint32_t)((g_u16_ptr)p.vin)[xrow + kc];
  }
  return in;
}

// all lanes of the wave have finished their LDS accesses issued so far (a wave's LDS operations execute in
// order: this only keeps the compiler from moving accesses across)
__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// one 16-, 8- or 4-byte piece of a record: to global memory with the non-temporal hint (the records are read
// once, by the product launch that follows; with plain stores the write-back of 40 to 55 MB of dirty lines
// runs into that launch: measured on the 336-layer workload, 257 -> 248 us per step with the hint), or to LDS
template <bool TO_LDS, class V>
__device__ __forceinline__ void record_store(unsigned char* base, int index, V v) {
  if constexpr (TO_LDS) ((MDBF_LDS V*)base)[index] = v;
  else __builtin_nontemporal_store(v, &((MDBF_GLOBAL V*)base)[index]);
}

// A lane's 32 values of a block in operand order (val, divided by their nibble values; m = their largest
// magnitude) -> block exponent, three fp6 limbs, the record's slots, scales and column sums at `blk`.
template <bool RANK8, bool TO_LDS>
__device__ __forceinline__ void quantise_store(const float (&val)[32], float m, int lane, unsigned char* blk) {
  constexpr bool rank8 = RANK8;   // the launch's rank: every problem of it has l = 8, or every one l = 16
  const int n = lane & 15;
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
  const v32f b1 = fp6_decode32(l1, sc1);
  float r[32];
#pragma unroll
  for (int j = 0; j < 32; ++j) r[j] = val[j] - b1[j];
  const v6u l2 = fp6_encode32(r, sc2);
  const v32f b2 = fp6_decode32(l2, sc2);
#pragma unroll
  for (int j = 0; j < 32; ++j) r[j] -= b2[j];
  const v6u l3 = fp6_encode32(r, sc3);
  const v32f b3 = fp6_decode32(l3, sc3);
  // quantised value = val - (last residual); back at the scale of xs, summed over the lane's columns
  float part = 0.f;
#pragma unroll
  for (int j = 0; j < 32; ++j) {
    const float inv = (j < 8) ? 0.5f : (j < 16 ? 1.f : 2.f);
    if (j < 24) part += (val[j] - (r[j] - b3[j])) * inv;   // the fourth register's columns need no fix-up
  }
  // record slots: rank 16: limbs 1, 2, 3 of mode n.  Rank 8: slot 0 = limb 1 (n < 8) or limb 2 (n >= 8) of
  // mode n & 7, slot 1 = limb 3 (n < 8) or zeros, slot 2 unused and not written; each lane's scale bytes
  // follow its slots.
  const bool upper = rank8 && n >= 8;
  v6u slot[3];
#pragma unroll
  for (int c = 0; c < 6; ++c) {
    slot[0][c] = upper ? l2[c] : l1[c];
    slot[1][c] = rank8 ? (upper ? 0u : l3[c]) : l2[c];
    slot[2][c] = l3[c];
  }
  const uint32_t e0 = (uint32_t)(upper ? E + 123 : E + 127);
  const uint32_t e1 = (uint32_t)(rank8 ? E + 119 : E + 123);
#pragma unroll
  for (int L = 0; L < 3; ++L) {
    if (L < 2 || !rank8) {
      u32x4 a;
      a.x = slot[L][0]; a.y = slot[L][1]; a.z = slot[L][2]; a.w = slot[L][3];
      u32x2 bpart;
      bpart.x = slot[L][4]; bpart.y = slot[L][5];
      record_store<TO_LDS>(blk + L * kLimbBytes, lane, a);
      record_store<TO_LDS>(blk + L * kLimbBytes + 64 * 16, lane, bpart);
    }
  }
  record_store<TO_LDS>(blk + kScaleOff, lane, e0 | (e1 << 8) | ((uint32_t)(E + 119) << 16));
  if (upper) part = 0.f;   // the column sum of a mode is stored once

  // ---- 3. column sums of the block
  part += __shfl_xor(part, 16);
  part += __shfl_xor(part, 32);
  if (lane < 16) record_store<TO_LDS>(blk + kColsumOff, lane, part);
}


// the record of block q of the problem's contraction dimension, from the inputs `in`, written to `blk`
template <bool RANK8, bool TO_LDS>
__device__ __forceinline__ void prep_record_to(const StageProb& p, int q, int lane, const PrepInput& in, float* pr,
                                               unsigned char* blk) {
  const int kg = lane >> 4, n = lane & 15;
  const bool has_modes = (lane & 1) < (p.l >> 3);

  // ---- 1. products
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const bool live = (q * kBlockCols + (lane >> 1) + 32 * i < p.K) && has_modes;
    const float xk = (p.vin_dt == MDBF_F32)   ? __builtin_bit_cast(float, in.xbits[i])
                     : (p.vin_dt == MDBF_F16) ? (float)__builtin_bit_cast(_Float16, (uint16_t)in.xbits[i])
                                              : __builtin_bit_cast(float, in.xbits[i] << 16);
    const uint32_t w[4] = {in.raw[i].x, in.raw[i].y, in.raw[i].z, in.raw[i].w};
    float* dst = pr + ((lane >> 1) + 32 * i) * kProdStride + (lane & 1) * 8;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const float lo = (float)__builtin_bit_cast(_Float16, (uint16_t)(w[t] & 0xFFFFu));
      const float hi = (float)__builtin_bit_cast(_Float16, (uint16_t)(w[t] >> 16));
      dst[2 * t] = live ? lo * xk : 0.f;
      dst[2 * t + 1] = live ? hi * xk : 0.f;
    }
  }
  wave_lds_sync();

  // ---- 2. gather in operand order, quantise.  Rank 8: lanes n and n + 8 both take mode n; the first
  //         keeps limbs 1 and 3, the second limb 2, so that two matrix-core instructions cover three limbs
  const int nsrc = RANK8 ? (n & 7) : n;
  float val[32];
  float m = 0.f;
#pragma unroll
  for (int j = 0; j < 32; ++j) {
    const float presc = (j < 8) ? 2.f : (j < 16 ? 1.f : (j < 24 ? 0.5f : -0.5f));   // undo the nibble values 0.5, 1, 2, -2
    val[j] = pr[(local_col_of_element(j, 0) + 8 * kg) * kProdStride + nsrc] * presc;
    m = fmaxf(m, fabsf(val[j]));
  }
  wave_lds_sync();   // the next record's products may overwrite the buffer
  quantise_store<RANK8, TO_LDS>(val, m, lane, blk);
}

// record of unit (token, block) of the problem's activation stream in global memory
template <bool RANK8>
__device__ __forceinline__ void prep_record(const StageProb& p, int unit, int lane, const PrepInput& in, float* pr) {
  const int b = unit / p.KB, q = unit - b * p.KB;
  unsigned char* blk = (unsigned char*)p.xs + ((size_t)b * p.KB + q) * (size_t)kBlockBytes;
  prep_record_to<RANK8, false>(p, q, lane, in, pr, blk);
}

template <bool RANK8>
__global__ __launch_bounds__(64 * kPrepWaves) void mx_scale_in_kernel(const StageProb* __restrict__ probs,
                                                                      StageProb single, int per_wave) {
  __shared__ __attribute__((aligned(16))) float prod[kPrepWaves][128 * kProdStride];
  StageProb p;
  if (probs) p = probs[blockIdx.y];
  else p = single;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int units = p.KB * p.T;                          // (token, block) pairs of the problem
  int unit = (blockIdx.x * kPrepWaves + wv) * per_wave;
  const int end = min(unit + per_wave, units);
  if (unit >= end) return;
  float* pr = prod[wv];
  PrepInput cur = prep_load(p, unit, lane);
  for (; unit < end; ++unit) {
    PrepInput next = cur;
    if (unit + 1 < end) next = prep_load(p, unit + 1, lane);
    prep_record<RANK8>(p, unit, lane, cur, pr);
    cur = next;
  }
}

// ---------------------------------------------------------------------------------------------------
// main kernel
// ---------------------------------------------------------------------------------------------------
// The constants of the fourth operand register, held in registers the optimiser cannot see through: the
// three-operand and-or instruction takes no literal constants on this target.
struct SignConsts {
  uint32_t sign_bits;   // 0x88888888, scalar register
  uint32_t ones;        // 0x22222222 (1.0 in every nibble), vector register
};
__device__ __forceinline__ SignConsts sign_consts() {
  SignConsts c;
  asm("s_mov_b32 %0, 0x88888888" : "=s"(c.sign_bits));
  asm("v_mov_b32 %0, 0x22222222" : "=v"(c.ones));
  return c;
}

__device__ __forceinline__ v8i sign_operand(uint32_t w, const SignConsts& k) {
  v8i r;
  r[0] = (int)(w & 0x11111111u);
  r[1] = (int)(w & 0x22222222u);
  r[2] = (int)(w & 0x44444444u);
  r[3] = (int)((w & k.sign_bits) | k.ones);
  r[4] = 0; r[5] = 0; r[6] = 0; r[7] = 0;
  return r;
}

__device__ __forceinline__ floatx4 mx_mfma(v8i a, v8i b, floatx4 c, int L, uint32_t sc) {
  // A: fp4 (format 4), scale 2^0; B: fp6 e2m3 (format 2), scale byte L of sc
  if (L == 0) return __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, b, c, 4, 2, 0, 0x7F7F7F7F, 0, (int)sc);
  if (L == 1) return __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, b, c, 4, 2, 0, 0x7F7F7F7F, 1, (int)sc);
  return __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, b, c, 4, 2, 0, 0x7F7F7F7F, 2, (int)sc);
}

__device__ __forceinline__ float row16_sum(float v) {
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, true));
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x4E, 0xF, 0xF, true));
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x141, 0xF, 0xF, true));
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x140, 0xF, 0xF, true));
  return v;
}

// What both roles need to know about a work item; every field is wave-uniform.
struct ItemInfo {
  const unsigned char* S;      // packed signs of the problem
  const unsigned char* xs;     // activation stream of the problem (token 0)
  const unsigned char* Eout;
  void* out;
  int64_t out_ld;
  int rows, KB, T, out_dt, flags;
  int tile0, ntl;
  // fused launches only: the next factor's input-side envelope rows (one per row of this problem), its
  // activation stream (written here) and its block count
  const unsigned char* Enext;
  unsigned char* xs_next;
  int KB_next;
};

template <bool BATCH, int R, bool FUSE>
__device__ __forceinline__ ItemInfo load_item(const WorkItem* __restrict__ items, const StageProb& single, int item,
                                              const StageProb* __restrict__ next_probs) {
  ItemInfo it;
  it.Enext = nullptr;
  it.xs_next = nullptr;
  it.KB_next = 0;
  if (BATCH) {
    const WorkItem& w = items[item];   // uniform address: scalar loads
    if (FUSE) {
      const StageProb& nx = next_probs[w.prob];
      it.Enext = (const unsigned char*)nx.Ein;
      it.xs_next = (unsigned char*)nx.xs;
      it.KB_next = nx.KB;
    }
    it.S = (const unsigned char*)w.p.S;
    it.xs = (const unsigned char*)w.p.xs;
    it.Eout = (const unsigned char*)w.p.Eout;
    it.out = w.p.out;
    it.out_ld = w.p.out_ld;
    it.rows = w.p.rows;
    it.KB = w.p.KB;
    it.T = w.p.T;
    it.out_dt = w.p.out_dt;
    it.flags = w.p.flags;
    it.tile0 = w.tile0;
    it.ntl = w.ntiles;
  } else {
    it.S = (const unsigned char*)single.S;
    it.xs = (const unsigned char*)single.xs;
    it.Eout = (const unsigned char*)single.Eout;
    it.out = single.out;
    it.out_ld = single.out_ld;
    it.rows = single.rows;
    it.KB = single.KB;
    it.T = single.T;
    it.out_dt = single.out_dt;
    it.flags = single.flags;
    it.tile0 = item * Geo<R>::kItemTiles;
    it.ntl = min(Geo<R>::kItemTiles, single.ntiles - it.tile0);
  }
  return it;
}

// one loader instruction: 64 lanes x 16 bytes from per-lane global addresses to 1 KB of LDS at `lds`.
// STREAM: data read once per launch (sign words, envelope rows) carries the non-temporal hint: measured on
// this chip, streaming reads reach about 7.2 TB/s with it and 6.0 - 6.3 TB/s without.
template <bool STREAM>
__device__ __forceinline__ void dma16(const unsigned char* gbase, uint32_t lane_off, unsigned char* lds) {
  constexpr int kNonTemporal = 2;   // cache-policy operand of the instruction: bit 1 = nt
  __builtin_amdgcn_global_load_lds((const MDBF_GLOBAL void*)(gbase + lane_off), (MDBF_LDS void*)lds, 16, 0,
                                   STREAM ? kNonTemporal : 0);
}

// Addresses of the sign-word instructions of loader wave LW (it takes every kLoaderWaves-th instruction):
// instruction 2 * jj + LW of a block carries tiles 4 * (2 * jj + LW) .. + 3 of the item, 16 bytes per lane;
// tiles past the item's end repeat its last tile.  An item may straddle the packed layout's groups of 64
// tiles, an instruction's four tiles never do (items start at multiples of four tiles): per instruction, one
// lane offset from the start of the packed matrix (block 0) and the byte distance between blocks, which is
// that of the instruction's group.  One set per item, so that an instruction costs no vector arithmetic.
template <int LW, int R>
__device__ __forceinline__ void sign_lane_offsets(const ItemInfo& it, int lane, uint32_t (&voff)[R],
                                                  uint32_t (&bstride)[R]) {
  const int ntiles = num_tiles(it.rows);
#pragma unroll
  for (int jj = 0; jj < R; ++jj) {
    const int a = jj * kLoaderWaves + LW;
    const int first = it.tile0 + min(4 * a, it.ntl - 1);                 // wave-uniform
    const int g0 = first & ~(kGroupTiles - 1);
    const int gt = min(kGroupTiles, ntiles - g0);
    const int tile = it.tile0 + min(4 * a + (lane >> 4), it.ntl - 1);    // in the group of `first`
    voff[jj] = ((uint32_t)g0 * (uint32_t)it.KB + (uint32_t)(tile - g0)) * 256u + (uint32_t)(lane & 15) * 16u;
    bstride[jj] = (uint32_t)gt * 256u;
  }
}

// loader wave LW: blocks [q0, q0 + SB) of the item's tiles and of token b's activation stream into `stage`
template <int LW, int R>
__device__ __forceinline__ void issue_stage(const ItemInfo& it, int b, int q0, unsigned char* stage, int lane,
                                            const uint32_t (&voff)[R], const uint32_t (&bstride)[R]) {
  typedef Geo<R> G;
  // activation records: each record is five instructions; a block past the end repeats the last one
#pragma unroll
  for (int j = 0; j < kXsInstr / kLoaderWaves; ++j) {
    constexpr int kPerRecord = kBlockBytes / 1024;
    const int i = j * kLoaderWaves + LW;
    const int blk = i / kPerRecord, part = i - blk * kPerRecord;
    const int q = min(q0 + blk, it.KB - 1);
    const unsigned char* src = it.xs + ((size_t)b * it.KB + q) * (size_t)kBlockBytes;
    dma16<false>(src + part * 1024, (uint32_t)lane * 16u, stage + i * 1024);
  }
  // sign words: in the packed layout the tiles of a group are contiguous per block (256 bytes per tile);
  // a block past the end repeats the last block
#pragma unroll
  for (int j = 0; j < G::kSignInstr / kLoaderWaves; ++j) {
    const int i = j * kLoaderWaves + LW;
    const int blk = i / (G::kItemTiles / 4);
    const int jj = j % G::kSignInstrPerBlock;
    // (one scalar multiplication and one vector addition per instruction; the whole offset fits 32 bits)
    const uint32_t qoff = (uint32_t)min(q0 + blk, it.KB - 1) * bstride[jj];
    dma16<true>(it.S, voff[jj] + qoff, stage + kStageXs + i * 1024);
  }
}

// loader: the item's envelope rows (RANK modes of fp16: 32 or 16 bytes per row, rows back to back) into
// `stage`.  With 16-byte rows the second half of the instructions repeats the last row past the item's end.
template <int RANK, int LW, int R>
__device__ __forceinline__ void issue_eo(const ItemInfo& it, const unsigned char* rows_base, unsigned char* stage, int lane) {
  constexpr int hsh = RANK >> 4;                // log2 of the 16-byte pieces per row: 1 or 0
#pragma unroll
  for (int j = 0; j < Geo<R>::kEoInstr / kLoaderWaves; ++j) {
    const int i = j * kLoaderWaves + LW;
    const int piece = 64 * i + lane;
    const int row = min(it.tile0 * kTileRows + (piece >> hsh), it.rows - 1);
    dma16<true>(rows_base, ((uint32_t)row << (4 + hsh)) + (uint32_t)(piece & hsh) * 16u, stage + i * 1024);
  }
}

// What a contraction wave reads from LDS for one 128-column block of a stage: the block's three limbs with
// their scales and column sum, and the sign words of the wave's R tiles.
template <int R>
struct BlockOperands {
  v8i limb[3];
  uint32_t scales;
  float colsum;
  uint32_t w[R];
};

// NL: record slots the matrix cores contract: 3 (rank 16), 2 (rank 8)
template <int NL, int R>
__device__ __forceinline__ BlockOperands<R> read_block(const unsigned char* stage, int blk, int lane, int n, int wave) {
  const unsigned char* rec = stage + blk * kBlockBytes;
  BlockOperands<R> o;
#pragma unroll
  for (int L = 0; L < NL; ++L) {
    const u32x4 a = reinterpret_cast<const u32x4*>(rec + L * kLimbBytes)[lane];
    const u32x2 c = reinterpret_cast<const u32x2*>(rec + L * kLimbBytes + 64 * 16)[lane];
    o.limb[L][0] = (int)a.x; o.limb[L][1] = (int)a.y; o.limb[L][2] = (int)a.z; o.limb[L][3] = (int)a.w;
    o.limb[L][4] = (int)c.x; o.limb[L][5] = (int)c.y; o.limb[L][6] = 0; o.limb[L][7] = 0;
  }
  o.scales = reinterpret_cast<const uint32_t*>(rec + kScaleOff)[lane];
  o.colsum = reinterpret_cast<const float*>(rec + kColsumOff)[n];
  const uint32_t* sw = reinterpret_cast<const uint32_t*>(stage + kStageXs) + blk * Geo<R>::kItemTiles * 64 + lane;
#pragma unroll
  for (int r = 0; r < R; ++r) o.w[r] = sw[(wave * R + r) * 64];
  return o;
}

// R tiles of this wave against the block's limbs.  Tiles past the item's end are contracted too (their
// sign words repeat the last tile's; the results are not stored): skipping them costs more registers and
// branches than it saves.
template <int NL, int R>
__device__ __forceinline__ void contract_block(const BlockOperands<R>& o, floatx4 (&acc)[R], float& colsum,
                                               const SignConsts& k) {
  colsum += o.colsum;
  // all tiles' sign operands first (4 R registers), limb outermost: consecutive instructions write different
  // accumulators
  v8i a[R];
#pragma unroll
  for (int r = 0; r < R; ++r) a[r] = sign_operand(o.w[r], k);
#pragma unroll
  for (int L = 0; L < NL; ++L) {
#pragma unroll
    for (int r = 0; r < R; ++r) acc[r] = mx_mfma(a[r], o.limb[L], acc[r], L, o.scales);
  }
}

// The loader role of wave LW of a workgroup: walks the workgroup's stage sequence (for every item, for
// every token, ceil(KB / SB) contraction stages followed by one stage with the envelope rows; stage g lives
// in ring slot g % kStages), two stages ahead of the contraction waves.  Barrier g opens stage g for them
// and tells the loader that stage g - 1 has been drained, so that its slot can take stage g + 2.
template <bool BATCH, int RANK, int LW, int R, bool FUSE>
__device__ __forceinline__ void loader_role(const WorkItem* __restrict__ items, const StageProb& single, int item0,
                                            int i_hi, int stride, unsigned char* smem, int lane,
                                            const StageProb* __restrict__ next_probs) {
  typedef Geo<R> G;
  int item = item0;
  ItemInfo it = load_item<BATCH, R, FUSE>(items, single, item, next_probs);
  uint32_t voff[R], bstride[R];
  sign_lane_offsets<LW, R>(it, lane, voff, bstride);
  int b = 0, t = 0;                       // cursor: next stage to issue = stage t of (item, b)
  int nst = (it.KB + SB - 1) / SB;        // contraction stages of the cursor's unit
  bool more = true;                       // the cursor points at an existing stage
  int slot = 0;                           // ring slot of the next stage to issue
  int kind_prev = 0;                      // kind of the newest issued stage: 0 contraction, 1 envelope rows
  auto issue_next = [&]() {
    unsigned char* stage = smem + slot * G::kStageBytes;
    if (t < nst) {
      issue_stage<LW, R>(it, b, t * SB, stage, lane, voff, bstride);
      kind_prev = 0;
    } else {
      // the output side's envelope rows, then (fused launches) the next factor's input-side rows
      issue_eo<RANK, LW, R>(it, t == nst ? it.Eout : it.Enext, stage, lane);
      kind_prev = 1;
    }
    slot = (slot + 1 == kStages) ? 0 : slot + 1;
    // advance the cursor
    if (t < nst + (FUSE ? 1 : 0)) {
      ++t;
    } else {
      t = 0;
      if (b + 1 < it.T) {
        ++b;
      } else {
        b = 0;
        item += stride;
        if (item < i_hi) {
          it = load_item<BATCH, R, FUSE>(items, single, item, next_probs);
          sign_lane_offsets<LW, R>(it, lane, voff, bstride);
          nst = (it.KB + SB - 1) / SB;
        } else {
          more = false;
        }
      }
    }
  };
  // prologue: stages 0 and 1 (every unit has at least two stages)
  issue_next();
  issue_next();
  int outstanding = 2;                    // issued stages not yet handed over
  for (;;) {
    // hand over the oldest outstanding stage: all but the newest stage's loads must have landed
    if (outstanding == 2) {
      if (kind_prev == 0) asm volatile("s_waitcnt vmcnt(%0)" ::"n"((kXsInstr + G::kSignInstr) / kLoaderWaves) : "memory");
      else asm volatile("s_waitcnt vmcnt(%0)" ::"n"(G::kEoInstr / kLoaderWaves) : "memory");
    } else {
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
    asm volatile("s_barrier" ::: "memory");
    --outstanding;
    if (more) {
      issue_next();
      ++outstanding;
    }
    if (outstanding == 0) break;
  }
}

// RANK: the envelope rank of every problem of the launch, 16 or 8.  The matrix-core tile is 16 columns wide
// either way; with rank 8, column n < 8 carries limbs 1 and 3 of mode n and column n + 8 limb 2 of the same
// mode (each column has its own scales), so a tile and block take two instructions instead of three; the
// sum over the 16 columns in the epilogue, with mode n's envelope entry on both of its columns, joins them.
// FUSE (plans whose next factor runs this kernel too): the launch also writes the next factor's activation
// records, so that factor needs no scale-in launch and the result of this one never travels through memory.
// Row r of this problem is column r of the next factor's contraction, an item starts at a multiple of eight
// row tiles, so its rows are whole 128-column blocks of that contraction: the item's results go to LDS, the
// next factor's envelope rows of the item arrive in one more ring stage, and wave w builds the record of the
// item's w-th block from the two with the arithmetic of the scale-in kernel (the same products, exponents and
// limbs: bit-identical records).
template <bool BATCH, int RANK, int R, bool FUSE>
__global__ __launch_bounds__(kThreads)
void stage_mx_kernel(const WorkItem* __restrict__ items, int nitems, StageProb single,
                     const StageProb* __restrict__ next_probs) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int kg = lane >> 4, n = lane & 15;

  // ---- this workgroup's items: a contiguous range per XCD, walked with the XCD's workgroup count
  int item0, i_hi, stride;
  if ((gridDim.x & 7) == 0) {
    const int xcd = blockIdx.x & 7;
    const int i_lo = (int)(((long)nitems * xcd) >> 3);
    i_hi = (int)(((long)nitems * (xcd + 1)) >> 3);
    stride = gridDim.x >> 3;
    item0 = i_lo + (blockIdx.x >> 3);
  } else {
    i_hi = nitems;
    stride = gridDim.x;
    item0 = blockIdx.x;
  }
  if (item0 >= i_hi) return;

  // both roles walk the same stage sequence (see loader_role); one barrier per stage
  if (wave >= kComputeWaves) {
    static_assert(kLoaderWaves == 2, "one instantiation of the loader role per loader wave");
    if (wave == kComputeWaves) loader_role<BATCH, RANK, 0, R, FUSE>(items, single, item0, i_hi, stride, smem, lane, next_probs);
    else loader_role<BATCH, RANK, 1, R, FUSE>(items, single, item0, i_hi, stride, smem, lane, next_probs);
    return;
  }

  // =========================== contraction waves ===========================
  const SignConsts sconst = sign_consts();
  float* zbuf = reinterpret_cast<float*>(smem + Geo<R>::kSmemBytes);   // (fused launches)
  int item = item0;
  ItemInfo it = load_item<BATCH, R, FUSE>(items, single, item, next_probs);
  int slot = 0;
  for (;;) {
    const int nr = max(0, min(R, it.ntl - wave * R));   // valid tiles of this wave (it owns tiles wave * R ..)
    for (int b = 0; b < it.T; ++b) {
      floatx4 acc[R];
#pragma unroll
      for (int r = 0; r < R; ++r) acc[r] = floatx4{0.f, 0.f, 0.f, 0.f};
      float colsum = 0.f;
      const int nst = (it.KB + SB - 1) / SB;
#pragma unroll 1
      for (int t = 0; t < nst; ++t) {
        __syncthreads();
        const unsigned char* stage = smem + slot * Geo<R>::kStageBytes;
        slot = (slot + 1 == kStages) ? 0 : slot + 1;
#pragma unroll
        for (int blk = 0; blk < SB; ++blk) {
          if (t * SB + blk < it.KB && nr > 0) {   // (a wave past the item's end only keeps the barriers)
            constexpr int kSlots = RANK == 8 ? 2 : 3;
            const BlockOperands<R> o = read_block<kSlots, R>(stage, blk, lane, n, wave);
            contract_block<kSlots, R>(o, acc, colsum, sconst);
          }
        }
      }
      // ---- envelope rows: fix-up, accumulate over the modes, store
      __syncthreads();
      {
        const _Float16* eoh = reinterpret_cast<const _Float16*>(smem + slot * Geo<R>::kStageBytes);
        slot = (slot + 1 == kStages) ? 0 : slot + 1;
#pragma unroll
        for (int r = 0; r < R; ++r) {
          if (r < nr) {
            const int trel = wave * R + r;
            float v[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              const float ev = (float)eoh[(trel * kTileRows + 4 * kg + i) * RANK + (n & (RANK - 1))];
              const float P = colsum - 2.f * acc[r][i];
              v[i] = row16_sum(ev * P);
            }
            const int sel = n & 3;
            const float res = sel == 0 ? v[0] : sel == 1 ? v[1] : sel == 2 ? v[2] : v[3];
            const int row = (it.tile0 + trel) * kTileRows + 4 * kg + n;
            if (FUSE) {
              if (n < 4) zbuf[trel * kTileRows + 4 * kg + n] = (row < it.rows) ? res : 0.f;
            } else {
              if (n < 4 && row < it.rows) emit_result(it.out, (int64_t)b * it.out_ld + row, it.out_dt, res, it.flags);
            }
          } else if (FUSE) {
            if (n < 4) zbuf[(wave * R + r) * kTileRows + 4 * kg + n] = 0.f;   // rows past the item's end
          }
        }
      }
      if (FUSE) {
        // ---- the next factor's records of this item's blocks (the barrier also publishes zbuf)
        __syncthreads();
        const _Float16* qh = reinterpret_cast<const _Float16*>(smem + slot * Geo<R>::kStageBytes);
        slot = (slot + 1 == kStages) ? 0 : slot + 1;
        const int nblk = (it.ntl * kTileRows + kBlockCols - 1) / kBlockCols;
        if (wave < nblk) {
          const int q2 = (it.tile0 * kTileRows) / kBlockCols + wave;
          const int nsrc = n & (RANK - 1);
          float val[32];
          float m = 0.f;
#pragma unroll
          for (int j = 0; j < 32; ++j) {
            const float presc = (j < 8) ? 2.f : (j < 16 ? 1.f : (j < 24 ? 0.5f : -0.5f));
            const int rowi = wave * kBlockCols + local_col_of_element(j, 0) + 8 * kg;   // row inside the item
            float prod;
            {
              // rounded to fp32 by itself, as the scale-in kernel leaves it in LDS (not fused into the
              // subtraction of the first limb that follows): the same records bit for bit
#pragma clang fp contract(off)
              prod = (float)qh[rowi * RANK + nsrc] * zbuf[rowi];
            }
            val[j] = prod * presc;
            m = fmaxf(m, fabsf(val[j]));
          }
          quantise_store<RANK == 8, false>(val, m, lane,
                                           it.xs_next + ((size_t)b * it.KB_next + q2) * (size_t)kBlockBytes);
        }
      }
    }
    item += stride;
    if (item >= i_hi) break;
    it = load_item<BATCH, R, FUSE>(items, single, item, next_probs);
  }
}

// ---------------------------------------------------------------------------------------------------
// Split variant for one small problem (a single layer, one token): 64-tile items would leave most of the
// device idle and a workgroup would walk the whole contraction dimension by itself.  Here workgroup (g, s)
// takes row tiles 8g .. 8g + 7 (one per wave) and blocks [s * bs, s * bs + bs) of the contraction
// dimension, builds the records of its blocks in LDS itself (no scale-in launch), contracts, applies the
// envelope rows and ends up with one partial sum per row: the envelope-accumulate of Eq. "me-dbf-expand"
// is linear in P, so 16 floats per tile leave the workgroup instead of 16 x 16.
//  * first factor: the partial sums go to part_out[s][row]; the second factor's workgroups add them up in
//    the order of s as they load their activations (vin = the sum), so no launch or wait lies between.
//  * second factor: the partial sums are written through to memory (device-scope stores) and a counter per
//    tile group is raised; whichever workgroup raises it to nsplit adds the nsplit partial sums of the
//    group's rows in the order of s and stores the result.  Nobody waits for anybody, and the order of the
//    additions is fixed: the result is the same bits every time.
// The counters are cleared by the first factor's launch of the same call.
// ---------------------------------------------------------------------------------------------------
constexpr int kSplitWaves = 8;      // row tiles per workgroup
constexpr int kSplitMaxBs = 4;      // blocks per workgroup at most (one record-building wave each)

// sum of count values `ld` floats apart, added in index order.  The loads go out eight at a time before the
// first addition (each one is a trip to memory: partial sums are never in this workgroup's caches).
// COHERENT: written by other workgroups of the same launch with device-scope stores; read the same way.
template <bool COHERENT>
__device__ __forceinline__ float ordered_sum(const MDBF_GLOBAL float* first, int count, int64_t ld) {
  float sum = 0.f;
  for (int t0 = 0; t0 < count; t0 += 8) {
    float v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const MDBF_GLOBAL float* src = first + (size_t)min(t0 + j, count - 1) * ld;
      v[j] = COHERENT ? __hip_atomic_load(src, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : *src;
    }
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if (t0 + j < count) sum += v[j];
  }
  return sum;
}

struct SplitArgs {
  StageProb p;
  int32_t bs, nsplit;               // blocks per workgroup; workgroups per tile group
  const float* part_in;             // vin[j] = sum over s < nsplit_in of part_in[s * part_in_ld + j]; null: p.vin
  int64_t part_in_ld;
  float* part_out;                  // [nsplit][part_out_ld] partial sums (unused when nsplit == 1)
  int64_t part_out_ld;
  uint32_t* counters;               // one per tile group: this launch finishes its rows itself; null: the reader adds
  uint32_t* clear;                  // counters to clear for the launch that follows (null: none)
  int32_t nsplit_in, nclear;
};

template <bool RANK8>
__global__ __launch_bounds__(64 * kSplitWaves) void stage_mx_split_kernel(SplitArgs a) {
  __shared__ __attribute__((aligned(16))) unsigned char recs[kSplitMaxBs * kBlockBytes];
  __shared__ __attribute__((aligned(16))) float prod[kSplitMaxBs][128 * kProdStride];
  __shared__ uint32_t is_last;
  constexpr int RANK = RANK8 ? 8 : 16;
  constexpr int NL = RANK8 ? 2 : 3;
  const StageProb& p = a.p;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int kg = lane >> 4, n = lane & 15;
  const int g = (int)blockIdx.x / a.nsplit, s = (int)blockIdx.x - g * a.nsplit;
  const int q0 = s * a.bs;
  const int nb = min(a.bs, p.KB - q0);                 // >= 1: nsplit = ceil(KB / bs)
  if (a.clear && blockIdx.x == 0)
    for (int i = tid; i < a.nclear; i += 64 * kSplitWaves)
      __hip_atomic_store((MDBF_GLOBAL uint32_t*)a.clear + i, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);

  // ---- this wave's tile: sign words of the workgroup's blocks and the envelope rows (issued first)
  const int tile = g * kSplitWaves + wave;
  const int tile_c = min(tile, p.ntiles - 1);
  uint32_t w[kSplitMaxBs];
#pragma unroll
  for (int i = 0; i < kSplitMaxBs; ++i)
    w[i] = ((g_u32_ptr)p.S)[word_offset(tile_c, min(q0 + i, p.KB - 1), lane, p.KB, p.ntiles)];
  _Float16 ev[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int row = min(tile_c * kTileRows + 4 * kg + i, p.rows - 1);
    ev[i] = ((const MDBF_GLOBAL _Float16*)p.Eout)[(size_t)row * RANK + (n & (RANK - 1))];
  }

  // ---- records of the workgroup's blocks: wave i builds block q0 + i
  if (wave < nb) {
    const int q = q0 + wave;
    PrepInput in = prep_load(p, q, lane);              // (token 0; with part_in the activations read here are not used)
    StageProb pp = p;
    if (a.part_in) {
      pp.vin_dt = MDBF_F32;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int kc = min(q * kBlockCols + (lane >> 1) + 32 * i, p.K - 1);
        const float sum = ordered_sum<false>((g_f32_ptr)a.part_in + kc, a.nsplit_in, a.part_in_ld);
        in.xbits[i] = __builtin_bit_cast(uint32_t, sum);
      }
    }
    prep_record_to<RANK8, true>(pp, q, lane, in, prod[wave], recs + wave * kBlockBytes);
  }
  __syncthreads();

  // ---- contraction of the tile against the records
  const SignConsts sconst = sign_consts();
  floatx4 acc = floatx4{0.f, 0.f, 0.f, 0.f};
  float colsum = 0.f;
#pragma unroll
  for (int i = 0; i < kSplitMaxBs; ++i) {
    if (i < nb) {
      const unsigned char* rec = recs + i * kBlockBytes;
      const uint32_t scales = reinterpret_cast<const uint32_t*>(rec + kScaleOff)[lane];
      colsum += reinterpret_cast<const float*>(rec + kColsumOff)[n];
      const v8i sa = sign_operand(w[i], sconst);
#pragma unroll
      for (int L = 0; L < NL; ++L) {
        const u32x4 x = reinterpret_cast<const u32x4*>(rec + L * kLimbBytes)[lane];
        const u32x2 y = reinterpret_cast<const u32x2*>(rec + L * kLimbBytes + 64 * 16)[lane];
        v8i limb;
        limb[0] = (int)x.x; limb[1] = (int)x.y; limb[2] = (int)x.z; limb[3] = (int)x.w;
        limb[4] = (int)y.x; limb[5] = (int)y.y; limb[6] = 0; limb[7] = 0;
        acc = mx_mfma(sa, limb, acc, L, scales);
      }
    }
  }

  // ---- envelope rows: fix-up, accumulate over the modes; one partial sum per row
  float v[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) v[i] = row16_sum((float)ev[i] * (colsum - 2.f * acc[i]));
  const int sel = n & 3;
  const float res = sel == 0 ? v[0] : sel == 1 ? v[1] : sel == 2 ? v[2] : v[3];
  const int row = tile * kTileRows + 4 * kg + n;
  const bool mine = n < 4 && tile < p.ntiles && row < p.rows;
  if (a.nsplit == 1) {
    if (mine) emit_result(p.out, row, p.out_dt, res, p.flags);
    return;
  }
  // read by another workgroup, possibly on another XCD: written through to memory
  if (mine)
    __hip_atomic_store((MDBF_GLOBAL float*)a.part_out + (size_t)s * a.part_out_ld + row, res, __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
  if (!a.counters) return;

  // ---- the last workgroup of the tile group adds the partial sums up
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");     // this wave's partial sums are in memory
  __syncthreads();
  if (tid == 0) {
    const uint32_t old = __hip_atomic_fetch_add((MDBF_GLOBAL uint32_t*)a.counters + g, 1u, __ATOMIC_RELAXED,
                                                __HIP_MEMORY_SCOPE_AGENT);
    is_last = (old + 1u == (uint32_t)a.nsplit) ? 1u : 0u;
  }
  __syncthreads();
  if (!is_last) return;
  const int frow = g * (kSplitWaves * kTileRows) + tid;
  if (tid < kSplitWaves * kTileRows && frow < p.rows) {
    const float sum = ordered_sum<true>((g_f32_ptr)a.part_out + frow, a.nsplit, a.part_out_ld);
    emit_result(p.out, frow, p.out_dt, sum, p.flags);
  }
}

static int max_workgroups() { return kWgsPerCu * compute_units(); }

template <bool BATCH, int RANK, int R, bool FUSE>
static int launch_brrf(const WorkItem* items_dev, int nitems, const StageProb* single, const StageProb* next_probs,
                       hipStream_t s) {
  constexpr int kSmem = Geo<R>::kSmemBytes + (FUSE ? Geo<R>::kZBytes : 0);
  static_assert(kSmem <= 160 * 1024, "ring and result buffer fit the LDS of a compute unit");
  static KernelSetup setup;
  if (int e = kernel_setup(setup, [] {
        return hipFuncSetAttribute(reinterpret_cast<const void*>(&stage_mx_kernel<BATCH, RANK, R, FUSE>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, kSmem);
      }))
    return e;
  const int max_wgs = max_workgroups();
  const int nwg = nitems < max_wgs ? nitems : max_wgs;
  hipLaunchKernelGGL((stage_mx_kernel<BATCH, RANK, R, FUSE>), dim3((unsigned)nwg), dim3(kThreads), kSmem, s, items_dev,
                     nitems, *single, next_probs);
  return (int)hipGetLastError();
}

template <bool BATCH, int RANK, int R>
static int launch_brr(const WorkItem* items_dev, int nitems, const StageProb* single, const StageProb* next_probs,
                      hipStream_t s) {
  if constexpr (BATCH) {
    if (next_probs) return launch_brrf<BATCH, RANK, R, true>(items_dev, nitems, single, next_probs, s);
  }
  return launch_brrf<BATCH, RANK, R, false>(items_dev, nitems, single, nullptr, s);
}

// item_tiles: row tiles per work item of the launch, 8 R
template <bool BATCH, int RANK>
static int launch_br(const WorkItem* items_dev, int nitems, int item_tiles, const StageProb* single,
                     const StageProb* next_probs, hipStream_t s) {
  switch (item_tiles) {
    case 64: return launch_brr<BATCH, RANK, 8>(items_dev, nitems, single, next_probs, s);
    case 56: return launch_brr<BATCH, RANK, 7>(items_dev, nitems, single, next_probs, s);
    case 48: return launch_brr<BATCH, RANK, 6>(items_dev, nitems, single, next_probs, s);
    default: return (int)hipErrorInvalidValue;
  }
}

template <bool BATCH>
static int launch_b(const WorkItem* items_dev, int nitems, int item_tiles, const StageProb* single,
                    const StageProb* next_probs, hipStream_t s) {
  if (single->l == 8) return launch_br<BATCH, 8>(items_dev, nitems, item_tiles, single, next_probs, s);
  return launch_br<BATCH, 16>(items_dev, nitems, item_tiles, single, next_probs, s);
}

}  // namespace mx

int launch_scale_in_mx(const StageProb* probs_dev, int count, int max_units, const StageProb* single, hipStream_t s) {
  // records per wave: as many as it takes for the launch to be resident at once (three workgroups per
  // compute unit: their registers), so that a wave's memory round trips overlap its own arithmetic
  const long resident = (long)compute_units() * 3 * mx::kPrepWaves;
  long per_wave = ((long)count * max_units + resident - 1) / resident;
  per_wave = per_wave < 1 ? 1 : per_wave > mx::kPrepMaxPerWave ? mx::kPrepMaxPerWave : per_wave;
  const int waves = (max_units + (int)per_wave - 1) / (int)per_wave;
  const int wgs = (waves + mx::kPrepWaves - 1) / mx::kPrepWaves;
  if (single->l == 8)
    hipLaunchKernelGGL(mx::mx_scale_in_kernel<true>, dim3((unsigned)wgs, (unsigned)count), dim3(64 * mx::kPrepWaves),
                       0, s, probs_dev, *single, (int)per_wave);
  else
    hipLaunchKernelGGL(mx::mx_scale_in_kernel<false>, dim3((unsigned)wgs, (unsigned)count), dim3(64 * mx::kPrepWaves),
                       0, s, probs_dev, *single, (int)per_wave);
  return (int)hipGetLastError();
}

size_t xs_bytes_for_mx(int K, int T) { return (size_t)T * (size_t)num_blocks(K) * (size_t)mx::kBlockBytes; }

int mx_item_tiles() { return mx::kComputeWaves * mx::kMaxR; }

// Row tiles per work item for a launch over problems of ntiles[i] row tiles and kb[i] column blocks: 64, or
// 56 or 48 where that takes less time by this model: an item costs its blocks times the bytes a block of
// it moves into LDS (a 5 KB record and 2 KB of sign words per tile row of eight), whatever part of its tile
// slots is used.  Ties go to the larger item.
int mx_pick_item_tiles(int count, const int* ntiles, const int* kb) {
  long best = -1;
  int best_r = mx::kMaxR;
  for (int r = mx::kMaxR; r >= 6; --r) {
    long cost = 0;
    for (int i = 0; i < count; ++i)
      cost += (long)((ntiles[i] + mx::kComputeWaves * r - 1) / (mx::kComputeWaves * r)) * kb[i] * (5 + 2 * r);
    if (best < 0 || cost < best) {
      best = cost;
      best_r = r;
    }
  }
  return mx::kComputeWaves * best_r;
}

int mx_max_workgroups() { return mx::max_workgroups(); }

bool stage_is_mx(const StageProb& p) {
  // the sign words must be addressable with 32-bit offsets from the start of the packed matrix
  return (p.l == 16 || p.l == 8) && p.env_dt == MDBF_F16 && p.KB >= 2 && p.xs != nullptr && p.T <= kMaxPreTokens &&
         packed_words(p.rows, p.K) * 4u < (1ull << 31);
}

int launch_stage_mx(const WorkItem* items_dev, int nitems, const StageProb* single, const StageProb* next_probs_dev,
                    hipStream_t s) {
  if (!items_dev) {
    const int item_tiles = mx_pick_item_tiles(1, &single->ntiles, &single->KB);
    nitems = (single->ntiles + item_tiles - 1) / item_tiles;
    return mx::launch_b<false>(nullptr, nitems, item_tiles, single, nullptr, s);
  }
  // single->ntiles carries the plan's tiles per item of this stage
  return mx::launch_b<true>(items_dev, nitems, single->ntiles, single, next_probs_dev, s);
}

SplitGeom split_geom(int ntiles, int KB) {
  // enough workgroups for a device of 256 compute units whatever the device: the workspace layout follows
  // from these numbers and must not depend on where it is computed
  constexpr int kTargetWgs = 256;
  SplitGeom g;
  g.ngroup = (ntiles + mx::kSplitWaves - 1) / mx::kSplitWaves;
  const int want = (kTargetWgs + g.ngroup - 1) / g.ngroup;
  int bs = (KB + want - 1) / want;
  // at most eight partial sums per row where the block limit allows: whoever adds them up fetches eight at a
  // time, and every further round is another trip to memory
  if (bs < (KB + 7) / 8) bs = (KB + 7) / 8;
  bs = bs < 1 ? 1 : bs > mx::kSplitMaxBs ? mx::kSplitMaxBs : bs;
  g.bs = bs;
  g.nsplit = (KB + bs - 1) / bs;
  return g;
}

bool stage_is_split(const StageProb& p) {
  return (p.l == 16 || p.l == 8) && p.env_dt == MDBF_F16 && p.T == 1 && p.KB >= 1 && p.ntiles >= 1;
}

int launch_stage_mx_split(const StageProb* p, const SplitGeom& g, const float* part_in, int nsplit_in,
                          int64_t part_in_ld, float* part_out, int64_t part_out_ld, uint32_t* counters,
                          uint32_t* clear, int nclear, hipStream_t s) {
  mx::SplitArgs a;
  a.p = *p;
  a.bs = g.bs;
  a.nsplit = g.nsplit;
  a.part_in = part_in;
  a.part_in_ld = part_in_ld;
  a.part_out = part_out;
  a.part_out_ld = part_out_ld;
  a.counters = counters;
  a.clear = clear;
  a.nsplit_in = nsplit_in;
  a.nclear = nclear;
  const dim3 grid((unsigned)(g.ngroup * g.nsplit)), block(64 * mx::kSplitWaves);
  if (p->l == 8) hipLaunchKernelGGL(mx::stage_mx_split_kernel<true>, grid, block, 0, s, a);
  else hipLaunchKernelGGL(mx::stage_mx_split_kernel<false>, grid, block, 0, s, a);
  return (int)hipGetLastError();
}

}  // namespace mdbf
