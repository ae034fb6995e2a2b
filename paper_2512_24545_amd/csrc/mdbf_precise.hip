// fp32 vector-ALU evaluation of one envelope-scaled binary product (MDBF_FLAG_PRECISE).
// One wavefront per 16-row tile; lane = (row r, 8-column group kg) as in the packed layout.
// Per lane: acc[c] += (+-1) * Ein[j,c] * vin[j] over its columns, then the four kg lanes of a
// row are summed, and out[r] = sum_c Eout[r,c] * acc[c]   (paper Eq. "me-dbf-expand").
#include "mdbf_internal.h"

namespace mdbf {

__device__ inline int local_col_of_bit_p(int b, int kg) {
  const int h = b >> 4, bb = b & 15;
  const int f = 2 * (bb >> 3) + ((bb >> 2) & 1), i = bb & 3;
  return f * 32 + kg * 8 + 2 * i + h;
}

__global__ __launch_bounds__(64) void stage_precise_kernel(const StageProb* __restrict__ probs,
                                                           const WorkItem* __restrict__ items,
                                                           StageProb single) {
  int tile;
  const StageProb* pp;
  if (probs) {
    // in batch mode every work item is expanded to one block per tile by the launcher
    const WorkItem& it = items[blockIdx.y];
    if ((int)blockIdx.x >= it.ntiles) return;
    pp = &probs[it.prob];
    tile = it.tile0 + blockIdx.x;
  } else {
    pp = &single;
    tile = blockIdx.x;
  }
  const StageProb p = *pp;
  const int lane = threadIdx.x, r = lane & 15, kg = lane >> 4;
  const int row = tile * kTileRows + r;
  for (int b = 0; b < p.T; ++b) {
    float acc[MDBF_MAX_L];
#pragma unroll
    for (int c = 0; c < MDBF_MAX_L; ++c) acc[c] = 0.f;
    for (int q = 0; q < p.KB; ++q) {
      const uint32_t w = ((const MDBF_GLOBAL uint32_t*)p.S)[word_offset(tile, q, lane, p.KB, p.ntiles)];
      for (int bit = 0; bit < 32; ++bit) {
        const int col = q * kBlockCols + local_col_of_bit_p(bit, kg);
        if (col >= p.K) continue;
        const float v = load_as_float(p.vin, (int64_t)b * p.vin_ld + col, p.vin_dt);
        const float sv = ((w >> bit) & 1u) ? -v : v;
#pragma unroll
        for (int c = 0; c < MDBF_MAX_L; ++c)
          if (c < p.l) acc[c] += sv * load_as_float(p.Ein, (int64_t)col * p.l + c, p.env_dt);
      }
    }
    float o = 0.f;
#pragma unroll
    for (int c = 0; c < MDBF_MAX_L; ++c) {
      float a = acc[c];
      a += __shfl_xor(a, 16);
      a += __shfl_xor(a, 32);
      if (c < p.l && row < p.rows) o += a * load_as_float(p.Eout, (int64_t)row * p.l + c, p.env_dt);
    }
    if (kg == 0 && row < p.rows) emit_result(p.out, (int64_t)b * p.out_ld + row, p.out_dt, o, p.flags);
  }
}

int launch_stage_precise(const StageProb* probs_dev, const WorkItem* items_dev, int nitems,
                         const StageProb* single, hipStream_t s) {
  if (probs_dev) {
    // grid.x = upper bound of tiles per item is passed through single->ntiles by the caller
    hipLaunchKernelGGL(stage_precise_kernel, dim3((unsigned)single->ntiles, (unsigned)nitems), dim3(64), 0, s,
                       probs_dev, items_dev, *single);
  } else {
    hipLaunchKernelGGL(stage_precise_kernel, dim3((unsigned)single->ntiles), dim3(64), 0, s,
                       (const StageProb*)nullptr, (const WorkItem*)nullptr, *single);
  }
  return (int)hipGetLastError();
}

}  // namespace mdbf
