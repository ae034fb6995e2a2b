// Sign bit-packing kernels: logical int8 (+-1, row-major)  <->  device tile layout.
// The layout is described in mdbf_internal.h.  Offline work, not tuned.
#include "mdbf_internal.h"

namespace mdbf {

// local column (0..127) addressed by bit b of the word of 8-column group kg
__device__ inline int local_col_of_bit(int b, int kg) {
  const int h = b >> 4, bb = b & 15;
  const int f = 2 * (bb >> 3) + ((bb >> 2) & 1), i = bb & 3;
  return f * 32 + kg * 8 + 2 * i + h;
}

__global__ void pack_kernel(const int8_t* __restrict__ signs, int rows, int cols, int64_t ld,
                            uint32_t* __restrict__ packed, int KB, size_t nwords) {
  size_t widx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (widx >= nwords) return;
  // enumerate words as (tile, q, lane) and place them through word_offset()
  const int lane = (int)(widx & 63);
  const size_t tq = widx >> 6;
  const int q = (int)(tq % (size_t)KB);
  const int tile = (int)(tq / (size_t)KB);
  const int r = lane & 15, kg = lane >> 4;
  const int row = tile * kTileRows + r;
  uint32_t w = 0;
  if (row < rows) {
    for (int b = 0; b < 32; ++b) {
      const int col = q * kBlockCols + local_col_of_bit(b, kg);
      if (col < cols && signs[(int64_t)row * ld + col] < 0) w |= (1u << b);
    }
  }
  packed[word_offset(tile, q, lane, KB, num_tiles(rows))] = w;
}

__global__ void unpack_kernel(const uint32_t* __restrict__ packed, int rows, int cols,
                              int8_t* __restrict__ signs, int64_t ld, int KB) {
  size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (size_t)rows * (size_t)cols) return;
  const int row = (int)(idx / (size_t)cols), col = (int)(idx % (size_t)cols);
  const int tile = row / kTileRows, r = row % kTileRows;
  const int q = col / kBlockCols, kl = col % kBlockCols;
  const int lane = kgroup_of_local_col(kl) * 16 + r;
  const uint32_t w = packed[word_offset(tile, q, lane, KB, num_tiles(rows))];
  signs[(int64_t)row * ld + col] = ((w >> bit_of_local_col(kl)) & 1u) ? (int8_t)-1 : (int8_t)1;
}

int launch_pack(const int8_t* signs, int rows, int cols, int64_t ld, uint32_t* packed, hipStream_t s) {
  const size_t nwords = packed_words(rows, cols);
  const int KB = num_blocks(cols);
  const unsigned grid = (unsigned)((nwords + 255) / 256);
  hipLaunchKernelGGL(pack_kernel, dim3(grid), dim3(256), 0, s, signs, rows, cols, ld, packed, KB, nwords);
  return (int)hipGetLastError();
}

int launch_unpack(const uint32_t* packed, int rows, int cols, int8_t* signs, int64_t ld, hipStream_t s) {
  const size_t n = (size_t)rows * (size_t)cols;
  const int KB = num_blocks(cols);
  const unsigned grid = (unsigned)((n + 255) / 256);
  hipLaunchKernelGGL(unpack_kernel, dim3(grid), dim3(256), 0, s, packed, rows, cols, signs, ld, KB);
  return (int)hipGetLastError();
}

// Envelope factor with zero modes appended: dst[r, c] = src[r, c] for c < l, 0 for l <= c < l_to.
// The product is unchanged (the extra modes contribute nothing); ranks 8 and 16 are the ones the matrix-core
// kernels take.  Elements are moved as raw bits: es = bytes per element (2 or 4).
__global__ __launch_bounds__(256) void pad_envelope_kernel(const unsigned char* __restrict__ src, int rows, int l,
                                                           unsigned char* __restrict__ dst, int l_to, int es) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= (size_t)rows * (size_t)l_to) return;
  const size_t r = i / (size_t)l_to;
  const int c = (int)(i - r * (size_t)l_to);
  if (es == 2) {
    ((MDBF_GLOBAL uint16_t*)dst)[i] = c < l ? ((const MDBF_GLOBAL uint16_t*)src)[r * (size_t)l + c] : (uint16_t)0;
  } else {
    ((MDBF_GLOBAL uint32_t*)dst)[i] = c < l ? ((const MDBF_GLOBAL uint32_t*)src)[r * (size_t)l + c] : 0u;
  }
}

int launch_pad_envelope(const void* src, int rows, int l, void* dst, int l_to, int es, hipStream_t s) {
  const size_t n = (size_t)rows * (size_t)l_to;
  hipLaunchKernelGGL(pad_envelope_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s,
                     (const unsigned char*)src, rows, l, (unsigned char*)dst, l_to, es);
  return (int)hipGetLastError();
}

// Plain streaming read: lane t of the launch reads the 16-byte elements t, t + lanes, t + 2 * lanes, ...
// (four independent loads per trip) and XORs them; every wave stores one word.
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(256) void stream_read_kernel(const u32x4_t* __restrict__ src, size_t n16,
                                                          uint32_t* __restrict__ sink) {
  const MDBF_GLOBAL u32x4_t* g = (const MDBF_GLOBAL u32x4_t*)src;
  const size_t lanes = (size_t)gridDim.x * 256;
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  u32x4_t a0 = {0, 0, 0, 0}, a1 = a0, a2 = a0, a3 = a0;
  for (; i + 3 * lanes < n16; i += 4 * lanes) {
    a0 ^= __builtin_nontemporal_load(g + i);
    a1 ^= __builtin_nontemporal_load(g + i + lanes);
    a2 ^= __builtin_nontemporal_load(g + i + 2 * lanes);
    a3 ^= __builtin_nontemporal_load(g + i + 3 * lanes);
  }
  for (; i < n16; i += lanes) a0 ^= __builtin_nontemporal_load(g + i);
  a0 ^= a1 ^ a2 ^ a3;
  uint32_t v = a0.x ^ a0.y ^ a0.z ^ a0.w;
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) v ^= (uint32_t)__shfl_xor((int)v, d);
  if ((threadIdx.x & 63) == 0) ((MDBF_GLOBAL uint32_t*)sink)[blockIdx.x * 4 + (threadIdx.x >> 6)] = v;
}

int launch_stream_read(const void* src, size_t bytes, uint32_t* sink, int sink_words, hipStream_t s) {
  hipLaunchKernelGGL(stream_read_kernel, dim3((unsigned)(sink_words / 4)), dim3(256), 0, s, (const u32x4_t*)src,
                     bytes / 16, sink);
  return (int)hipGetLastError();
}

}  // namespace mdbf
