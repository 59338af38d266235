// Load-time re-tiling and the parity read-back of codes.
#pragma once
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include <cstdint>

#include "layout_device.hpp"

namespace dpllm {

__device__ __forceinline__ uint32_t rotr32(uint32_t v, int s) { return __builtin_rotateright32(v, s); }

// canonical planes [p][out][ncw] -> device planes; one thread per (plane, block of 64 rows, tile, row): it
// writes one 128-bit value (1 row x 4 words)
__global__ void retile_planes_kernel(const uint32_t* __restrict__ canon, uint4* __restrict__ dev,
                                     int p, int out, int ncw, int ncc, int nrq, size_t plane_stride_u4) {
  const size_t per_plane = (size_t)nrq * ncc * 64;
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= per_plane * p) return;
  int b = (int)(i / per_plane);
  size_t e = i % per_plane;
  uint32_t w[4];
  const int o = (int)(e / ((size_t)ncc * 64)) * 64 + (int)(e % 64), cc = (int)(e / 64 % ncc);
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int cw = cc * 4 + j;
    uint32_t v = (o < out && cw < ncw) ? canon[((size_t)b * out + o) * ncw + cw] : 0u;
    w[j] = rotr32(permute_word(v), b);
  }
  dev[(size_t)b * plane_stride_u4 + e] = make_uint4(w[0], w[1], w[2], w[3]);
}

// table [out][entries] -> [rows_padded][entries], zero rows appended
__global__ void copy_lut_kernel(const uint16_t* __restrict__ src, uint16_t* __restrict__ dst, int out,
                                int rows_padded, int entries) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t n = (size_t)rows_padded * entries;
  if (i >= n) return;
  size_t row = i / entries;
  dst[i] = (row < (size_t)out) ? src[i] : (uint16_t)0;
}

// device planes -> canonical k-bit codes uint8 [out][in]; one thread per (row, column word)
__global__ void debug_unpack_kernel(const uint32_t* __restrict__ dev, size_t plane_stride_u32, int p, int k,
                                    int out, int ncw, int ncc, uint8_t* __restrict__ idx) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (size_t)out * ncw) return;
  int o = (int)(i / ncw), cw = (int)(i % ncw);
  uint32_t w[8];
  for (int b = 0; b < p; ++b) {
    uint32_t s = dev[(size_t)b * plane_stride_u32 + plane_word_index(o, cw, ncc)];
    w[b] = unpermute_word((s << b) | (b ? (s >> (32 - b)) : 0u));  // undo rotation and permutation
  }
  for (int c = 0; c < 32; ++c) {
    uint32_t code = 0;
    for (int b = 0; b < p; ++b) code = (code << 1) | ((w[b] >> c) & 1u);
    idx[(size_t)o * ncw * 32 + (size_t)cw * 32 + c] = (uint8_t)(code >> (p - k));
  }
}

// n 32-bit words = v: clears counters and sets the target word (a kernel, not a memset node, so that a caller may
// capture it in a graph)
__global__ void fill_u32_kernel(uint32_t* __restrict__ dst, size_t n, uint32_t v) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = v;
}

// plain 128-bit copy of a known size: the yardstick the HBM byte counters are scaled by
__global__ void __launch_bounds__(256) plain_copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) dst[i] = src[i];
}

// plain non-temporal 128-bit streaming read of a known size: the measured ceiling the GEMV rates are compared
// with (launched with 8 workgroups per compute unit and one load in flight per lane, the fastest of the
// configurations tried: more requests in flight lower the rate).  The sink is written only for one improbable
// value of the running XOR, which keeps the loads alive.
__global__ void __launch_bounds__(256) plain_read_kernel(const uint4* __restrict__ src, size_t n, uint4* __restrict__ sink) {
  typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
  const u32x4_t* p = reinterpret_cast<const u32x4_t*>(src);
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  u32x4_t acc = {0u, 0u, 0u, 0u};
#pragma unroll 1
  for (; i < n; i += stride) acc ^= __builtin_nontemporal_load(p + i);
  if (acc.x == 0x12345678u && acc.y == 0x9abcdef0u && acc.z == 0x0f1e2d3cu) *sink = make_uint4(acc.x, acc.y, acc.z, acc.w);
}

}  // namespace dpllm
