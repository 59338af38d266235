// Load-time re-tiling, the parity read-back of codes, and the precision selector kernels.
#pragma once
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include <cstdint>

#include "layout_device.hpp"

namespace dpllm {

__device__ __forceinline__ uint32_t rotr32(uint32_t v, int s) { return __builtin_rotateright32(v, s); }

// canonical planes [p][out][ncw] -> device planes; one thread per (plane, row quad, column word)
__global__ void retile_planes_kernel(const uint32_t* __restrict__ canon, uint4* __restrict__ dev,
                                     int p, int out, int ncw, int nrq, size_t plane_stride_u4) {
  size_t per_plane = (size_t)nrq * ncw;
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= per_plane * p) return;
  int b = (int)(i / per_plane);
  size_t e = i % per_plane;
  int rq = (int)(e / ncw), cw = (int)(e % ncw);
  uint32_t w[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    int o = rq * 4 + r;
    uint32_t v = (o < out) ? canon[((size_t)b * out + o) * ncw + cw] : 0u;
    w[r] = rotr32(permute_word(v), b);
  }
  dev[(size_t)b * plane_stride_u4 + e] = make_uint4(w[0], w[1], w[2], w[3]);
}

// table [out][entries] -> [nrq*4][entries], zero rows appended
__global__ void copy_lut_kernel(const uint16_t* __restrict__ src, uint16_t* __restrict__ dst, int out,
                                int rows_padded, int entries) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t n = (size_t)rows_padded * entries;
  if (i >= n) return;
  size_t row = i / entries;
  dst[i] = (row < (size_t)out) ? src[i] : (uint16_t)0;
}

// device planes -> canonical k-bit codes uint8 [out][in]; one thread per (row, column word)
__global__ void debug_unpack_kernel(const uint4* __restrict__ dev, size_t plane_stride_u4, int p, int k,
                                    int out, int ncw, uint8_t* __restrict__ idx) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (size_t)out * ncw) return;
  int o = (int)(i / ncw), cw = (int)(i % ncw);
  int rq = o / 4, r = o % 4;
  uint32_t w[8];
  for (int b = 0; b < p; ++b) {
    uint4 v = dev[(size_t)b * plane_stride_u4 + (size_t)rq * ncw + cw];
    uint32_t s = r == 0 ? v.x : r == 1 ? v.y : r == 2 ? v.z : v.w;
    w[b] = unpermute_word((s << b) | (b ? (s >> (32 - b)) : 0u));  // undo rotation and permutation
  }
  for (int c = 0; c < 32; ++c) {
    uint32_t code = 0;
    for (int b = 0; b < p; ++b) code = (code << 1) | ((w[b] >> c) & 1u);
    idx[(size_t)o * ncw * 32 + (size_t)cw * 32 + c] = (uint8_t)(code >> (p - k));
  }
}

// ---------------------------------------------------------------------------------------------
// Precision selector (paper Sec. 3 rule, Sec. 5.1 estimators).  The estimate and the compare are
// taken in fp64 so that the decision does not depend on the summation order beyond ~1e-13.

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int s = 32; s >= 1; s >>= 1) v += __shfl_xor(v, s, 64);
  return v;
}

__device__ __forceinline__ void publish_decision(double e, float T, int l, int h, float* e_out,
                                                 int32_t* k_out) {
  *e_out = (float)e;
  *k_out = (e > (double)T) ? h : l;
}

constexpr int kSelThreads = 128;   // 2 waves, one 8-column vector per thread and pass
constexpr int kSelSplitCols = 1024;

// grid (nsplit, r): block (s, j) sums G[j][c] * x[c] over its column slice; the last block to
// finish adds the slices in a fixed order, takes the norm and decides.
__global__ void __launch_bounds__(kSelThreads)
selector_proj_kernel(const uint16_t* __restrict__ G, const uint16_t* __restrict__ x, int in, int r,
                     int nsplit, double* __restrict__ partial, unsigned* __restrict__ counter, float T,
                     int l, int h, float* __restrict__ e_out, int32_t* __restrict__ k_out) {
  __shared__ double red[kSelThreads / 64];
  __shared__ bool last;
  const int s = blockIdx.x, j = blockIdx.y, tid = threadIdx.x;
  const int c0 = s * kSelSplitCols;
  const int c1 = min(in, c0 + kSelSplitCols);
  double acc = 0.0;
  for (int c = c0 + tid * 8; c < c1; c += kSelThreads * 8) {
    uint4 gv = *reinterpret_cast<const uint4*>(G + (size_t)j * in + c);
    uint4 xv = *reinterpret_cast<const uint4*>(x + c);
    const __half* gh = reinterpret_cast<const __half*>(&gv);
    const __half* xh = reinterpret_cast<const __half*>(&xv);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      float prod = __half2float(gh[i]) * __half2float(xh[i]);  // exact: 11-bit x 11-bit significands
      acc += (double)prod;
    }
  }
  acc = wave_sum(acc);
  if ((tid & 63) == 0) red[tid >> 6] = acc;
  __syncthreads();
  if (tid == 0) {
    double tot = 0.0;
    for (int w = 0; w < kSelThreads / 64; ++w) tot += red[w];
    partial[(size_t)j * nsplit + s] = tot;
    __threadfence();
    unsigned done = atomicAdd(counter, 1u);
    last = (done == (unsigned)(nsplit * r) - 1u);
  }
  __syncthreads();
  if (!last) return;
  __threadfence();
  double sq = 0.0;
  for (int jj = tid; jj < r; jj += kSelThreads) {
    double g = 0.0;
    for (int ss = 0; ss < nsplit; ++ss) g += partial[(size_t)jj * nsplit + ss];
    sq += g * g;
  }
  sq = wave_sum(sq);
  __syncthreads();
  if ((tid & 63) == 0) red[tid >> 6] = sq;
  __syncthreads();
  if (tid == 0) {
    double tot = 0.0;
    for (int w = 0; w < kSelThreads / 64; ++w) tot += red[w];
    publish_decision(sqrt(tot), T, l, h, e_out, k_out);
    *counter = 0u;  // ready for the next launch on this stream
  }
}

// e = alpha * ||x|| + beta, one block
__global__ void __launch_bounds__(256)
selector_linreg_kernel(const uint16_t* __restrict__ x, int in, float alpha, float beta, float T, int l, int h,
                       float* __restrict__ e_out, int32_t* __restrict__ k_out) {
  __shared__ double red[4];
  const int tid = threadIdx.x;
  double acc = 0.0;
  for (int c = tid * 8; c < in; c += 256 * 8) {
    uint4 xv = *reinterpret_cast<const uint4*>(x + c);
    const __half* xh = reinterpret_cast<const __half*>(&xv);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      float v = __half2float(xh[i]);
      acc += (double)(v * v);
    }
  }
  acc = wave_sum(acc);
  if ((tid & 63) == 0) red[tid >> 6] = acc;
  __syncthreads();
  if (tid == 0) {
    double tot = red[0] + red[1] + red[2] + red[3];
    publish_decision((double)alpha * sqrt(tot) + (double)beta, T, l, h, e_out, k_out);
  }
}

__global__ void selector_fixed_kernel(int l, float* __restrict__ e_out, int32_t* __restrict__ k_out) {
  *e_out = 0.f;
  *k_out = l;
}

}  // namespace dpllm
