// Precision selector kernels (paper Sec. 3: the layer takes h when the relative error exceeds its threshold
// T, else l; Sec. 5.1: the error is estimated as ||G x|| with G = A (W_h - W_l) precomputed, or as
// alpha ||x|| + beta).  One launch serves a list of selector jobs; the bitwidth lands in device memory,
// where the GEMV kernels read it.
//
// The estimate and the compare are taken in fp64: fp16 x fp16 products are exact in fp32, their sum runs in
// fp64, and the order of the final sums is fixed, so a decision is reproducible and differs from an
// ideal-arithmetic decision only when |e - T| is below ~1e-13 relative.
#pragma once
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include <cstdint>

namespace dpllm {

constexpr int kSelThreads = 128;     // 2 wavefronts; one 8-column vector per thread
constexpr int kSelSplitCols = 1024;  // columns per block
constexpr int kSelRows = 8;          // rows of G per block (the activation slice is loaded once for them)

struct SelJob {
  const uint16_t* G;   // fp16 [r][in] (projection kind)
  const uint16_t* x;   // fp16 [in]
  double* partial;     // workspace [r][nsplit]
  unsigned* counter;   // workspace, zero between launches
  float* e_out;
  int32_t* k_out;
  float T, alpha, beta;
  int32_t in, r, nsplit, l, h, kind;  // kind: 0 none, 1 projection, 2 linear regression
  int32_t nblocks;
  int32_t block_start;
};

__device__ __forceinline__ double wave_sum_f64(double v) {
#pragma unroll
  for (int s = 32; s >= 1; s >>= 1) v += __shfl_xor(v, s, 64);
  return v;
}

__device__ __forceinline__ void publish_decision(double e, float T, int l, int h, float* e_out, int32_t* k_out) {
  *e_out = (float)e;
  *k_out = (e > (double)T) ? h : l;  // strictly exceeding T selects h; +inf pins l, -inf pins h
}

__host__ __device__ inline int sel_job_blocks(int kind, int in, int r) {
  if (kind != 1) return 1;
  int nsplit = (in + kSelSplitCols - 1) / kSelSplitCols;
  return nsplit * ((r + kSelRows - 1) / kSelRows);
}

__device__ __forceinline__ void selector_block(const SelJob& job, int lb, int tid) {
  __shared__ double red[kSelThreads / 64][kSelRows];
  __shared__ bool last;
  if (job.kind == 0) {
    if (tid == 0) { *job.e_out = 0.f; *job.k_out = job.l; }
    return;
  }
  if (job.kind == 2) {
    double acc = 0.0;
    for (int c = tid * 8; c < job.in; c += kSelThreads * 8) {
      uint4 xv = *reinterpret_cast<const uint4*>(job.x + c);
      const __half* xh = reinterpret_cast<const __half*>(&xv);
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        float v = __half2float(xh[i]);
        acc += (double)(v * v);  // exact square in fp32
      }
    }
    acc = wave_sum_f64(acc);
    if ((tid & 63) == 0) red[tid >> 6][0] = acc;
    __syncthreads();
    if (tid == 0) {
      double tot = 0.0;
      for (int w = 0; w < kSelThreads / 64; ++w) tot += red[w][0];
      publish_decision((double)job.alpha * sqrt(tot) + (double)job.beta, job.T, job.l, job.h, job.e_out, job.k_out);
    }
    return;
  }
  // projection: block (s, g) sums rows 8g..8g+7 of G over columns [1024 s, 1024 s + 1024)
  const int s = lb % job.nsplit, g = lb / job.nsplit;
  const int j0 = g * kSelRows;
  const int c = s * kSelSplitCols + tid * 8;
  double acc[kSelRows];
#pragma unroll
  for (int i = 0; i < kSelRows; ++i) acc[i] = 0.0;
  if (c < job.in) {
    uint4 xv = *reinterpret_cast<const uint4*>(job.x + c);
    const __half* xh = reinterpret_cast<const __half*>(&xv);
    float xf[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) xf[i] = __half2float(xh[i]);
    uint4 gv[kSelRows];
#pragma unroll
    for (int rr = 0; rr < kSelRows; ++rr) {
      int j = min(j0 + rr, job.r - 1);
      gv[rr] = *reinterpret_cast<const uint4*>(job.G + (size_t)j * job.in + c);
    }
#pragma unroll
    for (int rr = 0; rr < kSelRows; ++rr) {
      const __half* gh = reinterpret_cast<const __half*>(&gv[rr]);
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[rr] += (double)(__half2float(gh[i]) * xf[i]);  // product exact in fp32
    }
  }
#pragma unroll
  for (int rr = 0; rr < kSelRows; ++rr) {
    double v = wave_sum_f64(acc[rr]);
    if ((tid & 63) == 0) red[tid >> 6][rr] = v;
  }
  __syncthreads();
  if (tid < kSelRows && j0 + tid < job.r) {
    double tot = 0.0;
    for (int w = 0; w < kSelThreads / 64; ++w) tot += red[w][tid];
    job.partial[(size_t)(j0 + tid) * job.nsplit + s] = tot;
  }
  __threadfence();
  __syncthreads();
  if (tid == 0) {
    unsigned done = atomicAdd(job.counter, 1u);
    last = (done == (unsigned)job.nblocks - 1u);
  }
  __syncthreads();
  if (!last) return;
  __threadfence();
  // the last block to arrive adds the slices in a fixed order, takes the norm and decides
  double sq = 0.0;
  for (int jj = tid; jj < job.r; jj += kSelThreads) {
    double gsum = 0.0;
    for (int ss = 0; ss < job.nsplit; ++ss) gsum += job.partial[(size_t)jj * job.nsplit + ss];
    sq += gsum * gsum;
  }
  sq = wave_sum_f64(sq);
  __syncthreads();
  if ((tid & 63) == 0) red[tid >> 6][0] = sq;
  __syncthreads();
  if (tid == 0) {
    double tot = 0.0;
    for (int w = 0; w < kSelThreads / 64; ++w) tot += red[w][0];
    publish_decision(sqrt(tot), job.T, job.l, job.h, job.e_out, job.k_out);
    *job.counter = 0u;  // ready for the next launch
  }
}

// jobs == nullptr: the single job passed by value; else block b belongs to the last job with block_start <= b
__global__ void __launch_bounds__(kSelThreads) selector_kernel(const SelJob* __restrict__ jobs, int njobs, SelJob one) {
  if (jobs == nullptr) {
    selector_block(one, blockIdx.x, threadIdx.x);
    return;
  }
  const int b = blockIdx.x;
  int lo = 0, hi = njobs - 1;
  while (lo < hi) {
    int mid = (lo + hi + 1) >> 1;
    if (jobs[mid].block_start <= b) lo = mid; else hi = mid - 1;
  }
  SelJob job = jobs[lo];
  selector_block(job, b - job.block_start, threadIdx.x);
}

}  // namespace dpllm
