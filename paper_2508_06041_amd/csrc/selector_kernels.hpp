// Precision selector kernel (paper Sec. 3: the layer takes h when the relative error exceeds its threshold
// T, else l; Sec. 5.1: the error is estimated as ||G x|| with G = A (W_h - W_l) precomputed, or as
// alpha ||x|| + beta).  One launch serves a list of selector jobs, one workgroup (one compute unit) per
// job; the bitwidth lands in device memory, where the GEMV kernels read it.
//
// A job reads 0.5 - 3.5 MB of G; a workgroup of 16 wavefronts keeps enough loads in flight to pull that
// through one compute unit in about ten microseconds, and a decode step has about as many jobs as the chip
// has compute units, so no cross-workgroup reduction (atomics, fences, a second pass) is needed.
//
// The estimate and the compare are taken in fp64: fp16 x fp16 products are exact in fp32, their sum runs in
// fp64 in a fixed order, so a decision is reproducible and differs from an ideal-arithmetic decision only
// when |e - T| is below ~1e-13 relative.
#pragma once
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include <cstdint>

namespace dpllm {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;
constexpr int kSelRowsPerPass = 4;   // rows of G a wavefront carries at once (they share the activation loads)
constexpr int kSelMaxRank = 1024;

struct SelJob {
  const uint16_t* G;   // fp16 [r][in] (projection kind)
  const uint16_t* x;   // fp16 [in]
  float* e_out;
  int32_t* k_out;
  float T, alpha, beta;
  int32_t in, r, l, h, kind;  // kind: 0 none, 1 projection, 2 linear regression
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

__device__ __forceinline__ void accumulate8(const uint4& gv, const float (&xf)[8], double& acc) {
  const __half* gh = reinterpret_cast<const __half*>(&gv);
#pragma unroll
  for (int i = 0; i < 8; ++i) acc += (double)(__half2float(gh[i]) * xf[i]);  // product exact in fp32
}

__device__ __forceinline__ void selector_block(const SelJob& job, int tid) {
  __shared__ double g[kSelMaxRank];
  __shared__ double red[kSelWaves];
  const int wave = tid >> 6, lane = tid & 63;
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
    if (lane == 0) red[wave] = acc;
    __syncthreads();
    if (tid == 0) {
      double tot = 0.0;
      for (int w = 0; w < kSelWaves; ++w) tot += red[w];
      publish_decision((double)job.alpha * sqrt(tot) + (double)job.beta, job.T, job.l, job.h, job.e_out, job.k_out);
    }
    return;
  }
  // projection: wavefront w owns rows w, w + 16, ...; four of them per pass over the columns
  for (int j0 = wave; j0 < job.r; j0 += kSelWaves * kSelRowsPerPass) {
    const uint16_t* rows[kSelRowsPerPass];
#pragma unroll
    for (int i = 0; i < kSelRowsPerPass; ++i)
      rows[i] = job.G + (size_t)min(j0 + i * kSelWaves, job.r - 1) * job.in;
    double acc[kSelRowsPerPass];
#pragma unroll
    for (int i = 0; i < kSelRowsPerPass; ++i) acc[i] = 0.0;
    for (int c = lane * 8; c < job.in; c += 64 * 8) {
      uint4 xv = *reinterpret_cast<const uint4*>(job.x + c);
      typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
      uint4 gv[kSelRowsPerPass];
#pragma unroll
      for (int i = 0; i < kSelRowsPerPass; ++i) {
        u32x4_t t = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(rows[i] + c));
        gv[i] = make_uint4(t.x, t.y, t.z, t.w);
      }
      const __half* xh = reinterpret_cast<const __half*>(&xv);
      float xf[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) xf[i] = __half2float(xh[i]);
#pragma unroll
      for (int i = 0; i < kSelRowsPerPass; ++i) accumulate8(gv[i], xf, acc[i]);
    }
#pragma unroll
    for (int i = 0; i < kSelRowsPerPass; ++i) {
      double v = wave_sum_f64(acc[i]);
      int j = j0 + i * kSelWaves;
      if (lane == 0 && j < job.r) g[j] = v;
    }
  }
  __syncthreads();
  if (wave == 0) {
    double sq = 0.0;
    for (int j = lane; j < job.r; j += 64) sq += g[j] * g[j];
    sq = wave_sum_f64(sq);
    if (lane == 0) publish_decision(sqrt(sq), job.T, job.l, job.h, job.e_out, job.k_out);
  }
}

// jobs == nullptr: the single job passed by value; else workgroup b serves jobs[b]
__global__ void __launch_bounds__(kSelThreads) selector_kernel(const SelJob* __restrict__ jobs, SelJob one) {
  if (jobs == nullptr) {
    selector_block(one, threadIdx.x);
  } else {
    SelJob job = jobs[blockIdx.x];
    selector_block(job, threadIdx.x);
  }
}

}  // namespace dpllm
