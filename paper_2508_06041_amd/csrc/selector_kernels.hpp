// Precision selector kernels (paper Sec. 3: the layer takes h when the relative error exceeds its threshold
// T, else l; Sec. 5.1: the error is estimated as ||G x|| with G = A (W_h - W_l) precomputed, or as
// alpha ||x|| + beta).  One launch serves a list of selector jobs; the bitwidth lands in device memory, where
// the GEMV kernels read it.
//
// A job reads 0.5 - 3.5 MB of G.  It is cut into parts of 16 rows of G (one workgroup of four wavefronts,
// four rows per wavefront sharing the activation loads) by a chunk of columns: the whole row when the launch
// has enough parts to fill the chip, down to 512 columns when it serves a few linears only (a part that
// streams a whole row alone takes 10 - 30 us).  A part leaves the fp64 partial dot products of its rows in
// workspace slots of its own and takes a ticket from the job's counter; the part that draws the last ticket
// adds the partial products of every row in chunk order, squares, adds the rows in index order, takes the
// square root and the decision, and leaves the counter at zero for the next launch.  The order of all
// additions is fixed whichever part comes last.  (A separate kernel for this last step would cost a dependent
// launch per group of linears that run together.)
//
// The estimate and the compare are taken in fp64: fp16 x fp16 products are exact in fp32, their sum runs in
// fp64 in a fixed order, so a decision is reproducible and differs from an ideal-arithmetic decision only
// when |e - T| is below ~1e-13 relative.
#pragma once
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include <cstdint>

namespace dpllm {

constexpr int kSelPartThreads = 256;
constexpr int kSelPartWaves = kSelPartThreads / 64;
constexpr int kSelRowsPerWave = 4;   // rows of G a wavefront carries at once (they share the activation loads)
constexpr int kSelDepth = 2;         // column tiles in registers: one being accumulated, one in flight
constexpr int kSelPartRows = kSelPartWaves * kSelRowsPerWave;
constexpr int kSelMaxRank = 1024;
constexpr int kSelMaxChunks = 32;    // column chunks of a job
constexpr int kSelChunkStep = 512;   // columns a wavefront covers per tile: chunks are multiples of it

struct SelJob {
  const uint16_t* G;   // fp16 [r][in] (projection kind)
  const uint16_t* x;   // fp16 [in]
  float* e_out;
  int32_t* k_out;
  double* ws;          // projection: [nchunks][16 rowgroups] partial dot products; else one slot
  uint32_t* ticket;    // arrival counter of this job, zero between launches
  float T, alpha, beta;
  int32_t in, r, l, h, kind;  // kind: 0 none, 1 projection, 2 linear regression
  int32_t nparts;             // projection: rowgroups * nchunks; linear regression: 1; none: 1 (only the decision)
  int32_t nchunks, chunk_cols;  // projection: part p covers rows [16 (p / nchunks), + 16), columns [chunk_cols (p % nchunks), + chunk_cols)
};
struct SelPart {
  int32_t job;    // index into the job table of the launch
  int32_t part;   // part number inside the job: rows [16 part, 16 part + 16)
};

__host__ __device__ inline int sel_rowgroups_of(int kind, int r) {
  return kind == 1 ? (r + kSelPartRows - 1) / kSelPartRows : 1;
}
// workspace slots (doubles) of a job
__host__ __device__ inline int sel_slots_of(int kind, int r, int nchunks) {
  return kind == 1 ? sel_rowgroups_of(kind, r) * kSelPartRows * nchunks : 1;
}

__device__ __forceinline__ double wave_sum_f64(double v) {
#pragma unroll
  for (int s = 32; s >= 1; s >>= 1) v += __shfl_xor(v, s, 64);
  return v;
}

typedef uint32_t sel_u32x4 __attribute__((ext_vector_type(4)));

struct SelTile {
  sel_u32x4 g[kSelRowsPerWave];
  uint4 x;
};

// columns [c, c + 8) of the wavefront's four rows and of x; c is clamped by the caller, so the loads are
// unconditional and the next tile can be in flight while the current one is accumulated
// (pointers taken from a job record are generic; global-address-space loads keep them on the vector-memory path)
#define DPLLM_SEL_GLOBAL __attribute__((address_space(1)))
__device__ __forceinline__ void sel_load(SelTile& t, const uint16_t* const (&rows)[kSelRowsPerWave], const uint16_t* x, int c) {
#pragma unroll
  for (int i = 0; i < kSelRowsPerWave; ++i)
    t.g[i] = __builtin_nontemporal_load((const DPLLM_SEL_GLOBAL sel_u32x4*)(rows[i] + c));
  const sel_u32x4 xv = *(const DPLLM_SEL_GLOBAL sel_u32x4*)(x + c);
  t.x = make_uint4(xv.x, xv.y, xv.z, xv.w);
}

__device__ __forceinline__ void sel_accumulate(const SelTile& t, bool valid, double (&acc)[kSelRowsPerWave]) {
  const __half* xh = reinterpret_cast<const __half*>(&t.x);
  double xd[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) xd[i] = valid ? (double)__half2float(xh[i]) : 0.0;
#pragma unroll
  for (int r = 0; r < kSelRowsPerWave; ++r) {
    const __half* gh = reinterpret_cast<const __half*>(&t.g[r]);
    // an fp16 x fp16 product is exact in fp64, so the fused multiply-add rounds once, like an fp64 add of the
    // exact product
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[r] = fma((double)__half2float(gh[i]), xd[i], acc[r]);
  }
}

// the estimate from the sum of squares, and the decision
__device__ __forceinline__ void selector_decide(const SelJob& job, double tot) {
  double e = 0.0;
  if (job.kind == 1) e = sqrt(tot);
  else if (job.kind == 2) e = (double)job.alpha * sqrt(tot) + (double)job.beta;
  *job.e_out = (float)e;
  // strictly exceeding T selects h; +inf pins l, -inf pins h; no estimator: always l
  *job.k_out = (job.kind != 0 && e > (double)job.T) ? job.h : job.l;
}

__device__ __forceinline__ void selector_part(const SelJob& job, int part, int tid) {
  __shared__ double sq[kSelMaxRank];
  __shared__ uint32_t is_last;
  const int wave = tid >> 6, lane = tid & 63;
  if (job.kind == 0) {   // no estimator: only the decision
    if (tid == 0) selector_decide(job, 0.0);
    return;
  }
  if (job.kind == 2) {   // sum of x^2, one part
    double acc = 0.0;
    for (int c = tid * 8; c < job.in; c += kSelPartThreads * 8) {
      uint4 xv = *reinterpret_cast<const uint4*>(job.x + c);
      const __half* xh = reinterpret_cast<const __half*>(&xv);
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        float v = __half2float(xh[i]);
        acc += (double)(v * v);  // exact square in fp32
      }
    }
    acc = wave_sum_f64(acc);
    if (lane == 0) sq[wave] = acc;
    __syncthreads();
    if (tid == 0) {
      double tot = 0.0;
      for (int w = 0; w < kSelPartWaves; ++w) tot += sq[w];
      selector_decide(job, tot);
    }
    return;
  }
  // projection: wavefront w owns rows 16 rg + 4 w .. + 3 (clamped to r - 1; surplus rows are dropped), columns
  // [cb, ce) of them
  const int rg = part / job.nchunks, ch = part - rg * job.nchunks;
  const int cb = ch * job.chunk_cols, ce = min(job.in, cb + job.chunk_cols);
  const int row0 = rg * kSelPartRows + wave * kSelRowsPerWave;
  const uint16_t* rows[kSelRowsPerWave];
#pragma unroll
  for (int i = 0; i < kSelRowsPerWave; ++i) rows[i] = job.G + (size_t)min(row0 + i, job.r - 1) * job.in;
  double acc[kSelRowsPerWave];
#pragma unroll
  for (int i = 0; i < kSelRowsPerWave; ++i) acc[i] = 0.0;
  const int last = ce - 8;              // in % 32 == 0 and chunks are multiples of 512, so every 8-column group is whole
  const int nit = (ce - cb + kSelChunkStep - 1) / kSelChunkStep;
  // Rows of G are a power-of-two number of bytes apart in the common shapes, so wavefronts that all walk the
  // columns from the start would hit the same few memory channels at any moment: every wavefront starts its
  // (circular) walk at a different 1 KiB column chunk.
  int it = (int)((blockIdx.x * kSelPartWaves + wave) * 5u % (unsigned)nit);   // tile being loaded
  int ca = cb + it * kSelChunkStep + lane * 8;                                // first column of the tile being accumulated
  SelTile ring[kSelDepth];
#pragma unroll
  for (int d = 0; d < kSelDepth - 1; ++d) {
    sel_load(ring[d], rows, job.x, min(cb + it * kSelChunkStep + lane * 8, last));
    it = it + 1 == nit ? 0 : it + 1;
  }
  for (int k = 0; k < nit; k += kSelDepth) {
#pragma unroll
    for (int d = 0; d < kSelDepth; ++d) {
      // loads past the end of the walk re-read a tile that is never accumulated (uniform, unconditional issue)
      sel_load(ring[(d + kSelDepth - 1) % kSelDepth], rows, job.x, min(cb + it * kSelChunkStep + lane * 8, last));
      it = it + 1 == nit ? 0 : it + 1;
      if (k + d < nit) sel_accumulate(ring[d], ca <= last, acc);
      ca = ca + kSelChunkStep >= cb + nit * kSelChunkStep ? ca + kSelChunkStep - nit * kSelChunkStep : ca + kSelChunkStep;
    }
  }
  // The partial products are left with device-scope atomic exchanges and read with device-scope atomic loads.
  // A read-modify-write is carried out where all dies see it, like the ticket itself, and has been carried out
  // when its old value is back; a store, atomic or not, is acknowledged before other dies see it.  So every
  // exchange is waited for before the ticket is taken, and whoever draws the last ticket finds all of them.
  const int nrows = sel_rowgroups_of(1, job.r) * kSelPartRows;
  DPLLM_SEL_GLOBAL double* ws = (DPLLM_SEL_GLOBAL double*)job.ws;
  DPLLM_SEL_GLOBAL uint32_t* ticket = (DPLLM_SEL_GLOBAL uint32_t*)job.ticket;
  double rowsum[kSelRowsPerWave];
#pragma unroll
  for (int i = 0; i < kSelRowsPerWave; ++i) rowsum[i] = wave_sum_f64(acc[i]);
  if (lane == 0) {   // four exchanges in flight, one wait for their old values
    unsigned long long before[kSelRowsPerWave];
#pragma unroll
    for (int i = 0; i < kSelRowsPerWave; ++i)
      before[i] = __hip_atomic_exchange((DPLLM_SEL_GLOBAL unsigned long long*)(ws + (size_t)ch * nrows + row0 + i),
                                        __builtin_bit_cast(unsigned long long, rowsum[i]), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    static_assert(kSelRowsPerWave == 4, "the wait below names four values");
    asm volatile("" ::"v"((uint32_t)before[0]), "v"((uint32_t)(before[0] >> 32)), "v"((uint32_t)before[1]), "v"((uint32_t)(before[1] >> 32)),
                 "v"((uint32_t)before[2]), "v"((uint32_t)(before[2] >> 32)), "v"((uint32_t)before[3]), "v"((uint32_t)(before[3] >> 32)));
  }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __syncthreads();
  if (tid == 0) {
    const uint32_t old = __hip_atomic_fetch_add(ticket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    is_last = old == (uint32_t)(job.nparts - 1);
  }
  __syncthreads();
  if (!is_last) return;
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
  for (int t = tid; t < job.r; t += kSelPartThreads) {
    double g = 0.0;
    for (int c = 0; c < job.nchunks; ++c) g += __hip_atomic_load(ws + (size_t)c * nrows + t, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    sq[t] = g * g;
  }
  __syncthreads();
  if (tid == 0) {
    __hip_atomic_store(ticket, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    double tot = 0.0;
    for (int t = 0; t < job.r; ++t) tot += sq[t];
    selector_decide(job, tot);
  }
}

// parts == nullptr: the single job passed by value, workgroup b is its part b; else workgroup b serves parts[b]
__global__ void __launch_bounds__(kSelPartThreads) selector_part_kernel(const SelJob* __restrict__ jobs,
                                                                         const SelPart* __restrict__ parts, SelJob one) {
  if (parts == nullptr) {
    selector_part(one, blockIdx.x, threadIdx.x);
  } else {
    const SelPart p = parts[blockIdx.x];
    SelJob job = jobs[p.job];
    selector_part(job, p.part, threadIdx.x);
  }
}

}  // namespace dpllm
