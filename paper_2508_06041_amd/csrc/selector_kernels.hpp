// Precision selector kernels (paper Sec. 3: the layer takes h when the relative error exceeds its threshold
// T, else l; Sec. 5.1: the error is estimated as ||G x|| with G = A (W_h - W_l) precomputed, or as
// alpha ||x|| + beta).  One launch serves a list of selector jobs; the bitwidth lands in device memory, where
// the GEMV kernels read it.
//
// What a linear's selector is (candidate pair, estimator kind, G, alpha, beta, T) depends on the target
// precision the model runs under (Algorithm 1 hands out one threshold list per target; Sec. 5.1 keeps one G per
// candidate pair): the kernels read the number of the active target from device memory and take the linear's
// parameters from the row of that target in a table, so that a switch of target is one word written on the
// device and the launches stay what they are.
//
// A projection job reads 0.5 - 3.5 MB of G.  It is cut into parts of 16 rows of G (one workgroup of four
// wavefronts, four rows per wavefront sharing the activation loads) by a chunk of columns: the whole row when
// the launch has enough parts to fill the chip, down to 512 columns when it serves a few linears only (a part
// that streams a whole row alone takes 10 - 30 us).  A part leaves the fp64 partial dot products of its rows in
// workspace slots of its own, and that is all it does.  Linears whose estimator is the linear regression need
// sum x^2 only: the jobs of a launch that read the same input vector form a group with one extra part, which
// adds up x^2 once and leaves it in the slot of every member that asks for it.
//
// The estimate and the decision are taken by whoever consumes them, in a LATER launch on the same stream
// (selector_finish): the GEMV kernel, in the prologue of every workgroup of the linear (the first one also
// writes the estimate and the bitwidth to the caller's arrays), or selector_decide_kernel where no GEMV follows.
// The end of the launch that wrote the partial products and the start of the one that reads them order the two
// at device scope; no workgroup waits for another inside a launch.  (Handing the partial products to a last-
// arriving part inside the launch needs a device-scope release by every part and an acquire by the last one;
// the release writes back the die's whole L2 and measured 126 us for the 224 selectors of a 7B step, against
// 30 us for the parts alone.)  selector_finish adds the partial products of every row in chunk order, squares,
// adds the rows in index order, takes the square root and compares: the order of all additions is fixed, so every
// workgroup that repeats it gets the same bits.
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
constexpr int kSelDepth = 2;         // column tiles in registers: one being accumulated, one in flight (two in flight measured slower: 32 against 28 us for the 224 selectors of a 7B step)
constexpr int kSelPartRows = kSelPartWaves * kSelRowsPerWave;
constexpr int kSelMaxRank = 1024;
constexpr int kSelMaxChunks = 32;    // column chunks of a job
constexpr int kSelChunkStep = 512;   // columns a wavefront covers per tile: chunks are multiples of it

// What the selector of one linear is under one target.  kind: 0 none (always l), 1 projection, 2 linear regression
struct SelParams {
  const uint16_t* G;   // fp16 [r][in] (projection kind)
  float T, alpha, beta;
  int32_t r, l, h, kind;
  int32_t pad;
};

// The target-independent part of a selector job.
struct SelJob {
  const uint16_t* x;   // fp16 [in]: the vector the selector reads
  float* e_out;
  int32_t* k_out;
  double* ws;          // [nchunks][ws_rows] partial dot products (projection), or [0] = sum x^2 (linear regression)
  int32_t in;
  int32_t linear;      // row of the job's linear in the parameter table
  int32_t nchunks, chunk_cols;  // projection part p covers rows [16 (p / nchunks), + 16), columns [chunk_cols (p % nchunks), + chunk_cols)
  int32_t ws_rows;     // rows of one chunk's slots in ws (the largest rank of the linear's pairs, rounded up to 16)
  int32_t pad;
};
struct SelPart {
  int32_t job;     // index into the job table of the launch
  int32_t part;    // projection part number inside the job; -1: the group part of the group whose first member is `job`
  int32_t linear;  // the job's row in the parameter table (so that job record and parameters load side by side)
  int32_t count;   // group part: members of the group; they are members[first .. first + count) of the launch's member
  int32_t first;   //   table (indices into the job table), all reading the same vector
  int32_t pad;
};

__host__ __device__ inline int sel_rowgroups_of(int kind, int r) {
  return kind == 1 ? (r + kSelPartRows - 1) / kSelPartRows : 0;
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

// LDS of a selector workgroup / of the finishing step
struct SelShared {
  double sq[kSelMaxRank + 1];   // [kSelMaxRank]: the total
};

// What the finishing step needs of a selector job (a copy of it travels in the GEMV job record)
struct SelFinish {
  const double* ws;
  float* e_out;
  int32_t* k_out;
  int32_t in, linear, nchunks, ws_rows;
};
__host__ __device__ inline SelFinish sel_finish_of(const SelJob& j) {
  return SelFinish{j.ws, j.e_out, j.k_out, j.in, j.linear, j.nchunks, j.ws_rows};
}

// The estimate from what the selector launch left in the workspace, and the decision; called by all `nthreads`
// (a multiple of 64, at least 64) threads of a workgroup (it holds workgroup barriers), every thread returns the
// bitwidth.  write: thread 0 also stores the estimate and the bitwidth.  The partial products were written by an
// earlier launch.  Order of the additions (fixed, so that every workgroup that repeats them gets the same bits):
// per row of G its chunks in chunk order; the squares of rows t, t + 64, t + 128, ... in that order in lane t of
// the first wavefront; the 64 lane sums by a butterfly.  Loads are issued in batches ahead of the additions that
// consume them: a workgroup of the GEMV kernel pays this latency before it can start streaming.
__device__ __forceinline__ int selector_finish(const SelFinish& f, const SelParams* prow, int tid, int nthreads, double* sq, bool write) {
  const DPLLM_SEL_GLOBAL double* ws = (const DPLLM_SEL_GLOBAL double*)f.ws;
  // the first batch of partial products is asked for before the parameters, so that both arrive together (what
  // the batch means is known once the parameters are here: slot 0 may also be sum x^2)
  double v[8];
  const int t0 = min(tid, f.ws_rows - 1);
#pragma unroll
  for (int i = 0; i < 8; ++i) v[i] = ws[(size_t)min(i, f.nchunks - 1) * f.ws_rows + t0];
  const SelParams P = *prow;
  double e = 0.0;
  if (P.kind == 1) {
    for (int t = tid; t < P.r; t += nthreads) {
      double g = 0.0;
      for (int c0 = 0; c0 < f.nchunks; c0 += 8) {
        if (c0 > 0 || t != tid) {
#pragma unroll
          for (int i = 0; i < 8; ++i) v[i] = ws[(size_t)min(c0 + i, f.nchunks - 1) * f.ws_rows + t];
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) g += c0 + i < f.nchunks ? v[i] : 0.0;
      }
      sq[t] = g * g;
    }
    __syncthreads();
    if (tid < 64) {
      double part = 0.0;
      for (int t = tid; t < P.r; t += 64) part += sq[t];
      part = wave_sum_f64(part);
      if (tid == 0) sq[kSelMaxRank] = part;
    }
    __syncthreads();
    e = sqrt(sq[kSelMaxRank]);
    __syncthreads();                              // sq may be reused by the caller
  } else if (P.kind == 2) {
    e = (double)P.alpha * sqrt(ws[0]) + (double)P.beta;
  }
  // strictly exceeding T selects h; +inf pins l, -inf pins h; no estimator: always l
  const int k = (P.kind != 0 && e > (double)P.T) ? P.h : P.l;
  if (write && tid == 0) {
    *f.e_out = (float)e;
    *f.k_out = k;
  }
  return k;
}

// The group part: sum x^2, added up once for the jobs of the launch that read the same vector and left in the
// slot of every member whose estimator under the active target is the linear regression.
__device__ __forceinline__ void selector_group_part(const SelJob* jobs, const int32_t* members, int count, const SelParams* params,
                                                    const SelJob& lone, const SelParams& one, int tid, SelShared& sh) {
  const int wave = tid >> 6, lane = tid & 63;
  const SelJob& head = jobs ? jobs[members[0]] : lone;
  int need = 0;
  if (jobs) {
    for (int i = tid; i < count; i += kSelPartThreads) need |= params[jobs[members[i]].linear].kind == 2;
  } else {
    need = one.kind == 2;
  }
  if (!__syncthreads_or(need)) return;
  double acc = 0.0;
  for (int c = tid * 8; c < head.in; c += kSelPartThreads * 8) {
    const sel_u32x4 xv = *(const DPLLM_SEL_GLOBAL sel_u32x4*)(head.x + c);
    const __half* xh = reinterpret_cast<const __half*>(&xv);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      float v = __half2float(xh[i]);
      acc += (double)(v * v);  // exact square in fp32
    }
  }
  acc = wave_sum_f64(acc);
  if (lane == 0) sh.sq[wave] = acc;
  __syncthreads();
  double tot = 0.0;
  for (int w = 0; w < kSelPartWaves; ++w) tot += sh.sq[w];
  if (jobs) {
    for (int i = tid; i < count; i += kSelPartThreads) {
      const SelJob& j = jobs[members[i]];
      if (params[j.linear].kind == 2) j.ws[0] = tot;
    }
  } else if (tid == 0) {
    lone.ws[0] = tot;
  }
}

// One projection part: wavefront w owns rows 16 rg + 4 w .. + 3 (clamped to r - 1; surplus rows are dropped),
// columns [cb, ce) of them
__device__ __forceinline__ void selector_proj_part(const SelJob& job, const SelParams& P, int part, int tid) {
  const int wave = tid >> 6, lane = tid & 63;
  if (P.kind != 1) return;                                    // this target estimates the linear otherwise
  const int rg = part / job.nchunks, ch = part - rg * job.nchunks;
  if (rg >= sel_rowgroups_of(1, P.r)) return;                 // the pair of this target has fewer rows of G
  const int cb = ch * job.chunk_cols, ce = min(job.in, cb + job.chunk_cols);
  const int row0 = rg * kSelPartRows + wave * kSelRowsPerWave;
  const uint16_t* rows[kSelRowsPerWave];
#pragma unroll
  for (int i = 0; i < kSelRowsPerWave; ++i) rows[i] = P.G + (size_t)min(row0 + i, P.r - 1) * job.in;
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
  DPLLM_SEL_GLOBAL double* ws = (DPLLM_SEL_GLOBAL double*)job.ws;
#pragma unroll
  for (int i = 0; i < kSelRowsPerWave; ++i) {
    const double rowsum = wave_sum_f64(acc[i]);
    if (lane == 0) ws[(size_t)ch * job.ws_rows + row0 + i] = rowsum;
  }
}

// parts == nullptr: the single job `one_job` with the parameters `one`; workgroup b is its projection part b, or
// (linear regression: one workgroup) its group part.  Else workgroup b serves parts[b] of the launch's job table
// under the target *target (members: the launch's table of group members).
__global__ void __launch_bounds__(kSelPartThreads) __attribute__((amdgpu_waves_per_eu(5))) selector_part_kernel(const SelJob* __restrict__ jobs, const SelPart* __restrict__ parts,
                                                                         const int32_t* __restrict__ members,
                                                                         const SelParams* __restrict__ params,
                                                                         const int32_t* __restrict__ target, int n_linears,
                                                                         SelJob one_job, SelParams one) {
  __shared__ SelShared sh;
  if (parts == nullptr) {
    if (one.kind == 1) selector_proj_part(one_job, one, blockIdx.x, threadIdx.x);
    else selector_group_part(nullptr, nullptr, 1, nullptr, one_job, one, threadIdx.x, sh);
    return;
  }
  const SelPart p = parts[blockIdx.x];
  const SelParams* row = params + (size_t)(*target) * n_linears;
  if (p.part < 0) {
    selector_group_part(jobs, members + p.first, p.count, row, one_job, one, threadIdx.x, sh);
  } else {
    const SelParams P = row[p.linear];
    const SelJob job = jobs[p.job];
    selector_proj_part(job, P, p.part, threadIdx.x);
  }
}

// The estimates and decisions of a selector launch, where no GEMV launch follows that takes them itself:
// workgroup b finishes jobs[b] under the target *target (jobs == nullptr: the single job `one_job` with the
// parameters `one`).  Launched after selector_part_kernel on the same stream.
constexpr int kSelDecideThreads = 128;
__global__ void __launch_bounds__(kSelDecideThreads) selector_decide_kernel(const SelJob* __restrict__ jobs, const SelParams* __restrict__ params,
                                                                            const int32_t* __restrict__ target, int n_linears,
                                                                            SelJob one_job, SelParams one) {
  __shared__ SelShared sh;
  if (jobs == nullptr) {
    selector_finish(sel_finish_of(one_job), &one, threadIdx.x, kSelDecideThreads, sh.sq, true);
    return;
  }
  const SelJob job = jobs[blockIdx.x];
  selector_finish(sel_finish_of(job), params + (size_t)(*target) * n_linears + job.linear, threadIdx.x, kSelDecideThreads, sh.sq, true);
}

}  // namespace dpllm
