// Any-precision GEMV for gfx950, batch 1: y[o] = sum_c LUT_k[o][code_k(o,c)] * x[c]   (paper Sec. 3: the
// linear operation of a decode step; Sec. 2.2: the k-bit model is the top k planes of the parent).
//
// Work split: one 64-lane wavefront (= one workgroup) owns one row quad and walks its columns in strips
// of 64 words; a lane loads one 128-bit value per plane and strip (4 rows x 32 columns), so a wavefront
// load is 1 KiB of contiguous memory per plane.  Only planes 0..k-1 are read.
//
// Decoding: the layout keeps the k bits of a weight at adjacent descending positions of planes 0..k-1
// (see layout_device.hpp), so code fields are built by mask-merging whole plane words (v_bfi_b32), never
// bit by bit:
//   k = 3   : three merges give a word of four bytes [a2 a1 a0 b2 b1 b0 0 0]: the byte is the LDS offset
//             of entry (a,b) of a per-row table of fp16 pairs (64 entries); one LDS read returns both
//             weights packed, one v_dot2_f32_f16 multiplies them with the packed activations (2i, 2i+1).
//   k != 3  : a three-level merge tree (2-, 4-, 8-bit fields) gives eight words of four bytes [code << 1]
//             (k = 8: [code]); the byte is the LDS offset into the row's fp16 table; one fp32 mixed FMA
//             per weight.
// The per-row tables sit in LDS (wavefront-private: 64 B..2 KiB); activations are read from global memory
// (L1/L2 hits) straight into packed registers, because LDS lookups are the scarcest resource at low k.
// All accumulation is fp32; the four row sums are reduced across the wavefront at the end.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

#include "layout_device.hpp"

namespace dpllm {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct GemvJob {
  const char* arena;          // device planes start here; plane b at + b * plane_stride_u4 * 16 bytes
  const uint16_t* x;          // fp16 [in]
  uint16_t* y;                // fp16 [out]
  const int32_t* k_dev;       // nullptr: serve ka; else *k_dev is ka or kb
  uint32_t plane_stride_u4;
  uint32_t lut_off_a, lut_off_b;  // byte offsets of the ka / kb tables inside the arena
  int32_t ka, kb;
  int32_t out, ncw, nrq;
  int32_t block_start;        // index of this job's first workgroup inside a multi-job grid
};

__device__ __forceinline__ uint32_t bfi(uint32_t mask, uint32_t a, uint32_t b) { return (a & mask) | (b & ~mask); }

__device__ __forceinline__ float wave_sum_f32(float v) {
#pragma unroll
  for (int s = 32; s >= 1; s >>= 1) v += __shfl_xor(v, s, 64);
  return v;
}

__device__ __forceinline__ u32x4 load_stream(const u32x4* p) { return __builtin_nontemporal_load(p); }

// ---- where the byte field of a column ends up after the merge tree (all compile-time) -------------------
template <int K>
struct ByteFieldMap {
  static constexpr int d = (K == 8) ? 0 : 7 - K;  // plane b uses tree slot b + d; empty slots read as zero
  __host__ __device__ static constexpr int top(int col) { return (col_to_pos(col) + d) & 31; }  // field top bit
  __host__ __device__ static constexpr int word(int col) { return top(col) & 7; }
  __host__ __device__ static constexpr int rot(int c) { return (c + 1) & 7; }
  __host__ __device__ static constexpr int byte(int col) { return ((top(col) - rot(word(col))) & 31) >> 3; }
};

// planes of one row -> eight words, each four byte-aligned fields
template <int K>
__device__ __forceinline__ void merge_byte_fields(const uint32_t (&w)[K], uint32_t (&R)[8]) {
  constexpr int d = ByteFieldMap<K>::d;
  uint32_t v[8];
#pragma unroll
  for (int s = 0; s < 8; ++s) v[s] = (s >= d && s < d + K) ? w[(s >= d && s < d + K) ? s - d : 0] : 0u;
  uint32_t A[4][2];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    A[i][0] = bfi(field_mask(2, 0, 1), v[2 * i], v[2 * i + 1]);
    A[i][1] = bfi(field_mask(2, 1, 1), v[2 * i], v[2 * i + 1]);
  }
  uint32_t B[2][4];
#pragma unroll
  for (int g = 0; g < 2; ++g) {
    B[g][0] = bfi(field_mask(4, 0, 2), A[2 * g][0], A[2 * g + 1][0]);
    B[g][1] = bfi(field_mask(4, 1, 2), A[2 * g][1], A[2 * g + 1][1]);
    B[g][2] = bfi(field_mask(4, 2, 2), A[2 * g][0], A[2 * g + 1][0]);
    B[g][3] = bfi(field_mask(4, 3, 2), A[2 * g][1], A[2 * g + 1][1]);
  }
  R[0] = __builtin_rotateright32(bfi(field_mask(8, 0, 4), B[0][0], B[1][0]), 1);
  R[1] = __builtin_rotateright32(bfi(field_mask(8, 1, 4), B[0][1], B[1][1]), 2);
  R[2] = __builtin_rotateright32(bfi(field_mask(8, 2, 4), B[0][2], B[1][2]), 3);
  R[3] = __builtin_rotateright32(bfi(field_mask(8, 3, 4), B[0][3], B[1][3]), 4);
  R[4] = __builtin_rotateright32(bfi(field_mask(8, 4, 4), B[0][0], B[1][0]), 5);
  R[5] = __builtin_rotateright32(bfi(field_mask(8, 5, 4), B[0][1], B[1][1]), 6);
  R[6] = __builtin_rotateright32(bfi(field_mask(8, 6, 4), B[0][2], B[1][2]), 7);
  R[7] = bfi(field_mask(8, 7, 4), B[0][3], B[1][3]);
}

// one row x 32 columns, single lookups; tbl = this row's fp16 table in LDS
template <int K, int COL>
__device__ __forceinline__ _Float16 lookup_col(const uint32_t (&R)[8], const char* tbl) {
  using M = ByteFieldMap<K>;
  uint32_t f = (R[M::word(COL)] >> (8 * M::byte(COL))) & 0xffu;
  if (K == 8) f <<= 1;
  return *reinterpret_cast<const _Float16*>(tbl + f);
}

template <int K, int I>
__device__ __forceinline__ float mac_pairs(const uint32_t (&R)[8], const uint32_t (&xp)[16], const char* tbl, float acc) {
  if constexpr (I < 16) {
    half2_t xv = __builtin_bit_cast(half2_t, xp[I]);
    acc = __builtin_fmaf((float)lookup_col<K, 2 * I>(R, tbl), (float)xv.x, acc);
    acc = __builtin_fmaf((float)lookup_col<K, 2 * I + 1>(R, tbl), (float)xv.y, acc);
    return mac_pairs<K, I + 1>(R, xp, tbl, acc);
  } else {
    return acc;
  }
}

template <int K>
__device__ __forceinline__ float row_dot(const uint32_t (&w)[K], const uint32_t (&xp)[16], const char* tbl, float acc) {
  if constexpr (K == 3) {
    // pair lookups: byte n of merged word jj holds 4 * (8 a + b) for columns (2i, 2i+1), i = 4 jj + n
    constexpr uint32_t m0 = 0x90909090u;
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) {
      const int j = 2 * jj;
      uint32_t o = (w[0] & rotl_c(m0, j)) | (w[1] & rotl_c(m0 >> 1, j)) | (w[2] & rotl_c(m0 >> 2, j));
      uint32_t t = __builtin_rotateright32(o, j);
#pragma unroll
      for (int n = 0; n < 4; ++n) {
        uint32_t f = (t >> (8 * n)) & 0xffu;
        half2_t wv = __builtin_bit_cast(half2_t, *reinterpret_cast<const uint32_t*>(tbl + f));
        acc = __builtin_amdgcn_fdot2(wv, __builtin_bit_cast(half2_t, xp[4 * jj + n]), acc, false);
      }
    }
    return acc;
  } else {
    uint32_t R[8];
    merge_byte_fields<K>(w, R);
    return mac_pairs<K, 0>(R, xp, tbl, acc);
  }
}

template <int K>
struct Strip {
  u32x4 w[K];
  u32x4 x[4];
};

template <int K>
__device__ __forceinline__ void load_strip(Strip<K>& s, const GemvJob& job, int rq, int cw) {
  if (cw < job.ncw) {
    const u32x4* p = reinterpret_cast<const u32x4*>(job.arena) + (size_t)rq * job.ncw + cw;
#pragma unroll
    for (int b = 0; b < K; ++b) s.w[b] = load_stream(p + (size_t)b * job.plane_stride_u4);
    const u32x4* xp = reinterpret_cast<const u32x4*>(job.x) + (size_t)cw * 4;
#pragma unroll
    for (int i = 0; i < 4; ++i) s.x[i] = xp[i];
  }
}

template <int K>
__device__ __forceinline__ constexpr int row_table_bytes() { return K == 3 ? 256 : (2 << K); }

template <int K>
__device__ __forceinline__ void compute_strip(const Strip<K>& s, int cw, int ncw, const char* lds, float (&acc)[4]) {
  if (cw >= ncw) return;
  uint32_t xp[16];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    xp[4 * i + 0] = s.x[i].x;
    xp[4 * i + 1] = s.x[i].y;
    xp[4 * i + 2] = s.x[i].z;
    xp[4 * i + 3] = s.x[i].w;
  }
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    uint32_t w[K];
#pragma unroll
    for (int b = 0; b < K; ++b) w[b] = s.w[b][r];
    acc[r] = row_dot<K>(w, xp, lds + r * row_table_bytes<K>(), acc[r]);
  }
}

// one wavefront, one row quad
template <int K>
__device__ __forceinline__ void gemv_rowquad(const GemvJob& job, uint32_t lut_off, int rq, int lane, char* lds) {
  const uint16_t* lut = reinterpret_cast<const uint16_t*>(job.arena + lut_off) + ((size_t)rq * 4 << K);
  Strip<K> s0, s1;
  load_strip<K>(s0, job, rq, lane);
  if constexpr (K == 3) {
    const int a = lane >> 3, b = lane & 7;
#pragma unroll
    for (int r = 0; r < 4; ++r)
      reinterpret_cast<uint32_t*>(lds)[r * 64 + lane] = (uint32_t)lut[r * 8 + a] | ((uint32_t)lut[r * 8 + b] << 16);
  } else {
    constexpr int dwords = (4 << K) / 2;
    const uint32_t* src = reinterpret_cast<const uint32_t*>(lut);
    for (int e = lane; e < dwords; e += 64) reinterpret_cast<uint32_t*>(lds)[e] = src[e];
  }
  __syncthreads();
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  const int ncw = job.ncw;
  for (int c0 = 0; c0 < ncw; c0 += 128) {
    if (c0 + 64 < ncw) load_strip<K>(s1, job, rq, c0 + 64 + lane);
    compute_strip<K>(s0, c0 + lane, ncw, lds, acc);
    if (c0 + 64 < ncw) {
      if (c0 + 128 < ncw) load_strip<K>(s0, job, rq, c0 + 128 + lane);
      compute_strip<K>(s1, c0 + 64 + lane, ncw, lds, acc);
    }
  }
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    float s = wave_sum_f32(acc[r]);
    int o = rq * 4 + r;
    if (lane == 0 && o < job.out) job.y[o] = __builtin_bit_cast(uint16_t, (_Float16)s);
  }
}

__device__ __forceinline__ void gemv_dispatch(const GemvJob& job, int rq, int lane, char* lds) {
  int k = job.ka;
  uint32_t off = job.lut_off_a;
  if (job.k_dev != nullptr) {
    int kd = __builtin_amdgcn_readfirstlane(*job.k_dev);
    if (kd == job.kb) { k = job.kb; off = job.lut_off_b; }
  }
  switch (k) {
    case 1: gemv_rowquad<1>(job, off, rq, lane, lds); break;
    case 2: gemv_rowquad<2>(job, off, rq, lane, lds); break;
    case 3: gemv_rowquad<3>(job, off, rq, lane, lds); break;
    case 4: gemv_rowquad<4>(job, off, rq, lane, lds); break;
    case 5: gemv_rowquad<5>(job, off, rq, lane, lds); break;
    case 6: gemv_rowquad<6>(job, off, rq, lane, lds); break;
    case 7: gemv_rowquad<7>(job, off, rq, lane, lds); break;
    case 8: gemv_rowquad<8>(job, off, rq, lane, lds); break;
    default: break;
  }
}

__global__ void __launch_bounds__(64) gemv_one_kernel(GemvJob job) {
  __shared__ __attribute__((aligned(16))) char lds[2048];
  gemv_dispatch(job, blockIdx.x, threadIdx.x, lds);
}

// jobs[j].block_start ascending; block b belongs to the last job whose block_start <= b
__global__ void __launch_bounds__(64) gemv_multi_kernel(const GemvJob* __restrict__ jobs, int njobs) {
  __shared__ __attribute__((aligned(16))) char lds[2048];
  const int b = blockIdx.x;
  int lo = 0, hi = njobs - 1;
  while (lo < hi) {
    int mid = (lo + hi + 1) >> 1;
    if (jobs[mid].block_start <= b) lo = mid; else hi = mid - 1;
  }
  GemvJob job = jobs[lo];
  gemv_dispatch(job, b - job.block_start, threadIdx.x, lds);
}

}  // namespace dpllm
