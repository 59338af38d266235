// Pieces shared by the any-precision GEMV kernels for gfx950: the job record, global-memory helpers and the
// mask-merge trees that turn bitplane words into code fields (paper Sec. 2.2: the k-bit model is the top k
// planes of the parent; Sec. 3: the linear operation of a decode step is a GEMV).
//
// Decoding: the layout keeps the k bits of a weight at adjacent descending positions of planes 0..k-1
// (see layout_device.hpp), so code fields are built by mask-merging whole plane words, never bit by bit:
//   k = 3   : three instructions per word give four bytes [a2 a1 a0 b2 b1 b0 . .]: entry (a,b) of a per-row
//             table of fp16 pairs (64 entries); one LDS read returns both weights packed, one v_dot2
//             multiplies them with the packed activations (2i, 2i+1).
//   k = 4   : the 4-bit code words are bytes 16 a + b of two weights four positions apart; a 256-entry pair
//             table per row is built in LDS from the row's 16 centroids; activations are re-paired to match.
//   k >= 5  : a three-level merge tree (2-, 4-, 8-bit fields) gives eight words of four byte fields [code];
//             one lookup per weight.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

#include "layout_device.hpp"
#include "selector_kernels.hpp"

namespace dpllm {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kFastKMin = 3, kFastKMax = 8;   // bitwidths the streaming kernel serves; others take the plain kernel

struct GemvJob {
  const char* arena;          // device planes start here; plane b at + b * plane_stride_u4 * 16 bytes
  const uint16_t* x;          // fp16 [in]
  uint16_t* y;                // fp16 [out]
  const int32_t* k_dev;       // nullptr: serve k; else the bitwidth is *k_dev (written by a selector)
  // has_fin != 0: neither; the bitwidth is decided in the workgroup's prologue from the partial results an earlier
  // selector launch left in the workspace (selector_finish), and the job's first workgroup writes it and the
  // estimate to the caller's arrays
  int32_t has_fin;
  SelFinish fin;
  uint32_t plane_stride_u4;
  uint32_t lut_off[kFastKMax - kFastKMin + 1];  // byte offset of the k-bit table inside the arena, k = 3..8
  int32_t k;                  // the bitwidth when k_dev == nullptr
  int32_t kmin, p;            // bitwidths the linear serves: a value read from k_dev outside them is not served
  int32_t out, ncw;           // rows; 32-column words per row
  int32_t nrq, ncc;           // blocks of 64 rows; 128-column tiles per row
  int32_t nblocks;            // workgroups of this job; workgroup b streams row blocks b / nsplit, + nblocks / nsplit, ...
  int32_t block_start;        // index of this job's first workgroup inside a multi-job grid
  int32_t nsamples;           // right-hand sides served together (1..NB): sample s reads x + s * in, writes y + s * out
  // column split: nsplit workgroups share every block of rows, each taking 1 / nsplit of its column tiles
  // (nblocks counts all of them).  Their fp32 partial sums meet in ws ([row block][sample][split][64 rows]);
  // cnt ([row block][sample], zero between launches) tells the last one to arrive, which adds them up.
  int32_t nsplit;
  float* ws;
  uint32_t* cnt;
};

__device__ __forceinline__ uint32_t bfi(uint32_t mask, uint32_t a, uint32_t b) { return (a & mask) | (b & ~mask); }

// v_bfi_b32 with a wavefront-uniform mask (held in a scalar register)
__device__ __forceinline__ uint32_t bfi_insn(uint32_t mask, uint32_t a, uint32_t b) {
  uint32_t r;
  asm("v_bfi_b32 %0, %1, %2, %3" : "=v"(r) : "s"(mask), "v"(a), "v"(b));
  return r;
}

// (a & m) | (b & ~m) with all three operands in vector registers: v_bitop3_b32 runs at full rate (a wavefront
// instruction every two cycles per SIMD) only in that form; with a scalar or literal operand, and v_bfi_b32 /
// v_and_or_b32 in any form, take four cycles (measured).  The masks of the merge trees are therefore kept in
// vector registers (vreg_const, once per workgroup).
__device__ __forceinline__ uint32_t bfi_v(uint32_t m, uint32_t a, uint32_t b) {
  uint32_t r;
  asm("v_bitop3_b32 %0, %1, %2, %3 bitop3:0xca" : "=v"(r) : "v"(m), "v"(a), "v"(b));
  return r;
}
// (a & m) | b, same form
__device__ __forceinline__ uint32_t and_or_v(uint32_t a, uint32_t m, uint32_t b) {
  uint32_t r;
  asm("v_bitop3_b32 %0, %1, %2, %3 bitop3:0xea" : "=v"(r) : "v"(a), "v"(m), "v"(b));
  return r;
}
__device__ __forceinline__ uint32_t vreg_const(uint32_t c) {
  uint32_t r;
  asm volatile("v_mov_b32 %0, %1" : "=v"(r) : "s"(c));
  return r;
}

// Pointers read from a job record are generic; the kernels turn them into global-address-space pointers so
// that loads use the vector-memory counter only and do not tie up the LDS counter the lookups wait on.
#define DPLLM_GLOBAL __attribute__((address_space(1)))
template <class T>
__device__ __forceinline__ const DPLLM_GLOBAL T* as_global(const T* p) { return (const DPLLM_GLOBAL T*)p; }
template <class T>
__device__ __forceinline__ DPLLM_GLOBAL T* as_global(T* p) { return (DPLLM_GLOBAL T*)p; }

// streamed once: non-temporal loads measured about 10 % faster than plain ones on this access pattern
__device__ __forceinline__ u32x4 load_stream(const DPLLM_GLOBAL u32x4* p) { return __builtin_nontemporal_load(p); }

// planes of one row -> eight words, each four byte-aligned fields [code << (8 - K - D)]
template <int K, int D>
__device__ __forceinline__ void merge_byte_fields(const uint32_t (&w)[K], uint32_t (&R)[8]) {
  constexpr int d = D;
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

// k = 4: planes of one row -> four words of four bytes 16 a + b.  Word c collects the 4-bit codes whose top
// bit sits at a position congruent to c (mod 4) and is rotated so that codes fill whole nibbles; the two
// weights of a byte are four positions apart.
__device__ __forceinline__ void merge_nibble_pairs(const uint32_t (&w)[4], uint32_t (&T)[4]) {
  uint32_t A[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    A[i][0] = bfi(field_mask(2, 0, 1), w[2 * i], w[2 * i + 1]);
    A[i][1] = bfi(field_mask(2, 1, 1), w[2 * i], w[2 * i + 1]);
  }
  T[0] = __builtin_rotateright32(bfi(field_mask(4, 0, 2), A[0][0], A[1][0]), 1);
  T[1] = __builtin_rotateright32(bfi(field_mask(4, 1, 2), A[0][1], A[1][1]), 2);
  T[2] = __builtin_rotateright32(bfi(field_mask(4, 2, 2), A[0][0], A[1][0]), 3);
  T[3] = bfi(field_mask(4, 3, 2), A[0][1], A[1][1]);
}

// The same trees with their masks in vector registers (MergeMasks<K>::init, once per workgroup).
template <int K>
struct MergeMasks {
  static constexpr int count = K == 3 ? 8 : K == 4 ? 6 : 15;   // k >= 5: 14 masks and a zero
  uint32_t m[count];
  __device__ __forceinline__ void init() {
    if constexpr (K == 3) {
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) {
        m[2 * jj] = vreg_const(rotl_c(0x90909090u, 2 * jj));
        m[2 * jj + 1] = vreg_const(rotl_c(0x48484848u, 2 * jj));
      }
    } else {
      m[0] = vreg_const(field_mask(2, 0, 1));
      m[1] = vreg_const(field_mask(2, 1, 1));
#pragma unroll
      for (int c = 0; c < 4; ++c) m[2 + c] = vreg_const(field_mask(4, c, 2));
      if constexpr (K >= 5) {
#pragma unroll
        for (int c = 0; c < 8; ++c) m[6 + c] = vreg_const(field_mask(8, c, 4));
        m[14] = vreg_const(0u);
      }
    }
  }
};

template <int K, int D>
__device__ __forceinline__ void merge_byte_fields_v(const uint32_t (&w)[K], uint32_t (&R)[8], const MergeMasks<K>& M) {
  constexpr int d = D;
  const uint32_t zero = M.m[14];
  uint32_t v[8];
#pragma unroll
  for (int s = 0; s < 8; ++s) v[s] = (s >= d && s < d + K) ? w[(s >= d && s < d + K) ? s - d : 0] : zero;
  uint32_t A[4][2];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    if (2 * i + 1 >= d && 2 * i < d + K) {   // at least one of the two slots holds a plane
      A[i][0] = bfi_v(M.m[0], v[2 * i], v[2 * i + 1]);
      A[i][1] = bfi_v(M.m[1], v[2 * i], v[2 * i + 1]);
    } else {
      A[i][0] = A[i][1] = zero;
    }
  }
  uint32_t B[2][4];
#pragma unroll
  for (int g = 0; g < 2; ++g) {
    B[g][0] = bfi_v(M.m[2], A[2 * g][0], A[2 * g + 1][0]);
    B[g][1] = bfi_v(M.m[3], A[2 * g][1], A[2 * g + 1][1]);
    B[g][2] = bfi_v(M.m[4], A[2 * g][0], A[2 * g + 1][0]);
    B[g][3] = bfi_v(M.m[5], A[2 * g][1], A[2 * g + 1][1]);
  }
  R[0] = __builtin_rotateright32(bfi_v(M.m[6], B[0][0], B[1][0]), 1);
  R[1] = __builtin_rotateright32(bfi_v(M.m[7], B[0][1], B[1][1]), 2);
  R[2] = __builtin_rotateright32(bfi_v(M.m[8], B[0][2], B[1][2]), 3);
  R[3] = __builtin_rotateright32(bfi_v(M.m[9], B[0][3], B[1][3]), 4);
  R[4] = __builtin_rotateright32(bfi_v(M.m[10], B[0][0], B[1][0]), 5);
  R[5] = __builtin_rotateright32(bfi_v(M.m[11], B[0][1], B[1][1]), 6);
  R[6] = __builtin_rotateright32(bfi_v(M.m[12], B[0][2], B[1][2]), 7);
  R[7] = bfi_v(M.m[13], B[0][3], B[1][3]);
}

__device__ __forceinline__ void merge_nibble_pairs_v(const uint32_t (&w)[4], uint32_t (&T)[4], const MergeMasks<4>& M) {
  uint32_t A[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    A[i][0] = bfi_v(M.m[0], w[2 * i], w[2 * i + 1]);
    A[i][1] = bfi_v(M.m[1], w[2 * i], w[2 * i + 1]);
  }
  T[0] = __builtin_rotateright32(bfi_v(M.m[2], A[0][0], A[1][0]), 1);
  T[1] = __builtin_rotateright32(bfi_v(M.m[3], A[0][1], A[1][1]), 2);
  T[2] = __builtin_rotateright32(bfi_v(M.m[4], A[0][0], A[1][0]), 3);
  T[3] = bfi_v(M.m[5], A[0][1], A[1][1]);
}

// columns of the two weights in byte m of word c of merge_nibble_pairs: upper nibble, lower nibble
__host__ __device__ constexpr int nibble_pair_col_hi(int c, int m) { return pos_to_col((8 * m + 7 + ((c + 1) & 3)) & 31); }
__host__ __device__ constexpr int nibble_pair_col_lo(int c, int m) { return pos_to_col((8 * m + 3 + ((c + 1) & 3)) & 31); }

__device__ __forceinline__ void sched_fence() { __builtin_amdgcn_sched_barrier(0); }

// Orders the LDS writes of a wavefront against its own later LDS reads.  The LDS executes one wavefront's
// operations in issue order, so only the compiler has to be held back; no counter wait is wanted here (a
// workgroup barrier would also drain the prefetched global loads).
__device__ __forceinline__ void lds_order() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

}  // namespace dpllm
