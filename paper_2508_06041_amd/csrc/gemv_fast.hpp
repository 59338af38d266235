// Any-precision GEMV for gfx950: y[o] = sum_c LUT_k[o][code_k(o,c)] * x[c]   (paper Sec. 3: the linear
// operation of a decode step; Sec. 2.2: the k-bit model is the top k planes of the parent), for one right-hand
// side or a small group of them.
//
// Work split: one 64-lane wavefront (= one workgroup) streams row quads b, b + nblocks, ... strip by strip
// (strip = 4 rows x 64 words of 32 columns).  A lane loads one 128-bit value per plane and strip, so a wavefront
// load is 1 KiB of contiguous memory per plane; only planes 0..k-1 are read.  The loads of strip t+1 (also
// across row-quad boundaries) are in flight while strip t is decoded.
//
// Decoding: the layout keeps the k bits of a weight at adjacent descending positions of planes 0..k-1
// (see layout_device.hpp), so code fields are built by mask-merging whole plane words (v_bfi_b32), never
// bit by bit:
//   k = 3   : three instructions per word give four bytes [a2 a1 a0 b2 b1 b0 0 0]: the byte is the LDS offset
//             of entry (a,b) of a per-row table of fp16 pairs (64 entries); one LDS read returns both
//             weights packed, one v_dot2_f32_f16 multiplies them with the packed activations (2i, 2i+1).
//   k = 4   : the 4-bit code words are bytes 16 a + b of two weights four positions apart; a 256-entry pair
//             table per row is built in LDS from the row's 16 centroids; activations are re-paired to match.
//   k >= 5  : a three-level merge tree (2-, 4-, 8-bit fields) gives eight words of four bytes [code << s];
//             the byte is the LDS offset into the row's table (k = 5: fp32 entries, k >= 6: fp16 entries); one
//             multiply-add per weight.
// The per-row tables sit in LDS (wavefront-private: 1 KiB..4 KiB per row quad); activations are read from
// global memory (L1/L2 hits) straight into packed registers, because LDS lookups are the scarcest resource.
// All accumulation is fp32; the four row sums are reduced across the wavefront with DPP adds.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

#include "layout_device.hpp"

namespace dpllm {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

struct GemvJob {
  const char* arena;          // device planes start here; plane b at + b * plane_stride_u4 * 16 bytes
  const uint16_t* x;          // fp16 [in]
  uint16_t* y;                // fp16 [out]
  const int32_t* k_dev;       // nullptr: serve ka; else *k_dev is ka or kb
  uint32_t plane_stride_u4;
  uint32_t lut_off_a, lut_off_b;  // byte offsets of the ka / kb tables inside the arena
  int32_t ka, kb;
  int32_t out, ncw, nrq;
  int32_t nblocks;            // workgroups of this job; workgroup b streams row quads b, b + nblocks, ...
  int32_t block_start;        // index of this job's first workgroup inside a multi-job grid
  int32_t nsamples;           // right-hand sides served together (1..NB): sample s reads x + s * in, writes y + s * out
  int32_t ncc;                // row-per-lane layout: 128-column tiles per row (there nrq counts blocks of 64 rows)
  // row-per-lane layout, column split: nsplit workgroups share every block of rows, each taking 1 / nsplit of its
  // column tiles (nblocks counts all of them).  Their fp32 partial sums meet in ws ([row block][sample][split]
  // [64 rows]); cnt ([row block][sample], zero between launches) tells the last one to arrive, which adds them up.
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

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_add(float v) {
  int moved = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, ROW_MASK, 0xf, false);
  return v + __builtin_bit_cast(float, moved);
}

// sum over the 64 lanes; the total is valid in lane 63
__device__ __forceinline__ float wave_sum_to_lane63(float v) {
  v = dpp_add<0xB1, 0xf>(v);   // quad_perm [1,0,3,2]
  v = dpp_add<0x4E, 0xf>(v);   // quad_perm [2,3,0,1]
  v = dpp_add<0x141, 0xf>(v);  // row_half_mirror
  v = dpp_add<0x140, 0xf>(v);  // row_mirror: every lane of a 16-lane row holds the row sum
  v = dpp_add<0x142, 0xa>(v);  // row_bcast15 into rows 1 and 3
  v = dpp_add<0x143, 0xc>(v);  // row_bcast31 into rows 2 and 3
  return v;
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

// ---- per-bitwidth decode scheme (all compile-time) ----------------------------------------------------
// kPair : k = 3, byte = 4 * (8 a + b); k = 4, byte = 16 a + b: table of fp16 pairs (LUT[a], LUT[b]), one
//         v_dot2_f32_f16 per two weights
// kF32  : k = 5, byte = code << 2, table of fp32 values, v_fma_f32 (activations converted once per strip)
// kF16  : k >= 6, byte = code << 1 (k = 8: code), table of fp16 values, v_fma_mix_f32
enum class Scheme { kPair, kF32, kF16 };
template <int K>
struct Decode {
  static constexpr Scheme scheme = (K <= 4) ? Scheme::kPair : (K <= 5 ? Scheme::kF32 : Scheme::kF16);
  static constexpr int shift = (scheme == Scheme::kF32) ? 2 : 1;        // log2 of the table entry size
  static constexpr int d = (K == 8) ? 0 : 8 - K - shift;                 // plane b uses merge-tree slot b + d
  // LDS bytes of one row's table (pair tables: 4^k entries of 4 bytes)
  static constexpr int row_bytes = (K == 3) ? 256 : (K == 4) ? 1024 : ((1 << K) << shift);
  // byte field of column `col`: which of the eight merged words, and which byte after the alignment rotation
  __host__ __device__ static constexpr int top(int col) { return (col_to_pos(col) + d) & 31; }
  __host__ __device__ static constexpr int word(int col) { return top(col) & 7; }
  __host__ __device__ static constexpr int rot(int c) { return (c + 1) & 7; }
  __host__ __device__ static constexpr int byte(int col) { return ((top(col) - rot(word(col))) & 31) >> 3; }
};

// planes of one row -> eight words, each four byte-aligned fields [code << shift]
template <int K, int D = Decode<K>::d>
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

// k = 3: planes of one row -> four words of four bytes 4 * (8 a + b), columns (2i, 2i+1), i = 4 jj + n
__device__ __forceinline__ void merge_pair_fields(const uint32_t (&w)[3], uint32_t (&T)[4]) {
#pragma unroll
  for (int jj = 0; jj < 4; ++jj) {
    const uint32_t m0 = rotl_c(0x90909090u, 2 * jj), m1 = rotl_c(0x48484848u, 2 * jj), m2 = rotl_c(0x24242424u, 2 * jj);
    // three instructions per word; written as instructions because the compiler rewrites the expression into
    // three ANDs and a three-way OR
    uint32_t o = bfi_insn(m0, w[0], bfi_insn(m1, w[1], w[2] & m2));
    T[jj] = jj ? __builtin_rotateright32(o, 2 * jj) : o;
  }
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

// columns of the two weights in byte m of word c of merge_nibble_pairs: upper nibble, lower nibble
__host__ __device__ constexpr int nibble_pair_col_hi(int c, int m) { return pos_to_col((8 * m + 7 + ((c + 1) & 3)) & 31); }
__host__ __device__ constexpr int nibble_pair_col_lo(int c, int m) { return pos_to_col((8 * m + 3 + ((c + 1) & 3)) & 31); }

// activations re-paired to match merge_nibble_pairs: xq[4 c + m] = (x[col_hi], x[col_lo]), one v_perm_b32 each
template <int I>
__device__ __forceinline__ void nibble_pair_x(const uint32_t (&xp)[16], uint32_t (&xq)[16]) {
  if constexpr (I < 16) {
    constexpr int ca = nibble_pair_col_hi(I / 4, I % 4), cb = nibble_pair_col_lo(I / 4, I % 4);
    constexpr uint32_t ba = 4 + 2 * (ca & 1), bb = 2 * (cb & 1);   // first byte of the wanted half in {src0, src1}
    constexpr uint32_t sel = ba | ((ba + 1) << 8) | (bb << 16) | ((bb + 1) << 24);
    xq[I] = __builtin_amdgcn_perm(xp[ca / 2], xp[cb / 2], sel);
    nibble_pair_x<I + 1>(xp, xq);
  }
}

// byte n of a word (optionally doubled).  A wavefront issues about one instruction per five cycles whatever
// the opcode, so the middle bytes use one v_bfe_u32 rather than a shift and a mask.
template <int N, bool TIMES2 = false>
__device__ __forceinline__ uint32_t byte_of(uint32_t w) {
  if constexpr (TIMES2) {
    if constexpr (N == 0) return (w << 1) & 0x1feu;
    else return (w >> (8 * N - 1)) & 0x1feu;
  } else {
    if constexpr (N == 0) return w & 0xffu;
    else if constexpr (N == 3) return w >> 24;
    else {
      uint32_t r;
      asm("v_bfe_u32 %0, %1, %2, 8" : "=v"(r) : "v"(w), "n"(8 * N));
      return r;
    }
  }
}

__device__ __forceinline__ void sched_fence() { __builtin_amdgcn_sched_barrier(0); }

template <int K>
struct PlaneStrip {
  u32x4 w[K];   // 4 rows x 32 columns of planes 0..K-1
};
template <int NB>
struct XStrip {
  u32x4 x[NB][4];   // per right-hand side: the lane's 32 activations as 16 fp16 pairs
};

// Loads are never predicated: a lane past the end of a ragged strip re-reads the last word (its result is
// discarded at compute time).  Unconditional issue keeps the compiler's outstanding-load counts exact, so
// it waits only for the strip it is about to decode and leaves the prefetched ones in flight.
// `real` = false (ring slots past the end of the run): the K loads still issue, but from the activation
// vector, which is hot in L2, so they cost no HBM traffic; the values are never decoded.
template <int K>
__device__ __forceinline__ void load_planes(PlaneStrip<K>& s, const GemvJob& job, int rq, int cw, bool real = true) {
  const int cwc = min(cw, job.ncw - 1);
  const DPLLM_GLOBAL u32x4* planes = as_global(reinterpret_cast<const u32x4*>(job.arena)) + (size_t)rq * job.ncw + cwc;
  const DPLLM_GLOBAL u32x4* xs = as_global(reinterpret_cast<const u32x4*>(job.x)) + (size_t)cwc * 4;
  const DPLLM_GLOBAL u32x4* p = real ? planes : xs;
  const size_t step = real ? (size_t)job.plane_stride_u4 : 0;
#pragma unroll
  for (int b = 0; b < K; ++b) s.w[b] = load_stream(p + (size_t)b * step);
}

template <int NB>
__device__ __forceinline__ void load_x(XStrip<NB>& s, const GemvJob& job, int cw) {
  const int cwc = min(cw, job.ncw - 1);
#pragma unroll
  for (int b = 0; b < NB; ++b) {
    // a group with fewer than NB samples re-reads its last one (the sums are not stored)
    const int sample = NB == 1 ? 0 : min(b, job.nsamples - 1);
    const DPLLM_GLOBAL u32x4* xp = as_global(reinterpret_cast<const u32x4*>(job.x)) + ((size_t)sample * job.ncw + cwc) * 4;
#pragma unroll
    for (int i = 0; i < 4; ++i) s.x[b][i] = xp[i];
  }
}

// Orders the LDS table writes of a wavefront against its own lookups.  A workgroup is a single wavefront and
// the LDS executes one wavefront's operations in issue order, so only the compiler has to be held back; no
// counter wait is wanted here (a workgroup barrier would also drain the prefetched global loads).
__device__ __forceinline__ void lds_order() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <int K>
__host__ __device__ constexpr int row_table_bytes() { return Decode<K>::row_bytes; }
template <int KA, int KB>
__host__ __device__ constexpr int lds_bytes() {
  // + 128: staging area of the k = 4 raw tables
  return 4 * (row_table_bytes<KA>() > row_table_bytes<KB>() ? row_table_bytes<KA>() : row_table_bytes<KB>()) + 128;
}

// Lookups run as a software pipeline of chunks of 8: the LDS reads of chunk c+1 are issued before the
// multiply-adds of chunk c, so LDS latency overlaps ALU work inside one wavefront.
// Chunk (jj, r) of the byte-field schemes: columns 8 jj .. 8 jj + 7 of row r.
template <int K, int JJ>
__device__ __forceinline__ void issue_chunk(const uint32_t (&R)[8], const char* tbl, uint32_t (&v)[8]) {
  using D = Decode<K>;
#define DPLLM_LOOKUP(N)                                                                                   \
  {                                                                                                       \
    constexpr int ce = 8 * JJ + 2 * N, co = ce + 1;                                                       \
    uint32_t fe = byte_of<D::byte(ce), K == 8>(R[D::word(ce)]), fo = byte_of<D::byte(co), K == 8>(R[D::word(co)]); \
    if constexpr (D::scheme == Scheme::kF32) {                                                            \
      v[2 * N] = *reinterpret_cast<const uint32_t*>(tbl + fe);                                            \
      v[2 * N + 1] = *reinterpret_cast<const uint32_t*>(tbl + fo);                                        \
    } else {                                                                                              \
      v[2 * N] = *reinterpret_cast<const uint16_t*>(tbl + fe);                                            \
      v[2 * N + 1] = *reinterpret_cast<const uint16_t*>(tbl + fo);                                        \
    }                                                                                                     \
  }
  DPLLM_LOOKUP(0) DPLLM_LOOKUP(1) DPLLM_LOOKUP(2) DPLLM_LOOKUP(3)
#undef DPLLM_LOOKUP
}

template <int K>
__device__ __forceinline__ void consume_chunk(const uint32_t (&v)[8], const uint32_t* xp4, const float (&xf)[8],
                                              float& acc0, float& acc1) {
  using D = Decode<K>;
  // last lookup first: LDS answers in issue order, so one counter wait covers the chunk
#pragma unroll
  for (int n = 3; n >= 0; --n) {
    if constexpr (D::scheme == Scheme::kF32) {
      acc1 = __builtin_fmaf(__builtin_bit_cast(float, v[2 * n + 1]), xf[2 * n + 1], acc1);
      acc0 = __builtin_fmaf(__builtin_bit_cast(float, v[2 * n]), xf[2 * n], acc0);
    } else {
      half2_t xv = __builtin_bit_cast(half2_t, xp4[n]);
      acc1 = __builtin_fmaf((float)__builtin_bit_cast(_Float16, (uint16_t)v[2 * n + 1]), (float)xv.y, acc1);
      acc0 = __builtin_fmaf((float)__builtin_bit_cast(_Float16, (uint16_t)v[2 * n]), (float)xv.x, acc0);
    }
  }
}

// rows 2H, 2H+1 of the strip: chunk C = 2 * jj + rr uses buffer va; the next chunk is issued into vb first
template <int K, int NB, int H, int C>
__device__ __forceinline__ void byte_pipeline(const uint32_t (&R)[2][8], const uint32_t (&xp)[NB][16], const char* lds,
                                              uint32_t (&va)[8], uint32_t (&vb)[8], float (&xf)[NB][8], float (&acc)[NB][8]) {
  if constexpr (C < 8) {
    constexpr int jj = C / 2, rr = C % 2, row = 2 * H + rr;
    if constexpr (C + 1 < 8)
      issue_chunk<K, (C + 1) / 2>(R[(C + 1) % 2], lds + (2 * H + (C + 1) % 2) * Decode<K>::row_bytes, vb);
    sched_fence();
#pragma unroll
    for (int b = 0; b < NB; ++b) {
      if constexpr (Decode<K>::scheme == Scheme::kF32 && rr == 0) {
#pragma unroll
        for (int n = 0; n < 4; ++n) {
          half2_t xv = __builtin_bit_cast(half2_t, xp[b][4 * jj + n]);
          xf[b][2 * n] = (float)xv.x;
          xf[b][2 * n + 1] = (float)xv.y;
        }
      }
      consume_chunk<K>(va, &xp[b][4 * jj], xf[b], acc[b][2 * row], acc[b][2 * row + 1]);
    }
    sched_fence();
    byte_pipeline<K, NB, H, C + 1>(R, xp, lds, vb, va, xf, acc);
  }
}

template <int K, int NB, int H>
__device__ __forceinline__ void byte_rows(const PlaneStrip<K>& s, const uint32_t (&xp)[NB][16], const char* lds,
                                          float (&acc)[NB][8]) {
  uint32_t R[2][8];
#pragma unroll
  for (int rr = 0; rr < 2; ++rr) {
    uint32_t w[K];
#pragma unroll
    for (int b = 0; b < K; ++b) w[b] = s.w[b][2 * H + rr];
    merge_byte_fields<K>(w, R[rr]);
  }
  uint32_t va[8], vb[8];
  float xf[NB][8];
  issue_chunk<K, 0>(R[0], lds + 2 * H * Decode<K>::row_bytes, va);
  byte_pipeline<K, NB, H, 0>(R, xp, lds, va, vb, xf, acc);
}

// LDS offset of the pair entry named by byte n of a merged word: k = 3 bytes are pre-scaled, k = 4 bytes are
// entry numbers (the compiler selects the byte and scales it in one SDWA shift)
template <int K, int N>
__device__ __forceinline__ uint32_t pair_offset(uint32_t t) {
  if constexpr (K == 3) return byte_of<N>(t);
  else return ((t >> (8 * N)) & 0xffu) << 2;
}

// pair schemes, chunk C = 2 * jj + half: rows 2 half, 2 half + 1, four pair lookups each from word jj
template <int K, int C>
__device__ __forceinline__ void issue_pair_chunk(const uint32_t (&T)[4][4], const char* lds, uint32_t (&v)[8]) {
  constexpr int jj = C / 2, r0 = 2 * (C % 2);
#pragma unroll
  for (int rr = 0; rr < 2; ++rr) {
    const uint32_t t = T[r0 + rr][jj];
    const char* tbl = lds + (r0 + rr) * Decode<K>::row_bytes;
    v[4 * rr + 0] = *reinterpret_cast<const uint32_t*>(tbl + pair_offset<K, 0>(t));
    v[4 * rr + 1] = *reinterpret_cast<const uint32_t*>(tbl + pair_offset<K, 1>(t));
    v[4 * rr + 2] = *reinterpret_cast<const uint32_t*>(tbl + pair_offset<K, 2>(t));
    v[4 * rr + 3] = *reinterpret_cast<const uint32_t*>(tbl + pair_offset<K, 3>(t));
  }
}

template <int K, int NB, int C>
__device__ __forceinline__ void pair_pipeline(const uint32_t (&T)[4][4], const uint32_t (&xp)[NB][16], const char* lds,
                                              uint32_t (&va)[8], uint32_t (&vb)[8], float (&acc)[NB][8]) {
  if constexpr (C < 8) {
    constexpr int jj = C / 2, r0 = 2 * (C % 2);
    if constexpr (C + 1 < 8) issue_pair_chunk<K, C + 1>(T, lds, vb);
    sched_fence();
    // LDS answers in issue order: consuming the chunk's last lookup first lets one counter wait cover all eight
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
      for (int rr = 1; rr >= 0; --rr)
#pragma unroll
        for (int n = 3; n >= 0; --n) {
          float& a = acc[b][2 * (r0 + rr) + (n & 1)];
          a = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, va[4 * rr + n]), __builtin_bit_cast(half2_t, xp[b][4 * jj + n]), a, false);
        }
    sched_fence();
    pair_pipeline<K, NB, C + 1>(T, xp, lds, vb, va, acc);
  }
}

template <int K, int NB>
__device__ __forceinline__ void compute_strip(const PlaneStrip<K>& s, const XStrip<NB>& xs, int cw, int ncw, const char* lds,
                                              float (&acc)[NB][8]) {
  if (cw >= ncw) return;
  uint32_t xp[NB][16];
#pragma unroll
  for (int b = 0; b < NB; ++b)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      xp[b][4 * i + 0] = xs.x[b][i].x;
      xp[b][4 * i + 1] = xs.x[b][i].y;
      xp[b][4 * i + 2] = xs.x[b][i].z;
      xp[b][4 * i + 3] = xs.x[b][i].w;
    }
  if constexpr (K == 3) {
    uint32_t va[8], vb[8];
    uint32_t T[4][4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const uint32_t w[3] = {s.w[0][r], s.w[1][r], s.w[2][r]};
      merge_pair_fields(w, T[r]);
    }
    issue_pair_chunk<3, 0>(T, lds, va);
    pair_pipeline<3, NB, 0>(T, xp, lds, va, vb, acc);
  } else if constexpr (K == 4) {
    uint32_t va[8], vb[8];
    uint32_t T[4][4], xq[NB][16];
#pragma unroll
    for (int b = 0; b < NB; ++b) nibble_pair_x<0>(xp[b], xq[b]);
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const uint32_t w[4] = {s.w[0][r], s.w[1][r], s.w[2][r], s.w[3][r]};
      merge_nibble_pairs(w, T[r]);
    }
    issue_pair_chunk<4, 0>(T, lds, va);
    pair_pipeline<4, NB, 0>(T, xq, lds, va, vb, acc);
  } else {
    byte_rows<K, NB, 0>(s, xp, lds, acc);
    byte_rows<K, NB, 1>(s, xp, lds, acc);
  }
}

// The tables of one row quad, fetched one row quad ahead into registers and written to LDS at the boundary.
template <int K>
struct TableRegs {
  // per lane: k = 3 one pair entry per row; k = 4 one dword of the raw tables (the pair entries are formed
  // at store time); fp32 tables one entry per register; fp16 tables two
  static constexpr int kEntries = 4 << K;  // table entries of a row quad
  static constexpr int kDwords = (K == 3) ? 4 : (K == 4) ? 1
                               : (Decode<K>::scheme == Scheme::kF32 ? (kEntries + 63) / 64 : (kEntries / 2 + 63) / 64);
  uint32_t v[kDwords];
};

template <int K>
__device__ __forceinline__ void fetch_tables(TableRegs<K>& t, const DPLLM_GLOBAL uint16_t* lut_base, int rq, int lane) {
  const DPLLM_GLOBAL uint16_t* lut = lut_base + ((size_t)rq * 4 << K);
  if constexpr (K == 3) {
    const int a = lane >> 3, b = lane & 7;
#pragma unroll
    for (int r = 0; r < 4; ++r) t.v[r] = (uint32_t)lut[r * 8 + a] | ((uint32_t)lut[r * 8 + b] << 16);
  } else if constexpr (K == 4) {
    t.v[0] = reinterpret_cast<const DPLLM_GLOBAL uint32_t*>(lut)[lane & 31];   // 4 rows x 16 fp16 = 32 dwords
  } else if constexpr (Decode<K>::scheme == Scheme::kF32) {
    constexpr int entries = TableRegs<K>::kEntries;
#pragma unroll
    for (int i = 0; i < TableRegs<K>::kDwords; ++i) {
      int e = i * 64 + lane;
      t.v[i] = (entries >= 64 || e < entries) ? (uint32_t)lut[e] : 0u;
    }
  } else {
    constexpr int dwords = TableRegs<K>::kEntries / 2;
    const DPLLM_GLOBAL uint32_t* src = reinterpret_cast<const DPLLM_GLOBAL uint32_t*>(lut);
#pragma unroll
    for (int i = 0; i < TableRegs<K>::kDwords; ++i) {
      int e = i * 64 + lane;
      t.v[i] = (dwords >= 64 || e < dwords) ? src[e] : 0u;
    }
  }
}

template <int K>
__device__ __forceinline__ void store_tables(const TableRegs<K>& t, char* lds, int lane) {
  uint32_t* dst = reinterpret_cast<uint32_t*>(lds);
  if constexpr (K == 3) {
#pragma unroll
    for (int r = 0; r < 4; ++r) dst[r * 64 + lane] = t.v[r];
  } else if constexpr (K == 4) {
    // the raw tables go to a 128-byte staging area behind the four pair tables; lane (g, b) = (lane / 16,
    // lane % 16) then forms the entries (a, b), a = 4 g .. 4 g + 3, of every row
    uint32_t* raw = dst + 4 * (Decode<4>::row_bytes / 4);
    if (lane < 32) raw[lane] = t.v[0];
    lds_order();
    const int b = lane & 15, g = lane >> 4;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const uint16_t* row = reinterpret_cast<const uint16_t*>(raw) + r * 16;
      const uint32_t lb = (uint32_t)row[b] << 16;
      const u32x2 la = *reinterpret_cast<const u32x2*>(row + 4 * g);
      uint32_t* out = dst + r * 256 + 64 * g + b;
      out[0] = (la.x & 0xffffu) | lb;
      out[16] = (la.x >> 16) | lb;
      out[32] = (la.y & 0xffffu) | lb;
      out[48] = (la.y >> 16) | lb;
    }
  } else if constexpr (Decode<K>::scheme == Scheme::kF32) {
    constexpr int entries = TableRegs<K>::kEntries;
#pragma unroll
    for (int i = 0; i < TableRegs<K>::kDwords; ++i) {
      int e = i * 64 + lane;
      float f = (float)__builtin_bit_cast(_Float16, (uint16_t)t.v[i]);
      if (entries >= 64 || e < entries) dst[e] = __builtin_bit_cast(uint32_t, f);
    }
  } else {
    constexpr int dwords = TableRegs<K>::kEntries / 2;
#pragma unroll
    for (int i = 0; i < TableRegs<K>::kDwords; ++i) {
      int e = i * 64 + lane;
      if (dwords >= 64 || e < dwords) dst[e] = t.v[i];
    }
  }
}

template <int NB>
__device__ __forceinline__ void finish_rowquad(const GemvJob& job, int rq, int lane, float (&acc)[NB][8]) {
#pragma unroll
  for (int b = 0; b < NB; ++b) {
    float s[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      s[r] = wave_sum_to_lane63(acc[b][2 * r] + acc[b][2 * r + 1]);
      acc[b][2 * r] = acc[b][2 * r + 1] = 0.f;
    }
    if (lane == 63 && (NB == 1 || b < job.nsamples)) {
      half2_t lo = {(_Float16)s[0], (_Float16)s[1]}, hi = {(_Float16)s[2], (_Float16)s[3]};
      DPLLM_GLOBAL uint16_t* y = as_global(job.y) + (size_t)b * job.out + (size_t)rq * 4;
      if (rq * 4 + 4 <= job.out && (reinterpret_cast<uintptr_t>(y) & 7) == 0) {
        u32x2 v = {__builtin_bit_cast(uint32_t, lo), __builtin_bit_cast(uint32_t, hi)};
        *reinterpret_cast<DPLLM_GLOBAL u32x2*>(y) = v;
      } else {
#pragma unroll
        for (int r = 0; r < 4; ++r)
          if (rq * 4 + r < job.out) y[r] = __builtin_bit_cast(uint16_t, (_Float16)s[r]);
      }
    }
  }
}

// One wavefront streams row quads [rq0, rq1) of a job.  Plane strips travel through a ring of D register
// buffers: the loads of strips t+1 .. t+D-1 are in flight while strip t is decoded (HBM latency under load
// is several microseconds, so about 100 KiB per compute unit must be in flight to keep the memory busy).
// XS = true (exactly two strips per row): the activations of both strips stay in registers for the whole
// run.  XS = false: activations ride in a ring of their own, fetched with the planes (L2 hits).
template <int K, int D, bool XS, int NB>
struct StreamState {
  static_assert(!XS || D % 2 == 0, "resident activations are picked by ring-slot parity");
  PlaneStrip<K> pb[D];
  XStrip<NB> xb[XS ? 2 : D];
  TableRegs<K> tr;
  float acc[NB][8];
  int rq0, stride;
  int lrq, lc0, lt;   // load cursor: row quad, first word of the strip, strip counter
  int crq, cc0, ct;   // compute cursor
  int total;
};

template <int K, int D, bool XS, int NB, int I>
__device__ __forceinline__ bool stream_step(StreamState<K, D, XS, NB>& st, const GemvJob& job,
                                            const DPLLM_GLOBAL uint16_t* lut_base, int rq_last, int lane, char* lds) {
  const int ncw = job.ncw;
  constexpr int slot = (I + D - 1) % D;
  {
    // past the end of the run the slot is refilled with dummy loads (see load_planes)
    const bool more = st.lt < st.total;
    const int lrq = more ? st.lrq : st.rq0, lc0 = more ? st.lc0 : 0;
    load_planes<K>(st.pb[slot], job, lrq, lc0 + lane, more);
    if constexpr (!XS) load_x(st.xb[slot], job, lc0 + lane);
    if (more) {
      st.lt++;
      st.lc0 += 64;
      if (st.lc0 >= ncw) { st.lc0 = 0; st.lrq += st.stride; }
    }
  }
  compute_strip<K, NB>(st.pb[I], st.xb[XS ? (I & 1) : I], st.cc0 + lane, ncw, lds, st.acc);
  st.cc0 += 64;
  if (st.cc0 >= ncw) {
    finish_rowquad<NB>(job, st.crq, lane, st.acc);
    st.cc0 = 0;
    st.crq += st.stride;
    if (st.crq <= rq_last) {
      lds_order();
      store_tables<K>(st.tr, lds, lane);
      fetch_tables<K>(st.tr, lut_base, min(st.crq + st.stride, rq_last), lane);
      lds_order();
    }
  }
  return ++st.ct == st.total;
}

template <int K, int D, bool XS, int NB, int I>
__device__ __forceinline__ bool stream_round(StreamState<K, D, XS, NB>& st, const GemvJob& job,
                                             const DPLLM_GLOBAL uint16_t* lut_base, int rq_last, int lane, char* lds) {
  if constexpr (I < D) {
    if (stream_step<K, D, XS, NB, I>(st, job, lut_base, rq_last, lane, lds)) return true;
    return stream_round<K, D, XS, NB, I + 1>(st, job, lut_base, rq_last, lane, lds);
  } else {
    return false;
  }
}

template <int K, int D, bool XS, int NB>
__device__ __forceinline__ void gemv_stream(const GemvJob& job, uint32_t lut_off, int rq0, int stride, int nq, int lane,
                                            char* lds) {
  const DPLLM_GLOBAL uint16_t* lut_base = as_global(reinterpret_cast<const uint16_t*>(job.arena + lut_off));
  const int ncw = job.ncw;
  StreamState<K, D, XS, NB> st;
  const int ns = (ncw + 63) >> 6;
  const int rq_last = rq0 + (nq - 1) * stride;
  st.total = nq * ns;
  st.rq0 = rq0;
  st.stride = stride;
  st.lrq = rq0; st.lc0 = 0; st.lt = 0;
  st.crq = rq0; st.cc0 = 0; st.ct = 0;
#pragma unroll
  for (int i = 0; i < D - 1; ++i) {
    const bool more = st.lt < st.total;
    const int lrq = more ? st.lrq : rq0, lc0 = more ? st.lc0 : 0;
    load_planes<K>(st.pb[i], job, lrq, lc0 + lane, more);
    if constexpr (!XS) load_x(st.xb[i], job, lc0 + lane);
    if (more) {
      st.lt++;
      st.lc0 += 64;
      if (st.lc0 >= ncw) { st.lc0 = 0; st.lrq += stride; }
    }
  }
  if constexpr (XS) {
    load_x(st.xb[0], job, lane);
    load_x(st.xb[1], job, 64 + lane);
  }
  fetch_tables<K>(st.tr, lut_base, rq0, lane);
  store_tables<K>(st.tr, lds, lane);
  fetch_tables<K>(st.tr, lut_base, min(rq0 + stride, rq_last), lane);
  lds_order();
#pragma unroll
  for (int b = 0; b < NB; ++b)
#pragma unroll
    for (int r = 0; r < 8; ++r) st.acc[b][r] = 0.f;
  while (!stream_round<K, D, XS, NB, 0>(st, job, lut_base, rq_last, lane, lds)) {
  }
}

template <int K, int NB>
__device__ __forceinline__ void gemv_stream_any(const GemvJob& job, uint32_t lut_off, int rq0, int stride, int nq, int lane,
                                                char* lds) {
  // Ring depth 2 (one strip in flight behind the one being decoded) measured best at every k: deeper rings
  // cost registers (hence resident wavefronts) and put more requests in flight than the memory system likes.
  constexpr int kDepthXS = 2;   // even: ring slot parity must equal strip parity
  constexpr int kDepthRing = 2;
  // several right-hand sides: their activations always ride the ring (registers)
  if (NB == 1 && job.ncw > 64 && job.ncw <= 128)
    gemv_stream<K, kDepthXS, NB == 1, NB>(job, lut_off, rq0, stride, nq, lane, lds);
  else
    gemv_stream<K, kDepthRing, false, NB>(job, lut_off, rq0, stride, nq, lane, lds);
}

template <int KA, int KB, int NB>
__device__ __forceinline__ void gemv_block(const GemvJob& job, int block, int lane, char* lds) {
  // Workgroups that run at the same time take neighbouring row quads, so the chip reads one moving window
  // of each plane instead of thousands of separate streams.
  const int rq0 = block, stride = job.nblocks;
  const int nq = (job.nrq - block + job.nblocks - 1) / job.nblocks;
  if (nq <= 0) return;
  if constexpr (KA != KB) {
    if (job.k_dev != nullptr && __builtin_amdgcn_readfirstlane(*as_global(job.k_dev)) == KB) {
      gemv_stream_any<KB, NB>(job, job.lut_off_b, rq0, stride, nq, lane, lds);
      return;
    }
  }
  gemv_stream_any<KA, NB>(job, job.lut_off_a, rq0, stride, nq, lane, lds);
}

// jobs == nullptr: the job passed by value, for njobs right-hand sides in groups of NB that share one pass
// over the planes (group g reads x + g * NB * in and writes y + g * NB * out; workgroups [g * nblocks,
// (g + 1) * nblocks) serve it); else (NB = 1) block b belongs to job block_jobs[b] of the table
template <int KA, int KB, int NB>
__global__ void __launch_bounds__(64) gemv_kernel(const GemvJob* __restrict__ jobs, const int32_t* __restrict__ block_jobs,
                                                                 int njobs, GemvJob one) {
  __shared__ __attribute__((aligned(16))) char lds[lds_bytes<KA, KB>()];
  if (jobs == nullptr) {
    const int group = blockIdx.x / one.nblocks;
    one.x += (size_t)group * NB * one.ncw * 32;
    one.y += (size_t)group * NB * one.out;
    one.nsamples = min(NB, njobs - group * NB);
    gemv_block<KA, KB, NB>(one, blockIdx.x - group * one.nblocks, threadIdx.x, lds);
    return;
  }
  if constexpr (NB == 1) {
    const int b = blockIdx.x;
    GemvJob job = jobs[block_jobs[b]];
    gemv_block<KA, KB, 1>(job, b - job.block_start, threadIdx.x, lds);
  }
}

}  // namespace dpllm
