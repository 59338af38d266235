// Bit-level part of the private device layout, shared by the re-tiling kernel and the GEMV kernels.
//
// Inside every 32-column word the columns are first permuted (column c -> position pi(c)), then the
// word of plane b is rotated right by b.  Bit q of the stored word of plane b therefore holds the
// plane-b bit of the weight whose position is (q + b) mod 32: the k bits of a weight sit at adjacent,
// descending bit positions of planes 0..k-1, whatever k is.
//
// pi is chosen so that the two weights whose 3-bit fields land in the same byte of a merged word
// (positions 3 apart) are the columns (2i, 2i+1): a packed fp16 pair of activations then multiplies
// a packed pair of looked-up weights without any shuffling.
#pragma once
#include <cstdint>

namespace dpllm {

// position of column c (0..31) inside its word
__host__ __device__ constexpr int col_to_pos(int c) {
  // natural pair i = c / 2 = 4 * jj + n  ->  byte n of the merged word with phase j = 2 * jj;
  // the even column takes the upper 3-bit field (top bit 8n + j + 7), the odd one the lower (8n + j + 4)
  return (8 * ((c / 2) % 4) + 2 * ((c / 2) / 4) + ((c & 1) ? 4 : 7)) % 32;
}

__host__ __device__ constexpr int pos_to_col(int q) {
  for (int c = 0; c < 32; ++c)
    if (col_to_pos(c) == q) return c;
  return -1;
}

__host__ __device__ constexpr uint32_t permute_word(uint32_t canon) {
  uint32_t v = 0;
  for (int c = 0; c < 32; ++c) v |= ((canon >> c) & 1u) << col_to_pos(c);
  return v;
}

__host__ __device__ constexpr uint32_t unpermute_word(uint32_t stored) {
  uint32_t v = 0;
  for (int c = 0; c < 32; ++c) v |= ((stored >> col_to_pos(c)) & 1u) << c;
  return v;
}

__host__ __device__ constexpr uint32_t rotl_c(uint32_t v, int s) {
  s &= 31;
  return s ? (v << s) | (v >> (32 - s)) : v;
}
__host__ __device__ constexpr uint32_t rotr_c(uint32_t v, int s) { return rotl_c(v, 32 - (s & 31)); }

// positions q with (c - q) mod period < width: the bits a field of `width` planes occupies when its top
// bit sits at a position congruent to c
__host__ __device__ constexpr uint32_t field_mask(int period, int c, int width) {
  uint32_t m = 0;
  for (int q = 0; q < 32; ++q)
    if ((((c - q) % period) + period) % period < width) m |= 1u << q;
  return m;
}

// index (in 32-bit words, from the start of a plane) of the word holding columns 32 cw .. 32 cw + 31 of row o:
// [block of 64 rows][tile of 4 words][row][4 words]
__host__ __device__ constexpr size_t plane_word_index(int o, int cw, int ncc) {
  return (((size_t)(o / 64) * ncc + cw / 4) * 64 + o % 64) * 4 + cw % 4;
}

}  // namespace dpllm
