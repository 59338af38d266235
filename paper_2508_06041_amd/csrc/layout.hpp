// Private device layout of one quantised linear (gfx950).
//
// Planes stay separable, so a k-bit GEMV touches the first k plane regions only (the
// overlay of Sec. 2.2 of the paper).  Inside a plane:
//   * the plane is cut into tiles of 64 rows x 128 columns; a tile stores, row after row, the four
//     32-column words of that row, so lane l of a wavefront reads its own row's 16 bytes with one
//     128-bit load and the wavefront reads 1 KiB of contiguous memory;
//   * the word of plane b is the (column-permuted, see layout_device.hpp) canonical word rotated right
//     by b bits: bit q of the stored word holds position (q + b) mod 32.  The k bits of one weight then
//     sit at descending adjacent positions q, q-1, ..., q-k+1 of planes 0..k-1, and whole code fields
//     are assembled with mask-merge instructions and no per-plane shifts, for every k.
// Rows are padded to a multiple of 64, columns to a multiple of 128, with zero words; tables are padded
// with zero rows.
#pragma once
#include <cstddef>
#include <cstdint>

namespace dpllm {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

struct LinearLayout {
  int out = 0, in = 0, p = 0, kmin = 0;
  int nrq = 0;               // blocks of 64 rows
  int ncw = 0;               // 32-column words per row
  int ncc = 0;               // 128-column tiles per row
  int rows_padded = 0;       // rows of the tables (zero rows appended)
  size_t plane_bytes = 0;    // stride between plane regions
  size_t lut_offset[9] = {}; // byte offset of the k-bit table, k = kmin..p
  size_t total_bytes = 0;

  static LinearLayout make(int out, int in, int p, int kmin) {
    LinearLayout L;
    L.out = out; L.in = in; L.p = p; L.kmin = kmin;
    L.ncw = in / 32;
    L.ncc = (L.ncw + 3) / 4;
    L.nrq = (out + 63) / 64;
    L.rows_padded = L.nrq * 64;
    L.plane_bytes = (size_t)L.nrq * L.ncc * 1024;
    size_t off = L.plane_bytes * p;
    for (int k = kmin; k <= p; ++k) {
      L.lut_offset[k] = off;
      off += align_up((size_t)L.rows_padded * ((size_t)1 << k) * 2, kAlign);
    }
    L.total_bytes = off;
    return L;
  }
};

}  // namespace dpllm
