// Private device layout of one quantised linear (gfx950).
//
// Planes stay separable, so a k-bit GEMV touches the first k plane regions only (the
// overlay of Sec. 2.2 of the paper).  Inside a plane:
//   * rows are grouped in quads; the four words of a quad that cover the same 32 columns
//     are adjacent, so one 128-bit load gives a lane 4 rows x 32 columns of one plane, and
//     64 consecutive lanes read 1 KiB of contiguous memory;
//   * the word of plane b is the canonical word rotated right by b bits: bit q of the stored
//     word holds column (q + b) mod 32.  The k bits of one weight then sit at descending
//     adjacent positions q, q-1, ..., q-k+1 of planes 0..k-1, and whole code fields are
//     assembled with mask-merge instructions and no per-plane shifts, for every k.
// Rows are padded to a multiple of 4 with zero words; tables are padded with zero rows.
//
// A second arrangement of the same words (kLayoutRowLane) serves the row-per-lane GEMV: a plane is cut into
// tiles of 64 rows x 128 columns; the tile stores, row after row, the four 32-column words of that row, so
// lane l of a wavefront reads its own row's 16 bytes and the wavefront reads 1 KiB of contiguous memory.
// Rows are padded to a multiple of 64, columns to a multiple of 128, with zero words.
#pragma once
#include <cstddef>
#include <cstdint>

namespace dpllm {

constexpr size_t kAlign = 256;
constexpr int kLayoutRowQuad = 0, kLayoutRowLane = 1;
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

struct LinearLayout {
  int out = 0, in = 0, p = 0, kmin = 0;
  int mode = kLayoutRowQuad;
  int nrq = 0;               // row groups: quads (ceil(out / 4)) or, row-per-lane, blocks of 64 rows
  int ncw = 0;               // 32-column words per row
  int ncc = 0;               // row-per-lane: 128-column tiles per row
  int rows_padded = 0;       // rows of the tables (zero rows appended)
  size_t plane_bytes = 0;    // stride between plane regions
  size_t lut_offset[9] = {}; // byte offset of the k-bit table, k = kmin..p
  size_t total_bytes = 0;

  static LinearLayout make(int out, int in, int p, int kmin, int mode = kLayoutRowQuad) {
    LinearLayout L;
    L.out = out; L.in = in; L.p = p; L.kmin = kmin; L.mode = mode;
    L.ncw = in / 32;
    L.ncc = (L.ncw + 3) / 4;
    if (mode == kLayoutRowLane) {
      L.nrq = (out + 63) / 64;
      L.rows_padded = L.nrq * 64;
      L.plane_bytes = (size_t)L.nrq * L.ncc * 1024;
    } else {
      L.nrq = (out + 3) / 4;
      L.rows_padded = L.nrq * 4;
      L.plane_bytes = align_up((size_t)L.nrq * L.ncw * 16, kAlign);
    }
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
