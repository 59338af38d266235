// Any-precision GEMV for gfx950, one row per lane: y[o] = sum_c LUT_k[o][code_k(o,c)] * x[c]   (paper Sec. 3:
// the linear operation of a decode step; Sec. 2.2: the k-bit model is the top k planes of the parent).
//
// Layout: a plane is cut into tiles of 64 rows x 128 columns; lane l of a wavefront owns row
// 64 rb + l of the tile and reads its four 32-column words with one 128-bit load, so a wavefront load is 1 KiB
// of contiguous memory per plane.  Words are permuted and rotated as in layout_device.hpp.
//
// Why rows on lanes: every lane looks its weights up in its own row's table.  The tables of the 64 rows are
// interleaved in LDS (entry e of row l at byte e * 256 + l * 4), so lane l only ever touches bank l mod 32 and
// lookups are free of bank conflicts whatever the table size; the two-weight tables of k = 3 and k = 4, which
// cost 4 - 6 LDS cycles per lookup when a whole wavefront shares one row's table, cost 2.
// The activations are the same for all lanes.  With every tile a lane fetches one dword of them (256 bytes per
// wavefront); before the tile is decoded the wavefront parks them in a private LDS slot.  A wavefront with at
// most four tiles per row block (rows up to 4096 columns) parks them once for its whole run instead.
// One right-hand side (the decode step): every lane reads back 16 bytes per word (lane l takes the pairs
// 4 (l mod 4) .. + 3) and the multiply-add v_dot2c_f32_f16 reads the pair it needs from the right lane of its quad
// with a DPP quad broadcast: 16 registers hold the 64 pairs of a tile, fp32 accumulation in the lane.
// Several right-hand sides (a small dense contraction: 64 rows x up to 4 samples per wavefront) run on the matrix
// pipe instead: v_mfma_f32_4x4x4_16b_f16 works on 16 blocks of four lanes; with the A operand of one block
// broadcast to all blocks (cbsz = 4, abid = Q) lane L gets
//     acc[i] += sum_n A(lane 4 Q + i)[n] * B(lane L)[n],  n = 0 .. 3,  i = 0 .. 3.
// B = four looked-up weights of the lane's own row; A = the four activations that go with them, held by the
// lanes of quad Q: lane 4 Q + i holds sample i's chunk, acc[i] is sample i's sum.  Quad Q of the wavefront holds
// chunks Q and 16 + Q of the tile's 32 chunks of four activations, so 4 registers carry a tile's activations and
// every lookup serves four samples: up to four right-hand sides share a pass at the cost of one.
// Each lane accumulates its own row: no cross-lane reduction.  A workgroup is eight wavefronts that split the
// columns of the same 64 rows and share the tables; their eight partial sums per row meet in LDS.
//
//   k = 3, 4 : two weights per lookup, tables of 64 / 256 fp16 pairs per row (16 / 64 KiB per workgroup)
//   k >= 5   : one weight per lookup (table of 2^k entries per row, 8 .. 64 KiB), two results packed into one
//              register of the B operand
// One kernel serves every bitwidth from 3 to 8: a workgroup reads the bitwidth of its job (a value, or the word a
// selector wrote in device memory) and branches to the code of that bitwidth.  Every branch stays below 128 vector
// registers and the workgroup's LDS is sized for the largest tables (64 KiB), so two workgroups share a compute
// unit whatever the bitwidth; which bitwidth runs is never a matter for the host.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>
#include <type_traits>

#include "gemv_common.hpp"
#include "layout_device.hpp"

namespace dpllm {

constexpr int kLaneWaves = 8;            // wavefronts per workgroup
constexpr int kLaneThreads = 64 * kLaneWaves;

template <int K>
struct LaneDecode {
  static constexpr bool pair = K <= 4;                        // two weights per lookup
  static constexpr int entries = pair ? (1 << (2 * K)) : (1 << K);
  static constexpr int table_bytes = entries * 256;           // 64 rows interleaved, 4 bytes per row and entry
  static constexpr int share = entries / kLaneWaves;          // entries a wavefront builds per row block
  // single-weight schemes: the byte of column `col` is its code; which of the eight merged words, which byte
  static constexpr int d = 8 - K;
  __host__ __device__ static constexpr int top(int col) { return (col_to_pos(col) + d) & 31; }
  __host__ __device__ static constexpr int word(int col) { return top(col) & 7; }
  __host__ __device__ static constexpr int rot(int c) { return (c + 1) & 7; }
  __host__ __device__ static constexpr int byte(int col) { return ((top(col) - rot(word(col))) & 31) >> 3; }
};
constexpr int kLaneRedBytes = kLaneWaves * 64 * 4;            // the partial sums of the eight wavefronts, per sample
constexpr int kLaneKeepTiles = 4;                             // a wavefront with so few tiles per row block keeps their activations in LDS
constexpr int kLaneTableBytes = 65536;                        // the largest tables: k = 4 (pairs) and k = 8
static_assert(LaneDecode<3>::table_bytes <= kLaneTableBytes && LaneDecode<4>::table_bytes <= kLaneTableBytes &&
              LaneDecode<5>::table_bytes <= kLaneTableBytes && LaneDecode<6>::table_bytes <= kLaneTableBytes &&
              LaneDecode<7>::table_bytes <= kLaneTableBytes && LaneDecode<8>::table_bytes <= kLaneTableBytes, "tables fit");
// NB right-hand sides per pass (1 or 4).  Per wavefront: a 256-byte slot for the parked activations of a tile per
// sample; with one sample, four more for the tiles it keeps across row blocks.
template <int NB>
__host__ __device__ constexpr int lane_x_bytes() { return NB == 1 ? 256 + kLaneKeepTiles * 256 : NB * 256; }
// tables, partial sums, activation slots.  Two things borrow space from the partial sums while these are not in
// use (between the barrier that opens a row block and the stores that close it): the 256 bytes a wavefront needs
// to re-pair the activations at k = 4 (its own partial sums of sample 0), and the word of the column-split
// hand-over (the first word; written after every reader of the partial sums has passed a barrier).  With four
// samples the total is exactly half of a compute unit's LDS.
template <int NB>
__host__ __device__ constexpr int lane_lds_bytes() { return kLaneTableBytes + NB * kLaneRedBytes + kLaneWaves * lane_x_bytes<NB>(); }
static_assert(lane_lds_bytes<4>() <= 81920 && lane_lds_bytes<1>() <= 81920, "two workgroups per compute unit");

// x pair held by lane Q of the quad, times the looked-up pair, added to acc
template <int Q>
__device__ __forceinline__ void dot2_quad(float& acc, uint32_t xreg, uint32_t wpair) {
  static_assert(Q >= 0 && Q < 4, "quad lane");
  if constexpr (Q == 0) asm("v_dot2c_f32_f16_dpp %0, %1, %2 quad_perm:[0,0,0,0] row_mask:0xf bank_mask:0xf" : "+v"(acc) : "v"(xreg), "v"(wpair));
  if constexpr (Q == 1) asm("v_dot2c_f32_f16_dpp %0, %1, %2 quad_perm:[1,1,1,1] row_mask:0xf bank_mask:0xf" : "+v"(acc) : "v"(xreg), "v"(wpair));
  if constexpr (Q == 2) asm("v_dot2c_f32_f16_dpp %0, %1, %2 quad_perm:[2,2,2,2] row_mask:0xf bank_mask:0xf" : "+v"(acc) : "v"(xreg), "v"(wpair));
  if constexpr (Q == 3) asm("v_dot2c_f32_f16_dpp %0, %1, %2 quad_perm:[3,3,3,3] row_mask:0xf bank_mask:0xf" : "+v"(acc) : "v"(xreg), "v"(wpair));
}

typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// acc[i] += sum_n x(lane 4 Q + i)[n] * w[n]: x = four fp16 (what this lane holds matters to the lanes whose Q is
// this lane's quad), w = the four weights {w0.lo, w0.hi, w1.lo, w1.hi} of this lane's row
template <int Q>
__device__ __forceinline__ void mfma_chunk(f32x4& acc, uint64_t x, uint32_t w0, uint32_t w1) {
  static_assert(Q >= 0 && Q < 16, "quad of the wavefront");
  const uint64_t w = (uint64_t)w0 | ((uint64_t)w1 << 32);
  acc = __builtin_amdgcn_mfma_f32_4x4x4f16(__builtin_bit_cast(f16x4, x), __builtin_bit_cast(f16x4, w), acc, 4, Q, 0);
}

// The lane's partial sums.  One sample: four fp32 sums that take turns.  Four samples: two sets of four (sum i
// of a set = sample i) that take turns, so that no matrix instruction waits for the one before it.
template <int NB>
struct LaneAcc;
template <>
struct LaneAcc<1> {
  float v[4];
  __device__ __forceinline__ void zero() { v[0] = v[1] = v[2] = v[3] = 0.f; }
  __device__ __forceinline__ float sum(int) const { return (v[0] + v[1]) + (v[2] + v[3]); }
};
template <>
struct LaneAcc<4> {
  f32x4 v[2];
  __device__ __forceinline__ void zero() { v[0] = v[1] = f32x4{0.f, 0.f, 0.f, 0.f}; }
  __device__ __forceinline__ float sum(int b) const { return v[0][b] + v[1][b]; }
};

// LDS address of entry (byte N of t) in the lane's table column: byte 1 = the entry, byte 0 = lane * 4
template <int N>
__device__ __forceinline__ uint32_t lane_entry_addr(uint32_t t, uint32_t lanecol) {
  constexpr uint32_t sel = 0x0c0c0000u | ((4u + N) << 8);   // {0, 0, t.byteN, lanecol.byte0}
  return __builtin_amdgcn_perm(t, lanecol, sel);
}

// The same for an entry byte whose two high bits are not part of the entry number: byte 1 of addr = byte N of t
// with those bits cleared, in one sub-dword instruction; the other bytes of addr keep what they hold (lane * 4,
// put there once).  mask: 0x3f in a register.
template <int N>
__device__ __forceinline__ void lane_entry_addr_masked(uint32_t t, uint32_t mask, uint32_t& addr) {
  static_assert(N >= 0 && N < 4, "byte");
  if constexpr (N == 0) asm("v_and_b32_sdwa %0, %1, %2 dst_sel:BYTE_1 dst_unused:UNUSED_PRESERVE src0_sel:BYTE_0 src1_sel:DWORD" : "+v"(addr) : "v"(t), "v"(mask));
  if constexpr (N == 1) asm("v_and_b32_sdwa %0, %1, %2 dst_sel:BYTE_1 dst_unused:UNUSED_PRESERVE src0_sel:BYTE_1 src1_sel:DWORD" : "+v"(addr) : "v"(t), "v"(mask));
  if constexpr (N == 2) asm("v_and_b32_sdwa %0, %1, %2 dst_sel:BYTE_1 dst_unused:UNUSED_PRESERVE src0_sel:BYTE_2 src1_sel:DWORD" : "+v"(addr) : "v"(t), "v"(mask));
  if constexpr (N == 3) asm("v_and_b32_sdwa %0, %1, %2 dst_sel:BYTE_1 dst_unused:UNUSED_PRESERVE src0_sel:BYTE_3 src1_sel:DWORD" : "+v"(addr) : "v"(t), "v"(mask));
}

__device__ __forceinline__ uint32_t lds_u32(const char* lds, uint32_t addr) { return *reinterpret_cast<const uint32_t*>(lds + addr); }

// ---- a tile: the lane's row, 128 columns, and the lane's dword of the tile's 128 activations -------------------
template <int K, int NB>
struct LaneTile {
  u32x4 w[K];
  uint32_t x[NB];
};

// the lane's dword of the 128 activations of tile cc (address clamped to the row).  Columns past the end of a
// ragged row hold zero codes, whose centroid is not zero: their activations must read as 0, which lane_mask_x
// sees to when the value is used.  (Masking right after the load would make the wavefront wait for the load,
// and with it for every tile load issued before it, at the point of issue.)
__device__ __forceinline__ uint32_t lane_load_x(const GemvJob& job, int cc, int lane, int sample = 0) {
  const int c = cc * 128 + lane * 2, last = job.ncw * 32 - 2;
  return *reinterpret_cast<const DPLLM_GLOBAL uint32_t*>(as_global(job.x) + (size_t)sample * job.ncw * 32 + min(c, last));
}
__device__ __forceinline__ uint32_t lane_mask_x(const GemvJob& job, int cc, int lane, uint32_t v) {
  return cc * 128 + lane * 2 <= job.ncw * 32 - 2 ? v : 0u;
}

// Loads are never predicated, which keeps the compiler's outstanding-load counts exact.  `real` = false (ring
// slots past the end of the run): the K loads still issue, but all from the first 16 bytes of the activation
// vector, which is hot in L2, so they cost no HBM traffic; the values are never decoded.
template <int K, int NB>
__device__ __forceinline__ void lane_load_tile(LaneTile<K, NB>& t, const GemvJob& job, int rb, int cc, int lane, bool with_x, bool real) {
  const DPLLM_GLOBAL u32x4* planes = as_global(reinterpret_cast<const u32x4*>(job.arena)) + ((size_t)rb * job.ncc + cc) * 64 + lane;
  const DPLLM_GLOBAL u32x4* p = real ? planes : as_global(reinterpret_cast<const u32x4*>(job.x));
  const size_t stride = real ? (size_t)job.plane_stride_u4 : 0;
#pragma unroll
  for (int b = 0; b < K; ++b) t.w[b] = load_stream(p + (size_t)b * stride);
  if (with_x) {
    // a group with fewer than NB samples re-reads its last one (the sums are not stored)
#pragma unroll
    for (int b = 0; b < NB; ++b) t.x[b] = lane_load_x(job, cc, lane, NB == 1 ? 0 : min(b, job.nsamples - 1));
  }
}

// Parks a tile's activations in LDS in the form the lanes read back: 64 dwords, dword 16 j + n = pair n of word
// j; chunk g of the tile (dwords 2 g, 2 g + 1) goes with the lookups of pairs 2 (g mod 8), + 1 of word g / 8.
// k != 4: the natural pairs (2i, 2i+1), so the lane's dword goes straight to `ready`.
// k = 4: the pairs (x[col_hi], x[col_lo]) of merged word q, byte m (see nibble_pair_col_hi / _lo), cut from a
// natural copy in `scratch`.
template <int K>
__device__ __forceinline__ void lane_park_x(uint32_t x, int lane, char* scratch, char* ready) {
  if constexpr (K == 4) {
    *reinterpret_cast<uint32_t*>(scratch + lane * 4) = x;
    lds_order();
    const int j = lane >> 4, q = (lane >> 2) & 3, m = lane & 3, mr = (m + 3) & 3;
    const int ca = q == 0 ? 17 + 2 * m : q == 1 ? 8 + 2 * m : q == 2 ? 25 + 2 * m : 2 * m;
    const int cb = q == 0 ? 1 + 2 * m : q == 1 ? 24 + 2 * mr : q == 2 ? 9 + 2 * m : 16 + 2 * mr;
    const uint32_t lo = *reinterpret_cast<const uint16_t*>(scratch + (j * 32 + ca) * 2);
    const uint32_t hi = *reinterpret_cast<const uint16_t*>(scratch + (j * 32 + cb) * 2);
    *reinterpret_cast<uint32_t*>(ready + lane * 4) = lo | (hi << 16);
  } else {
    *reinterpret_cast<uint32_t*>(ready + lane * 4) = x;
  }
  lds_order();
}

// ---- entry words of one 32-column word -----------------------------------------------------------------------
// k = 3: four words of four bytes (8 a + b) + 64 (two bits of other weights, cleared when the address is formed),
// the pairs (2i, 2i+1), i = 4 jj + n (word 3 is left rotated by one byte: its pair n sits in byte n + 1)
__device__ __forceinline__ void lane_entries3(uint32_t w0, uint32_t w1, uint32_t w2, uint32_t (&T)[4], const MergeMasks<3>& M) {
#pragma unroll
  for (int jj = 0; jj < 4; ++jj) {
    const uint32_t o = bfi_v(M.m[2 * jj], w0, bfi_v(M.m[2 * jj + 1], w1, w2));
    T[jj] = jj == 3 ? o : __builtin_rotateright32(o, 2 * jj + 2);   // jj = 3: a whole byte, taken care of by the byte index
  }
}

// two-weight schemes: eight lookups from entry words JA, JA + 1 (S: byte shift of word 3, see lane_entries3)
// k = 3 (S = 1): a[] = eight address registers holding lane * 4, mask = 0x3f
template <int JA, int S>
__device__ __forceinline__ void lane_issue_pairs(const uint32_t (&T)[4], uint32_t lanecol, const char* lds, uint32_t (&v)[8],
                                                 uint32_t (&a)[8], uint32_t mask) {
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const uint32_t t = T[JA + h];
    if constexpr (S == 1) {
      if (JA + h == 3) {
        lane_entry_addr_masked<1>(t, mask, a[4 * h + 0]);
        lane_entry_addr_masked<2>(t, mask, a[4 * h + 1]);
        lane_entry_addr_masked<3>(t, mask, a[4 * h + 2]);
        lane_entry_addr_masked<0>(t, mask, a[4 * h + 3]);
      } else {
        lane_entry_addr_masked<0>(t, mask, a[4 * h + 0]);
        lane_entry_addr_masked<1>(t, mask, a[4 * h + 1]);
        lane_entry_addr_masked<2>(t, mask, a[4 * h + 2]);
        lane_entry_addr_masked<3>(t, mask, a[4 * h + 3]);
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) v[4 * h + i] = lds_u32(lds, a[4 * h + i]);
    } else {
      v[4 * h + 0] = lds_u32(lds, lane_entry_addr<0>(t, lanecol));
      v[4 * h + 1] = lds_u32(lds, lane_entry_addr<1>(t, lanecol));
      v[4 * h + 2] = lds_u32(lds, lane_entry_addr<2>(t, lanecol));
      v[4 * h + 3] = lds_u32(lds, lane_entry_addr<3>(t, lanecol));
    }
  }
}

// One sample: the eight lookups of entry words JA, JA + 1 are the pairs 4 JA .. 4 JA + 7 of the word, which the
// lanes JA, JA + 1 of the quad hold in x.  Last lookup first: LDS answers in issue order, so one counter wait
// covers the eight.
template <int JA>
__device__ __forceinline__ void lane_consume_pairs(const uint32_t (&v)[8], const u32x4& x, float (&acc)[4]) {
  dot2_quad<JA + 1>(acc[3], x.w, v[7]);
  dot2_quad<JA + 1>(acc[2], x.z, v[6]);
  dot2_quad<JA + 1>(acc[1], x.y, v[5]);
  dot2_quad<JA + 1>(acc[0], x.x, v[4]);
  dot2_quad<JA>(acc[3], x.w, v[3]);
  dot2_quad<JA>(acc[2], x.z, v[2]);
  dot2_quad<JA>(acc[1], x.y, v[1]);
  dot2_quad<JA>(acc[0], x.x, v[0]);
}

// Four samples: the eight lookups of entry words JA, JA + 1 of word j (JO = j mod 2) are the chunks 8 JO + 2 JA .. + 3 of the
// tile's half j / 2, whose activations x holds.
template <int JA, int JO>
__device__ __forceinline__ void lane_consume_pairs(const uint32_t (&v)[8], uint64_t x, f32x4 (&acc)[2]) {
  mfma_chunk<8 * JO + 2 * JA + 3>(acc[1], x, v[6], v[7]);
  mfma_chunk<8 * JO + 2 * JA + 2>(acc[0], x, v[4], v[5]);
  mfma_chunk<8 * JO + 2 * JA + 1>(acc[1], x, v[2], v[3]);
  mfma_chunk<8 * JO + 2 * JA + 0>(acc[0], x, v[0], v[1]);
}

// single-weight schemes: the eight lookups of columns 8 JJ .. 8 JJ + 7
template <int K, int JJ>
__device__ __forceinline__ void lane_issue_singles(const uint32_t (&R)[8], uint32_t lanecol, const char* lds, uint32_t (&v)[8]) {
  using D = LaneDecode<K>;
#define DPLLM_LANE_LOOKUP(N)                                                                        \
  {                                                                                                 \
    constexpr int ce = 8 * JJ + 2 * N, co = ce + 1;                                                 \
    v[2 * N] = lds_u32(lds, lane_entry_addr<D::byte(ce)>(R[D::word(ce)], lanecol));                 \
    v[2 * N + 1] = lds_u32(lds, lane_entry_addr<D::byte(co)>(R[D::word(co)], lanecol));             \
  }
  DPLLM_LANE_LOOKUP(0) DPLLM_LANE_LOOKUP(1) DPLLM_LANE_LOOKUP(2) DPLLM_LANE_LOOKUP(3)
#undef DPLLM_LANE_LOOKUP
}

// a table entry is an fp16 in the low half of a dword: two of them pack into one fp16 pair.  One sample: columns
// 8 JJ .. + 7 of the word are the pairs lane JJ of the quad holds
template <int JJ>
__device__ __forceinline__ void lane_consume_singles(const uint32_t (&v)[8], const u32x4& x, float (&acc)[4]) {
  dot2_quad<JJ>(acc[3], x.w, v[6] | (v[7] << 16));
  dot2_quad<JJ>(acc[2], x.z, v[4] | (v[5] << 16));
  dot2_quad<JJ>(acc[1], x.y, v[2] | (v[3] << 16));
  dot2_quad<JJ>(acc[0], x.x, v[0] | (v[1] << 16));
}

// four samples: columns 8 JJ .. + 7 of word j (JO = j mod 2) are the chunks 8 JO + 2 JJ, + 1
template <int JJ, int JO>
__device__ __forceinline__ void lane_consume_singles(const uint32_t (&v)[8], uint64_t x, f32x4 (&acc)[2]) {
  mfma_chunk<8 * JO + 2 * JJ + 1>(acc[1], x, v[4] | (v[5] << 16), v[6] | (v[7] << 16));
  mfma_chunk<8 * JO + 2 * JJ + 0>(acc[0], x, v[0] | (v[1] << 16), v[2] | (v[3] << 16));
}

// k = 5, 6: the merge tree with its masks in vector registers (full-rate instructions); k = 7, 8 have no registers
// to spare for fifteen masks at two workgroups per compute unit and keep them in the instructions
template <int K>
__device__ __forceinline__ void lane_merge_fields(const uint32_t (&w)[K], uint32_t (&R)[8], const MergeMasks<K>& M) {
  if constexpr (K <= 6) merge_byte_fields_v<K, LaneDecode<K>::d>(w, R, M);
  else merge_byte_fields<K, LaneDecode<K>::d>(w, R);
}

// ---- one tile -------------------------------------------------------------------------------------------------
// Lookups run in chunks of eight; the next chunk's lookups are issued before the current chunk's multiply-adds.
// xmine: where this lane finds its part of the tile's parked activations.  One sample: the 16 bytes of its quad
// lane in word 0 (slot + 16 * (lane mod 4)), those of word j 64 j bytes on.  Four samples: its chunk of the tile's
// first half (its sample's slot + 8 * (lane / 4)), that of the second half 128 bytes on.
template <int K, int NB>
struct LaneX;
template <int K>
struct LaneX<K, 1> {
  u32x4 q[4];   // q[j][m] = pair 4 (lane mod 4) + m of word j
  __device__ __forceinline__ void load(const char* xmine) {
#pragma unroll
    for (int j = 0; j < 4; ++j) q[j] = *reinterpret_cast<const u32x4*>(xmine + j * 64);
  }
};
template <int K>
struct LaneX<K, 4> {
  uint64_t a[2];   // a[h] = chunk 16 h + lane / 4 of the tile, of sample lane mod 4
  __device__ __forceinline__ void load(const char* xmine) {
    a[0] = *reinterpret_cast<const uint64_t*>(xmine);
    a[1] = *reinterpret_cast<const uint64_t*>(xmine + 128);
  }
};

template <int JA, int J, int K>
__device__ __forceinline__ void lane_mac_pairs(const uint32_t (&v)[8], const LaneX<K, 1>& x, LaneAcc<1>& acc) {
  lane_consume_pairs<JA>(v, x.q[J], acc.v);
}
template <int JA, int J, int K>
__device__ __forceinline__ void lane_mac_pairs(const uint32_t (&v)[8], const LaneX<K, 4>& x, LaneAcc<4>& acc) {
  lane_consume_pairs<JA, J & 1>(v, x.a[J >> 1], acc.v);
}
template <int JJ, int J, int K>
__device__ __forceinline__ void lane_mac_singles(const uint32_t (&v)[8], const LaneX<K, 1>& x, LaneAcc<1>& acc) {
  lane_consume_singles<JJ>(v, x.q[J], acc.v);
}
template <int JJ, int J, int K>
__device__ __forceinline__ void lane_mac_singles(const uint32_t (&v)[8], const LaneX<K, 4>& x, LaneAcc<4>& acc) {
  lane_consume_singles<JJ, J & 1>(v, x.a[J >> 1], acc.v);
}

template <int K, int NB>
__device__ __forceinline__ void lane_compute(const LaneTile<K, NB>& t, uint32_t lanecol, const char* lds, const char* xmine,
                                             LaneAcc<NB>& acc, uint32_t (&addr)[8], uint32_t mask, const MergeMasks<K>& M) {
  uint32_t va[8], vb[8];
  LaneX<K, NB> x;
  x.load(xmine);
  using J0 = std::integral_constant<int, 0>;
  using J1 = std::integral_constant<int, 1>;
  using J2 = std::integral_constant<int, 2>;
  using J3 = std::integral_constant<int, 3>;
  if constexpr (LaneDecode<K>::pair) {
    uint32_t T[4][4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if constexpr (K == 3) {
        lane_entries3(t.w[0][j], t.w[1][j], t.w[2][j], T[j], M);
      } else {
        const uint32_t w[4] = {t.w[0][j], t.w[1][j], t.w[2][j], t.w[3][j]};
        merge_nibble_pairs_v(w, T[j], M);
      }
    }
    lane_issue_pairs<0, K == 3>(T[0], lanecol, lds, va, addr, mask);
    auto word = [&](auto jc) {
      constexpr int j = decltype(jc)::value;
      lane_issue_pairs<2, K == 3>(T[j], lanecol, lds, vb, addr, mask);
      sched_fence();
      lane_mac_pairs<0, j>(va, x, acc);
      sched_fence();
      if constexpr (j + 1 < 4) lane_issue_pairs<0, K == 3>(T[j + 1], lanecol, lds, va, addr, mask);
      sched_fence();
      lane_mac_pairs<2, j>(vb, x, acc);
      sched_fence();
    };
    word(J0{}); word(J1{}); word(J2{}); word(J3{});
  } else {
    uint32_t R[2][8];
    {
      uint32_t w[K];
#pragma unroll
      for (int b = 0; b < K; ++b) w[b] = t.w[b][0];
      lane_merge_fields<K>(w, R[0], M);
    }
    lane_issue_singles<K, 0>(R[0], lanecol, lds, va);
    auto word = [&](auto jc) {
      constexpr int j = decltype(jc)::value;
      if constexpr (j + 1 < 4) {
        uint32_t w[K];
#pragma unroll
        for (int b = 0; b < K; ++b) w[b] = t.w[b][j + 1];
        lane_merge_fields<K>(w, R[(j + 1) & 1], M);
      }
      lane_issue_singles<K, 1>(R[j & 1], lanecol, lds, vb);
      sched_fence();
      lane_mac_singles<0, j>(va, x, acc);
      sched_fence();
      lane_issue_singles<K, 2>(R[j & 1], lanecol, lds, va);
      sched_fence();
      lane_mac_singles<1, j>(vb, x, acc);
      sched_fence();
      lane_issue_singles<K, 3>(R[j & 1], lanecol, lds, vb);
      sched_fence();
      lane_mac_singles<2, j>(va, x, acc);
      sched_fence();
      if constexpr (j + 1 < 4) lane_issue_singles<K, 0>(R[(j + 1) & 1], lanecol, lds, va);
      sched_fence();
      lane_mac_singles<3, j>(vb, x, acc);
      sched_fence();
    };
    word(J0{}); word(J1{}); word(J2{}); word(J3{});
  }
}

// ---- tables -------------------------------------------------------------------------------------------------
// The lane's row of the k-bit table (the part this wavefront builds entries from), fetched one row block ahead.
//   k = 3: the whole row (8 fp16); k = 4: the whole row (16 fp16); k >= 5: entries [share * wave, + share)
template <int K>
struct LaneLut {
  static constexpr int kDwords = K == 3 ? 4 : K == 4 ? 8 : LaneDecode<K>::share / 2;
  uint32_t v[kDwords];
};

template <int K>
__device__ __forceinline__ void lane_fetch_lut(LaneLut<K>& L, const DPLLM_GLOBAL uint16_t* lut_base, int rb, int lane, int wave) {
  const DPLLM_GLOBAL uint32_t* row = reinterpret_cast<const DPLLM_GLOBAL uint32_t*>(lut_base + (((size_t)rb * 64 + lane) << K));
  const DPLLM_GLOBAL uint32_t* src = K <= 4 ? row : row + wave * LaneLut<K>::kDwords;
  if constexpr (LaneLut<K>::kDwords >= 4) {
#pragma unroll
    for (int i = 0; i < LaneLut<K>::kDwords / 4; ++i) {
      const u32x4 q = reinterpret_cast<const DPLLM_GLOBAL u32x4*>(src)[i];
      L.v[4 * i] = q.x; L.v[4 * i + 1] = q.y; L.v[4 * i + 2] = q.z; L.v[4 * i + 3] = q.w;
    }
  } else {
#pragma unroll
    for (int i = 0; i < LaneLut<K>::kDwords; ++i) L.v[i] = src[i];
  }
}

// half h (0 = low) of dword d, for a wavefront-uniform h
__device__ __forceinline__ uint32_t half_of(uint32_t d, int h) { return h ? d >> 16 : d & 0xffffu; }

template <int K>
__device__ __forceinline__ void lane_build_table(const LaneLut<K>& L, int wave, uint32_t lanecol, char* lds) {
  if constexpr (K == 3) {
    // wavefront w writes the entries (a = w, b = 0..7): (LUT[a], LUT[b])
    const uint32_t lw = wave < 2 ? L.v[0] : wave < 4 ? L.v[1] : wave < 6 ? L.v[2] : L.v[3];
    const uint32_t la = half_of(lw, wave & 1);
#pragma unroll
    for (int b = 0; b < 8; ++b) {
      const uint32_t hb = (b & 1) ? (L.v[b >> 1] & 0xffff0000u) : (L.v[b >> 1] << 16);
      *reinterpret_cast<uint32_t*>(lds + (uint32_t)(wave * 8 + b) * 256 + lanecol) = la | hb;
    }
  } else if constexpr (K == 4) {
    // wavefront w writes the entries (a = 2 w + s, b = 0..15), s = 0, 1
    uint32_t lw = L.v[0];
#pragma unroll
    for (int i = 1; i < 8; ++i) lw = wave == i ? L.v[i] : lw;
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      const uint32_t la = s ? lw >> 16 : lw & 0xffffu;
#pragma unroll
      for (int b = 0; b < 16; ++b) {
        const uint32_t hb = (b & 1) ? (L.v[b >> 1] & 0xffff0000u) : (L.v[b >> 1] << 16);
        *reinterpret_cast<uint32_t*>(lds + (uint32_t)((wave * 2 + s) * 16 + b) * 256 + lanecol) = la | hb;
      }
    }
  } else {
    // wavefront w writes its share of the entries, an fp16 in the low half of a dword
    constexpr int share = LaneDecode<K>::share;
#pragma unroll
    for (int e = 0; e < share; ++e) {
      const uint32_t v = (e & 1) ? L.v[e >> 1] >> 16 : L.v[e >> 1] & 0xffffu;
      *reinterpret_cast<uint32_t*>(lds + (uint32_t)(wave * share + e) * 256 + lanecol) = v;
    }
  }
}

__device__ __forceinline__ void lane_group_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Tiles in registers per wavefront: one being decoded, one in flight.  A third measured equal or up to 1.3 %
// slower in launches that fill the chip (with sixteen wavefronts on a compute unit the memory system has enough
// requests either way), and three or four tiles in flight did not help launches of a few hundred workgroups
// either (one dependency level of a chained step: 9.2 -> 10.3 us for q, k, v of a 7B block): those are bound by
// the chain launch -> job record -> selector results -> tables and first tiles -> decode, not by the number of
// requests in flight.
constexpr int kLaneDepth = 2;

// One workgroup: row blocks block, block + step, ... of a job (step = nblocks / nsplit); it is number `split` of
// the nsplit workgroups that share these row blocks, and its wavefront w takes slice v = 8 split + w of the
// 8 nsplit slices of the column tiles, [v ncc / (8 nsplit), (v + 1) ncc / (8 nsplit)), in every row block.  Tile
// loads run kLaneDepth - 1 tiles ahead, also across row blocks; past the end of the run the ring is refilled with
// dummy loads (see lane_load_tile).
template <int K, int NB>
__device__ __forceinline__ void gemv_lane(const GemvJob& job, uint32_t lut_off, int block, int split, int tid, char* lds) {
  constexpr int table_bytes = kLaneTableBytes;
  constexpr int D = kLaneDepth;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  const uint32_t lanecol = (uint32_t)lane * 4;  // the lane's column of the interleaved tables
  float* red = reinterpret_cast<float*>(lds + table_bytes);
  char* ready = lds + table_bytes + NB * kLaneRedBytes + wave * lane_x_bytes<NB>();   // + 256 b: the parked tile of sample b
  char* repair = reinterpret_cast<char*>(red) + wave * 256;   // k = 4: room to re-pair a tile's activations (see lane_lds_bytes)
  const int nsplit = job.nsplit;
  const int slice = split * kLaneWaves + wave, nslices = nsplit * kLaneWaves;
  const int c0 = slice * job.ncc / nslices, c1 = (slice + 1) * job.ncc / nslices;
  const int nrb = job.nrq;                     // row blocks of the job
  const int step = job.nblocks / nsplit;
  const DPLLM_GLOBAL uint16_t* lut_base = as_global(reinterpret_cast<const uint16_t*>(job.arena + lut_off));
  const bool idle = c0 >= c1;                  // fewer tiles than wavefronts: this one only helps with the tables
  // the table rows of the next row block travel one block ahead, except at k >= 7, where their 8 - 16 registers
  // would cost the second workgroup per compute unit
  constexpr bool kLutAhead = K <= 6;
  LaneTile<K, NB> ring[D];
  LaneLut<K> L;
  // few tiles per row block: their activations are parked once, for every row block of the run.  Their loads
  // go out first and are parked after the first table rows and tiles have been asked for, so that the
  // workgroup starts with one memory round trip, not two (k = 4 has no registers to spare for that: there the
  // tiles are asked for after the activations have been parked)
  constexpr bool kEarlyX = K != 4;
  const bool keep = NB == 1 && c1 - c0 <= kLaneKeepTiles;
  char* kept = ready + 256;
  // this lane's view of a tile's parked activations (see lane_compute)
  const int xlane = NB == 1 ? (lane & 3) * 16 : (lane & 3) * 256 + (lane >> 2) * 8;
  uint32_t xkeep[kLaneKeepTiles];
  if (keep) {
    if constexpr (kEarlyX) {
#pragma unroll
      for (int i = 0; i < kLaneKeepTiles; ++i) xkeep[i] = lane_load_x(job, min(c0 + i, job.ncc - 1), lane);
    } else {
      for (int cc = c0; cc < c1; ++cc)
        lane_park_x<K>(lane_mask_x(job, cc, lane, lane_load_x(job, cc, lane)), lane, repair, kept + (cc - c0) * 256);
    }
  }
  if constexpr (kLutAhead) lane_fetch_lut<K>(L, lut_base, block, lane, wave);
  int lrb = block, lcc = c0;                   // load cursor
  bool more = true;                            // the load cursor is still inside the run
  auto load_next = [&](LaneTile<K, NB>& t) {
    lane_load_tile<K, NB>(t, job, lrb, lcc, lane, !keep, more);
    if (++lcc >= c1) {
      lcc = c0;
      if (lrb + step < nrb) lrb += step; else more = false;
    }
  };
  if (!idle) {
#pragma unroll
    for (int i = 0; i < D - 1; ++i) load_next(ring[i]);
  }
  if (kEarlyX && keep) {
#pragma unroll
    for (int i = 0; i < kLaneKeepTiles; ++i)
      if (c0 + i < c1) lane_park_x<K>(lane_mask_x(job, c0 + i, lane, xkeep[i]), lane, repair, kept + i * 256);
  }
  LaneAcc<NB> acc;
  acc.zero();
  MergeMasks<K> M;
  if constexpr (K <= 6) M.init();
  uint32_t addr[8], mask = 0x3fu;              // k = 3: address registers of the lookups (see lane_issue_pairs)
#pragma unroll
  for (int i = 0; i < 8; ++i) addr[i] = lanecol;
  int rb = block, cc = c0;                     // compute cursor
  auto open_block = [&]() {
    if constexpr (!kLutAhead) lane_fetch_lut<K>(L, lut_base, rb, lane, wave);
    lane_build_table<K>(L, wave, lanecol, lds);
    if constexpr (kLutAhead) lane_fetch_lut<K>(L, lut_base, rb + step < nrb ? rb + step : rb, lane, wave);
    lane_group_barrier();
  };
  auto close_block = [&]() {
#pragma unroll
    for (int b = 0; b < NB; ++b) red[(b * kLaneWaves + wave) * 64 + lane] = acc.sum(b);
    acc.zero();
    lane_group_barrier();
    const bool storer = wave < NB && (NB == 1 || wave < job.nsamples);   // wavefront b stores sample b
    float s = 0.f;
    if (storer) {
#pragma unroll
      for (int w = 0; w < kLaneWaves; ++w) s += red[(wave * kLaneWaves + w) * 64 + lane];
    }
    bool last = true;
    if (nsplit > 1) {
      // Column split: every workgroup of the row block leaves its sums in the pool, then takes a ticket; the
      // holder of the last ticket finds all of them, adds them in the order of the splits (so the result does
      // not depend on who arrives last) and leaves the counter at zero again.  Ordering: plain stores ->
      // workgroup barrier -> thread 0: release fence at agent scope, ticket (agent-scope read-modify-write),
      // acquire fence at agent scope when the ticket is the last -> workgroup barrier -> plain loads.  The
      // release fence writes the sums back to where every die sees them before the ticket is taken; the acquire
      // fence drops what this die may still cache of the pool before the sums are read.
      DPLLM_GLOBAL float* part = as_global(job.ws) + (size_t)(rb * NB + wave) * nsplit * 64 + lane;
      DPLLM_GLOBAL uint32_t* ticket = as_global(job.cnt) + rb * NB;
      uint32_t* flag = reinterpret_cast<uint32_t*>(red);   // free by now: the sums above were read before the next barrier
      if (storer) part[split * 64] = s;
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
      __builtin_amdgcn_s_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
      if (tid == 0) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
        const uint32_t old = __hip_atomic_fetch_add(ticket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const bool mine = old == (uint32_t)(nsplit - 1);
        if (mine) {
          __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
          __hip_atomic_store(ticket, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        *flag = mine;
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
      __builtin_amdgcn_s_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
      last = *flag != 0;
      if (storer && last) {
        s = 0.f;
        for (int i = 0; i < nsplit; ++i) s += part[i * 64];
      }
    }
    const int o = rb * 64 + lane;
    if (storer && last && o < job.out) as_global(job.y)[(size_t)wave * job.out + o] = __builtin_bit_cast(uint16_t, (_Float16)s);
  };
  open_block();
  if (idle) {
    for (;;) {
      close_block();
      rb += step;
      if (rb >= nrb) return;
      open_block();
    }
  }
  for (;;) {
#pragma unroll
    for (int s = 0; s < D; ++s) {
      load_next(ring[(s + D - 1) % D]);
      const char* xready = kept + (cc - c0) * 256;
      if (!keep) {
#pragma unroll
        for (int b = 0; b < NB; ++b) lane_park_x<K>(lane_mask_x(job, cc, lane, ring[s].x[b]), lane, repair, ready + b * 256);
        xready = ready;
      }
      lane_compute<K, NB>(ring[s], lanecol, lds, xready + xlane, acc, addr, mask, M);
      if (++cc >= c1) {
        close_block();
        rb += step;
        if (rb >= nrb) return;
        cc = c0;
        open_block();
      }
    }
  }
}

// The bitwidth of the job: its own value, the word a selector left in device memory, or the decision taken here
// from the partial results of an earlier selector launch (every workgroup of the job repeats the same fixed-order
// sums, so all arrive at the same bits; the job's first workgroup writes bitwidth and estimate out).  A value the
// linear does not serve (outside [max(kmin, 3), p]) is not served: the workgroup returns and y keeps what it held.
template <int NB>
__device__ __forceinline__ void gemv_lane_block(const GemvJob& job, int block, int tid, char* lds, const SelParams* params,
                                                const int32_t* target, int n_linears) {   // params == nullptr: no decisions here
  const int first = block == 0;
  const int split = block % job.nsplit;
  block /= job.nsplit;
  if (block >= job.nrq) return;
  int k = job.k;
  if (job.has_fin && params != nullptr) {
    k = selector_finish(job.fin, params + (size_t)(*target) * n_linears + job.fin.linear, tid, kLaneThreads,
                        reinterpret_cast<double*>(lds), first);   // the tables are not built yet
    k = __builtin_amdgcn_readfirstlane(k);
  } else if (job.k_dev != nullptr) {
    k = __builtin_amdgcn_readfirstlane(*as_global(job.k_dev));
  }
  if (k < max(job.kmin, kFastKMin) || k > min(job.p, kFastKMax)) return;
  switch (k) {   // (the table offsets are taken by constant index: a run-time index would put the job record in scratch memory)
    case 3: gemv_lane<3, NB>(job, job.lut_off[0], block, split, tid, lds); break;
    case 4: gemv_lane<4, NB>(job, job.lut_off[1], block, split, tid, lds); break;
    case 5: gemv_lane<5, NB>(job, job.lut_off[2], block, split, tid, lds); break;
    case 6: gemv_lane<6, NB>(job, job.lut_off[3], block, split, tid, lds); break;
    case 7: gemv_lane<7, NB>(job, job.lut_off[4], block, split, tid, lds); break;
    default: gemv_lane<8, NB>(job, job.lut_off[5], block, split, tid, lds); break;
  }
}

// jobs == nullptr: the job passed by value, for njobs right-hand sides in groups of NB that share one pass over
// the planes (group g reads x + g * NB * in and writes y + g * NB * out; workgroups [g * nblocks, (g + 1) *
// nblocks) serve it); else (NB = 1) block b belongs to job block_jobs[b] of the table.  params / target /
// n_linears: the table of selector parameters, for jobs that take their decision here.
template <int NB>
__global__ void __launch_bounds__(kLaneThreads) gemv_lane_kernel(const GemvJob* __restrict__ jobs, const int32_t* __restrict__ block_jobs,
                                                                 int njobs, GemvJob one, const SelParams* __restrict__ params,
                                                                 const int32_t* __restrict__ target, int n_linears) {
  __shared__ __attribute__((aligned(256))) char lds[lane_lds_bytes<NB>()];
  // the lookup addresses are formed as (entry << 8) | (lane << 2): the tables must start at LDS address 0
  if ((uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)lds != 0u) return;
  if (jobs == nullptr) {
    const int group = blockIdx.x / one.nblocks;
    one.x += (size_t)group * NB * one.ncw * 32;
    one.y += (size_t)group * NB * one.out;
    one.nsamples = min(NB, njobs - group * NB);
    one.ws += (size_t)group * one.nrq * NB * one.nsplit * 64;
    one.cnt += (size_t)group * one.nrq * NB;
    gemv_lane_block<NB>(one, blockIdx.x - group * one.nblocks, threadIdx.x, lds, params, target, n_linears);
    return;
  }
  if constexpr (NB == 1) {
    const int b = blockIdx.x;
    GemvJob job = jobs[block_jobs[b]];
    gemv_lane_block<1>(job, b - job.block_start, threadIdx.x, lds, params, target, n_linears);
  }
}

}  // namespace dpllm
