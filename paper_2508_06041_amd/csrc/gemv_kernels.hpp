// Plain any-precision GEMV kernel: y = W_k x with W_k[o][c] = LUT_k[o][code_p(o,c) >> (p - k)], reading
// the top k bitplanes only (paper Sec. 3: the linear operation of a decode step is a GEMV;
// Sec. 2.2: the k-bit model is overlaid in the parent's memory).  One wavefront per four rows, one code bit
// at a time: it serves every bitwidth from 1 to 8 and every batch, and is what runs for the bitwidths below 3,
// which the streaming kernel (gemv_lane.hpp) has no decode scheme for.
#pragma once
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include <cstdint>

#include "layout_device.hpp"

namespace dpllm {

struct GemvArgs {
  const char* arena;         // device planes start here, plane b at + b * plane_bytes
  size_t plane_bytes;
  uint32_t lut_off[9];       // byte offset of the k-bit table inside the arena ([rows padded][2^k] fp16), k = kmin..p
  int k;                     // the bitwidth when k_dev == nullptr
  const int32_t* k_dev;      // else the bitwidth is *k_dev; a value outside [kmin, p] is not served
  int kmin, p;
  const uint16_t* x;         // fp16 [B][in]
  uint16_t* y;               // fp16 [B][out]
  int out, in, ncw, ncc;
};

template <int B>
__global__ void __launch_bounds__(256) gemv_plain_kernel(GemvArgs a) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int rq = blockIdx.x * 4 + wave;
  if (rq * 4 >= a.out) return;
  int k = a.k;
  if (a.k_dev != nullptr) k = *a.k_dev;
  if (k < a.kmin || k > a.p) return;
  const uint16_t* lut = reinterpret_cast<const uint16_t*>(a.arena + a.lut_off[k]);
  float acc[4][B];
#pragma unroll
  for (int r = 0; r < 4; ++r)
#pragma unroll
    for (int b = 0; b < B; ++b) acc[r][b] = 0.f;
  for (int cw = lane; cw < a.ncw; cw += 64) {
    uint4 w[8];
    for (int b = 0; b < k; ++b) {
      const uint32_t* pl = reinterpret_cast<const uint32_t*>(a.arena + (size_t)b * a.plane_bytes);
      // rows past `out` inside the last block of 64 are zero words of the padded layout
      w[b].x = pl[plane_word_index(rq * 4 + 0, cw, a.ncc)];
      w[b].y = pl[plane_word_index(rq * 4 + 1, cw, a.ncc)];
      w[b].z = pl[plane_word_index(rq * 4 + 2, cw, a.ncc)];
      w[b].w = pl[plane_word_index(rq * 4 + 3, cw, a.ncc)];
    }
    for (int q = 0; q < 32; ++q) {
      uint32_t code[4] = {0, 0, 0, 0};
      for (int b = 0; b < k; ++b) {
        int pos = (col_to_pos(q) - b) & 31;  // plane b keeps column q at bit pos(q) - b
        code[0] = (code[0] << 1) | ((w[b].x >> pos) & 1u);
        code[1] = (code[1] << 1) | ((w[b].y >> pos) & 1u);
        code[2] = (code[2] << 1) | ((w[b].z >> pos) & 1u);
        code[3] = (code[3] << 1) | ((w[b].w >> pos) & 1u);
      }
      float xv[B];
#pragma unroll
      for (int b = 0; b < B; ++b)
        xv[b] = __half2float(__ushort_as_half(a.x[(size_t)b * a.in + cw * 32 + q]));
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        float wv = __half2float(__ushort_as_half(lut[((size_t)(rq * 4 + r) << k) + code[r]]));
#pragma unroll
        for (int b = 0; b < B; ++b) acc[r][b] = fmaf(wv, xv[b], acc[r][b]);
      }
    }
  }
#pragma unroll
  for (int r = 0; r < 4; ++r)
#pragma unroll
    for (int b = 0; b < B; ++b) {
      float s = acc[r][b];
#pragma unroll
      for (int sh = 32; sh >= 1; sh >>= 1) s += __shfl_xor(s, sh, 64);
      int o = rq * 4 + r;
      if (lane == 0 && o < a.out) a.y[(size_t)b * a.out + o] = __half_as_ushort(__float2half_rn(s));
    }
}

}  // namespace dpllm
