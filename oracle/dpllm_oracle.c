/*
 * CPU oracle for the DP-LLM decode hot path.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, plain definition the GPU library is checked against.
 * It is built into its own shared object, shares no source, header, table or
 * helper with the HIP library, and may be called only from tests/, from the
 * smoke check and from the bench's cpu_baseline leg.  The product path never
 * links or loads it.
 *
 * Everything accumulates in IEEE double, left to right in the index order the
 * definitions state; fp16 inputs are taken at their exact values.
 *
 * What each function follows:
 *   orc_half_to_double  IEEE 754 binary16 (the activation / centroid format of
 *                       the weight-only-quantized model, paper Sec. 6: "fp16").
 *   orc_unpack          the multi-scale ("overlaid") weight store of Sec. 2.2:
 *                       one parent p-bit code per weight, stored as p bitplanes,
 *                       most significant plane first.
 *   orc_index_k         the k-bit child model is the k-bit prefix of the parent
 *                       code (Sec. 2.2, overlay of 3..n-bit variants).
 *   orc_dequant         W_{i,k} of Algorithm 1: per-row centroid table lookup.
 *   orc_gemv            the linear operation y = W_{i,k} x of Sec. 3 (a GEMV at
 *                       decode batch 1; B right-hand sides = B such GEMVs).
 *   orc_exact_err       the relative error ||dW x||, dW = W_h - W_l (Sec. 3,
 *                       Algorithm 1 Phase 3).
 *   orc_estimate        the random-projection estimate ||G x||, G = A dW
 *                       precomputed offline (Sec. 5.1, the inequality pair).
 *   orc_linreg_estimate the linear-regression estimate alpha*||x|| + beta
 *                       (Sec. 5.1).
 *   orc_decide          the precision selector rule of Sec. 3: relative error
 *                       exceeding T picks h, otherwise l.  T = +inf / -inf pins
 *                       the layer to l / h (App. B latency protocol).
 *   orc_effective_bits  parameter-weighted mean bitwidth, the first term inside
 *                       the regulariser of Eq. (1).
 *
 * Canonical host layout (fixed by the library boundary, not by the paper):
 *   planes : uint32 [p][out][in/32]; plane 0 holds the most significant bit of
 *            the p-bit code; column c is bit (c % 32) of word c / 32.
 *   lut_k  : uint16 (binary16 bit patterns) [out][2^k].
 *   x, G   : uint16 (binary16 bit patterns), row-major.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* exact value of a binary16 bit pattern */
double orc_half_to_double(uint16_t h) {
  int sign = (h >> 15) & 1;
  int expo = (h >> 10) & 0x1f;
  int frac = h & 0x3ff;
  double v;
  if (expo == 0) {
    v = ldexp((double)frac, -24); /* subnormal or zero: frac * 2^-24 */
  } else if (expo == 31) {
    v = frac ? NAN : INFINITY;
  } else {
    v = ldexp((double)(frac + 1024), expo - 25); /* (1 + frac/1024) * 2^(expo-15) */
  }
  return sign ? -v : v;
}

int orc_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* parent p-bit code of weight (o, c) */
static inline unsigned code_p(const uint32_t* planes, int p, int out, int in, int o, int c) {
  size_t words_per_row = (size_t)in / 32;
  size_t plane_words = (size_t)out * words_per_row;
  unsigned code = 0;
  for (int b = 0; b < p; ++b) {
    uint32_t word = planes[(size_t)b * plane_words + (size_t)o * words_per_row + (size_t)(c / 32)];
    unsigned bit = (word >> (c % 32)) & 1u;
    code |= bit << (p - 1 - b);
  }
  return code;
}

/* O1: bitplanes -> parent codes, uint8 [out][in] */
void orc_unpack(const uint32_t* planes, int p, int out, int in, uint8_t* idx_p) {
#pragma omp parallel for schedule(static)
  for (int o = 0; o < out; ++o)
    for (int c = 0; c < in; ++c)
      idx_p[(size_t)o * in + c] = (uint8_t)code_p(planes, p, out, in, o, c);
}

/* O2: k-bit code = top k bits of the p-bit code */
void orc_index_k(const uint8_t* idx_p, size_t n, int p, int k, uint8_t* idx_k) {
  for (size_t i = 0; i < n; ++i) idx_k[i] = (uint8_t)(idx_p[i] >> (p - k));
}

/* O3: dense dequantised matrix, double [out][in] */
void orc_dequant(const uint8_t* idx_k, const uint16_t* lut_k, int k, int out, int in, double* W) {
  size_t entries = (size_t)1 << k;
  for (int o = 0; o < out; ++o)
    for (int c = 0; c < in; ++c)
      W[(size_t)o * in + c] = orc_half_to_double(lut_k[(size_t)o * entries + idx_k[(size_t)o * in + c]]);
}

/* O4: y[b][o] = sum_c W_k[o][c] * x[b][c], double [B][out] */
void orc_gemv(const uint32_t* planes, int p, int k, const uint16_t* lut_k, int out, int in,
              const uint16_t* x, int B, double* y) {
  size_t entries = (size_t)1 << k;
  double* xd = (double*)malloc(sizeof(double) * (size_t)B * in);
  for (size_t i = 0; i < (size_t)B * in; ++i) xd[i] = orc_half_to_double(x[i]);
#pragma omp parallel for schedule(static)
  for (int o = 0; o < out; ++o) {
    for (int b = 0; b < B; ++b) {
      double acc = 0.0;
      for (int c = 0; c < in; ++c) {
        unsigned code = code_p(planes, p, out, in, o, c) >> (p - k);
        double w = orc_half_to_double(lut_k[(size_t)o * entries + code]);
        acc += w * xd[(size_t)b * in + c];
      }
      y[(size_t)b * out + o] = acc;
    }
  }
  free(xd);
}

/* O5: e* = || (W_h - W_l) x ||_2 ; also returns ||W_h x||_2 through norm_h when not NULL */
double orc_exact_err(const uint32_t* planes, int p, int l, int h, const uint16_t* lut_l,
                     const uint16_t* lut_h, int out, int in, const uint16_t* x, double* norm_h) {
  size_t el = (size_t)1 << l, eh = (size_t)1 << h;
  double* xd = (double*)malloc(sizeof(double) * (size_t)in);
  double* d = (double*)malloc(sizeof(double) * (size_t)out);
  double* yh = (double*)malloc(sizeof(double) * (size_t)out);
  for (int c = 0; c < in; ++c) xd[c] = orc_half_to_double(x[c]);
#pragma omp parallel for schedule(static)
  for (int o = 0; o < out; ++o) {
    double acc_d = 0.0, acc_h = 0.0;
    for (int c = 0; c < in; ++c) {
      unsigned code = code_p(planes, p, out, in, o, c);
      double wl = orc_half_to_double(lut_l[(size_t)o * el + (code >> (p - l))]);
      double wh = orc_half_to_double(lut_h[(size_t)o * eh + (code >> (p - h))]);
      acc_d += (wh - wl) * xd[c];
      acc_h += wh * xd[c];
    }
    d[o] = acc_d;
    yh[o] = acc_h;
  }
  double s = 0.0, sh = 0.0;
  for (int o = 0; o < out; ++o) {
    s += d[o] * d[o];
    sh += yh[o] * yh[o];
  }
  if (norm_h) *norm_h = sqrt(sh);
  free(xd);
  free(d);
  free(yh);
  return sqrt(s);
}

/* O6: e^ = || G x ||_2, G binary16 [r][in]; g (double [r]) is written when not NULL */
double orc_estimate(const uint16_t* G, int r, int in, const uint16_t* x, double* g) {
  double s = 0.0;
  for (int j = 0; j < r; ++j) {
    double acc = 0.0;
    for (int c = 0; c < in; ++c)
      acc += orc_half_to_double(G[(size_t)j * in + c]) * orc_half_to_double(x[c]);
    if (g) g[j] = acc;
    s += acc * acc;
  }
  return sqrt(s);
}

/* e^ = alpha * ||x||_2 + beta */
double orc_linreg_estimate(const uint16_t* x, int in, double alpha, double beta) {
  double s = 0.0;
  for (int c = 0; c < in; ++c) {
    double v = orc_half_to_double(x[c]);
    s += v * v;
  }
  return alpha * sqrt(s) + beta;
}

/* O7: strictly exceeding T selects h; equality and anything below selects l */
int orc_decide(double e, float T, int l, int h) { return (e > (double)T) ? h : l; }

/* parameter-weighted mean bitwidth */
double orc_effective_bits(const int32_t* k, const int64_t* params, int n) {
  double num = 0.0, den = 0.0;
  for (int i = 0; i < n; ++i) {
    num += (double)k[i] * (double)params[i];
    den += (double)params[i];
  }
  return num / den;
}
