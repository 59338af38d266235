// Host side of the C boundary declared in include/dpllm.h: argument checks, the model object,
// load-time re-tiling and kernel launches.  No kernel arithmetic lives here.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "../../include/dpllm.h"
#include "aux_kernels.hpp"
#include "gemv_fast.hpp"
#include "gemv_kernels.hpp"
#include "layout.hpp"

using namespace dpllm;

namespace {

struct Selector {
  bool set = false;
  int l = 0, h = 0, kind = DPLLM_SEL_NONE, r = 0;
  const uint16_t* G = nullptr;
  float alpha = 0.f, beta = 0.f, T = 0.f;
};

struct Linear {
  bool loaded = false;
  LinearLayout L;
  char* arena = nullptr;
  Selector sel[DPLLM_MAX_PAIRS];
  int active = -1;
  const uint4* planes() const { return reinterpret_cast<const uint4*>(arena); }
  const uint16_t* lut(int k) const { return reinterpret_cast<const uint16_t*>(arena + L.lut_offset[k]); }
  int find_pair(int l, int h) const {
    for (int i = 0; i < DPLLM_MAX_PAIRS; ++i)
      if (sel[i].set && sel[i].l == l && sel[i].h == h) return i;
    return -1;
  }
};

}  // namespace

struct dpllm_model {
  std::vector<Linear> linears;
  std::string err;
  double* sel_partial = nullptr;   // [DPLLM_MAX_RANK][max splits]
  unsigned* sel_counter = nullptr;
  int device = 0;
};

namespace {

constexpr int kMaxSelSplits = 64;  // up to 65536 input columns

int fail(dpllm_model* m, int code, const char* fmt, ...) {
  if (m) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    m->err = buf;
  }
  return code;
}

int hip_fail(dpllm_model* m, hipError_t e, const char* what) {
  return fail(m, DPLLM_EHIP, "%s: %s", what, hipGetErrorString(e));
}

#define HIP_TRY(m, call)                                 \
  do {                                                   \
    hipError_t e__ = (call);                             \
    if (e__ != hipSuccess) return hip_fail(m, e__, #call); \
  } while (0)

int check_shape(int out, int in, int p, int kmin) {
  if (out < 1 || in < 32 || in % 32 != 0) return DPLLM_ESHAPE;
  if (p < 1 || p > DPLLM_MAX_BITS || kmin < 1 || kmin > p) return DPLLM_ERANGE;
  return DPLLM_OK;
}

Linear* get_linear(dpllm_model* m, int id, int* rc) {
  if (!m) { *rc = DPLLM_EINVAL; return nullptr; }
  if (id < 0 || id >= (int)m->linears.size()) { *rc = fail(m, DPLLM_EINVAL, "linear id %d out of range", id); return nullptr; }
  Linear* lin = &m->linears[id];
  if (!lin->loaded) { *rc = fail(m, DPLLM_ESTATE, "linear %d is not loaded", id); return nullptr; }
  return lin;
}

int launch_selector(dpllm_model* m, const Linear& lin, const Selector& s, const void* x, float* e_dev,
                    int32_t* k_dev, hipStream_t st) {
  if (s.kind == DPLLM_SEL_PROJ) {
    int nsplit = (lin.L.in + kSelSplitCols - 1) / kSelSplitCols;
    if (nsplit > kMaxSelSplits) return fail(m, DPLLM_ESHAPE, "in = %d too wide for the selector workspace", lin.L.in);
    dim3 grid(nsplit, s.r);
    hipLaunchKernelGGL(selector_proj_kernel, grid, dim3(kSelThreads), 0, st, s.G, (const uint16_t*)x, lin.L.in,
                       s.r, nsplit, m->sel_partial, m->sel_counter, s.T, s.l, s.h, e_dev, k_dev);
  } else if (s.kind == DPLLM_SEL_LINREG) {
    hipLaunchKernelGGL(selector_linreg_kernel, dim3(1), dim3(256), 0, st, (const uint16_t*)x, lin.L.in, s.alpha,
                       s.beta, s.T, s.l, s.h, e_dev, k_dev);
  } else {
    hipLaunchKernelGGL(selector_fixed_kernel, dim3(1), dim3(1), 0, st, s.l, e_dev, k_dev);
  }
  HIP_TRY(m, hipGetLastError());
  return DPLLM_OK;
}

template <int B>
void launch_plain(const GemvArgs& a, hipStream_t st) {
  dim3 grid((a.nrq + 3) / 4);
  hipLaunchKernelGGL(gemv_plain_kernel<B>, grid, dim3(256), 0, st, a);
}

int launch_gemv(dpllm_model* m, const Linear& lin, int ka, int kb, const int32_t* k_dev, const void* x, void* y,
                int B, hipStream_t st) {
  GemvArgs a;
  a.planes = lin.planes();
  a.plane_stride_u4 = lin.L.plane_bytes / 16;
  a.ka = ka;
  a.kb = kb;
  a.lut_a = lin.lut(ka);
  a.lut_b = k_dev ? lin.lut(kb) : nullptr;
  a.k_dev = k_dev;
  a.x = (const uint16_t*)x;
  a.y = (uint16_t*)y;
  a.out = lin.L.out;
  a.in = lin.L.in;
  a.ncw = lin.L.ncw;
  a.nrq = lin.L.nrq;
  switch (B) {
    case 1: {
      GemvJob j;
      j.arena = lin.arena;
      j.x = (const uint16_t*)x;
      j.y = (uint16_t*)y;
      j.k_dev = k_dev;
      j.plane_stride_u4 = (uint32_t)(lin.L.plane_bytes / 16);
      j.lut_off_a = (uint32_t)lin.L.lut_offset[ka];
      j.lut_off_b = (uint32_t)lin.L.lut_offset[kb];
      j.ka = ka; j.kb = kb;
      j.out = lin.L.out; j.ncw = lin.L.ncw; j.nrq = lin.L.nrq;
      j.block_start = 0;
      hipLaunchKernelGGL(gemv_one_kernel, dim3(lin.L.nrq), dim3(64), 0, st, j);
      break;
    }
    case 2: launch_plain<2>(a, st); break;
    case 3: launch_plain<3>(a, st); break;
    case 4: launch_plain<4>(a, st); break;
    case 5: launch_plain<5>(a, st); break;
    case 6: launch_plain<6>(a, st); break;
    case 7: launch_plain<7>(a, st); break;
    case 8: launch_plain<8>(a, st); break;
    default: return fail(m, DPLLM_ESHAPE, "batch %d outside [1, %d]", B, DPLLM_MAX_BATCH);
  }
  HIP_TRY(m, hipGetLastError());
  return DPLLM_OK;
}

}  // namespace

extern "C" {

int dpllm_model_create(dpllm_model** out, int n_linears) {
  if (!out || n_linears < 1) return DPLLM_EINVAL;
  *out = nullptr;
  dpllm_model* m = new (std::nothrow) dpllm_model();
  if (!m) return DPLLM_EINVAL;
  m->linears.resize(n_linears);
  if (hipGetDevice(&m->device) != hipSuccess ||
      hipMalloc((void**)&m->sel_partial, sizeof(double) * DPLLM_MAX_RANK * kMaxSelSplits) != hipSuccess ||
      hipMalloc((void**)&m->sel_counter, 256) != hipSuccess ||
      hipMemset(m->sel_counter, 0, 256) != hipSuccess) {
    (void)hipGetLastError();
    if (m->sel_partial) (void)hipFree(m->sel_partial);
    if (m->sel_counter) (void)hipFree(m->sel_counter);
    delete m;
    return DPLLM_EHIP;
  }
  *out = m;
  return DPLLM_OK;
}

void dpllm_model_destroy(dpllm_model* m) {
  if (!m) return;
  if (m->sel_partial) (void)hipFree(m->sel_partial);
  if (m->sel_counter) (void)hipFree(m->sel_counter);
  delete m;
}

const char* dpllm_last_error(const dpllm_model* m) { return m ? m->err.c_str() : "null model"; }

int dpllm_linear_device_bytes(int out, int in, int p, int kmin, size_t* bytes) {
  if (!bytes) return DPLLM_EINVAL;
  int rc = check_shape(out, in, p, kmin);
  if (rc != DPLLM_OK) return rc;
  *bytes = LinearLayout::make(out, in, p, kmin).total_bytes;
  return DPLLM_OK;
}

int dpllm_load_linear(dpllm_model* m, int id, int out, int in, int p, int kmin, const uint32_t* planes,
                      const uint16_t* const* luts, int src_on_device, void* dev_arena, size_t arena_bytes,
                      void* stream) {
  if (!m) return DPLLM_EINVAL;
  if (id < 0 || id >= (int)m->linears.size()) return fail(m, DPLLM_EINVAL, "linear id %d out of range", id);
  if (!planes || !luts || !dev_arena) return fail(m, DPLLM_EINVAL, "null pointer");
  if (src_on_device != 0 && src_on_device != 1) return fail(m, DPLLM_EINVAL, "src_on_device must be 0 or 1");
  int rc = check_shape(out, in, p, kmin);
  if (rc != DPLLM_OK) return fail(m, rc, "bad shape out=%d in=%d p=%d kmin=%d", out, in, p, kmin);
  for (int k = kmin; k <= p; ++k)
    if (!luts[k - kmin]) return fail(m, DPLLM_EINVAL, "null table for k=%d", k);
  if ((uintptr_t)dev_arena % kAlign) return fail(m, DPLLM_EINVAL, "arena not %zu-byte aligned", kAlign);
  LinearLayout L = LinearLayout::make(out, in, p, kmin);
  if (arena_bytes < L.total_bytes)
    return fail(m, DPLLM_ESTATE, "arena holds %zu bytes, %zu needed", arena_bytes, L.total_bytes);
  hipStream_t st = (hipStream_t)stream;

  const size_t plane_words = (size_t)p * out * L.ncw;
  size_t lut_elems_total = 0;
  for (int k = kmin; k <= p; ++k) lut_elems_total += (size_t)out << k;
  const uint32_t* d_planes = planes;
  void* staging = nullptr;
  if (!src_on_device) {
    HIP_TRY(m, hipMalloc(&staging, plane_words * 4 + lut_elems_total * 2));
    hipError_t e = hipMemcpyAsync(staging, planes, plane_words * 4, hipMemcpyHostToDevice, st);
    char* dst = (char*)staging + plane_words * 4;
    for (int k = kmin; k <= p && e == hipSuccess; ++k) {
      size_t bytes = ((size_t)out << k) * 2;
      e = hipMemcpyAsync(dst, luts[k - kmin], bytes, hipMemcpyHostToDevice, st);
      dst += bytes;
    }
    if (e != hipSuccess) { (void)hipFree(staging); return hip_fail(m, e, "hipMemcpyAsync"); }
    d_planes = (const uint32_t*)staging;
  }
  {
    size_t n = (size_t)L.nrq * L.ncw * p;
    hipLaunchKernelGGL(retile_planes_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, d_planes,
                       (uint4*)dev_arena, p, out, L.ncw, L.nrq, L.plane_bytes / 16);
  }
  const char* lsrc = staging ? (const char*)staging + plane_words * 4 : nullptr;
  for (int k = kmin; k <= p; ++k) {
    const uint16_t* src = staging ? (const uint16_t*)lsrc : luts[k - kmin];
    size_t n = (size_t)L.nrq * 4 << k;
    hipLaunchKernelGGL(copy_lut_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, src,
                       (uint16_t*)((char*)dev_arena + L.lut_offset[k]), out, L.nrq * 4, 1 << k);
    if (staging) lsrc += ((size_t)out << k) * 2;
  }
  hipError_t e = hipGetLastError();
  if (e == hipSuccess) e = hipStreamSynchronize(st);
  if (staging) (void)hipFree(staging);
  if (e != hipSuccess) return hip_fail(m, e, "load kernels");
  Linear& lin = m->linears[id];
  lin = Linear();
  lin.loaded = true;
  lin.L = L;
  lin.arena = (char*)dev_arena;
  return DPLLM_OK;
}

int dpllm_set_selector(dpllm_model* m, int id, int l, int h, int kind, const void* G_dev, int r, float alpha,
                       float beta, float T) {
  int rc = DPLLM_OK;
  Linear* lin = get_linear(m, id, &rc);
  if (!lin) return rc;
  if (l < lin->L.kmin || h > lin->L.p || l > h) return fail(m, DPLLM_ERANGE, "pair (%d,%d) outside [%d,%d]", l, h, lin->L.kmin, lin->L.p);
  if (std::isnan(T)) return fail(m, DPLLM_EINVAL, "threshold is NaN");
  if (kind == DPLLM_SEL_PROJ) {
    if (!G_dev) return fail(m, DPLLM_EINVAL, "G is null");
    if (r < 1 || r > DPLLM_MAX_RANK) return fail(m, DPLLM_ERANGE, "rank %d outside [1,%d]", r, DPLLM_MAX_RANK);
    if ((uintptr_t)G_dev % 16) return fail(m, DPLLM_EINVAL, "G not 16-byte aligned");
  } else if (kind == DPLLM_SEL_LINREG) {
    if (std::isnan(alpha) || std::isnan(beta)) return fail(m, DPLLM_EINVAL, "alpha/beta NaN");
  } else if (kind == DPLLM_SEL_NONE) {
    if (l != h) return fail(m, DPLLM_EINVAL, "kind none needs l == h");
  } else {
    return fail(m, DPLLM_EINVAL, "unknown selector kind %d", kind);
  }
  int slot = lin->find_pair(l, h);
  if (slot < 0)
    for (int i = 0; i < DPLLM_MAX_PAIRS && slot < 0; ++i)
      if (!lin->sel[i].set) slot = i;
  if (slot < 0) return fail(m, DPLLM_ESTATE, "linear %d already holds %d pairs", id, DPLLM_MAX_PAIRS);
  Selector& s = lin->sel[slot];
  s.set = true; s.l = l; s.h = h; s.kind = kind; s.r = r; s.G = (const uint16_t*)G_dev;
  s.alpha = alpha; s.beta = beta; s.T = T;
  lin->active = slot;
  return DPLLM_OK;
}

int dpllm_set_threshold(dpllm_model* m, int id, int l, int h, float T) {
  int rc = DPLLM_OK;
  Linear* lin = get_linear(m, id, &rc);
  if (!lin) return rc;
  if (std::isnan(T)) return fail(m, DPLLM_EINVAL, "threshold is NaN");
  int slot = lin->find_pair(l, h);
  if (slot < 0) return fail(m, DPLLM_ESTATE, "pair (%d,%d) not set on linear %d", l, h, id);
  lin->sel[slot].T = T;
  return DPLLM_OK;
}

int dpllm_set_active_pair(dpllm_model* m, int id, int l, int h) {
  int rc = DPLLM_OK;
  Linear* lin = get_linear(m, id, &rc);
  if (!lin) return rc;
  int slot = lin->find_pair(l, h);
  if (slot < 0) return fail(m, DPLLM_ESTATE, "pair (%d,%d) not set on linear %d", l, h, id);
  lin->active = slot;
  return DPLLM_OK;
}

int dpllm_estimate(dpllm_model* m, int id, int l, int h, const void* x_dev, float* e_dev, int32_t* k_dev,
                   void* stream) {
  int rc = DPLLM_OK;
  Linear* lin = get_linear(m, id, &rc);
  if (!lin) return rc;
  if (!x_dev || !e_dev || !k_dev) return fail(m, DPLLM_EINVAL, "null pointer");
  if ((uintptr_t)x_dev % 16) return fail(m, DPLLM_EINVAL, "x not 16-byte aligned");
  int slot = lin->find_pair(l, h);
  if (slot < 0) return fail(m, DPLLM_ESTATE, "pair (%d,%d) not set on linear %d", l, h, id);
  return launch_selector(m, *lin, lin->sel[slot], x_dev, e_dev, k_dev, (hipStream_t)stream);
}

int dpllm_gemv(dpllm_model* m, int id, int k, const int32_t* k_dev, const void* x_dev, void* y_dev, int B,
               void* stream) {
  int rc = DPLLM_OK;
  Linear* lin = get_linear(m, id, &rc);
  if (!lin) return rc;
  if (!x_dev || !y_dev) return fail(m, DPLLM_EINVAL, "null pointer");
  if ((uintptr_t)x_dev % 16) return fail(m, DPLLM_EINVAL, "x not 16-byte aligned");
  if (B < 1 || B > DPLLM_MAX_BATCH) return fail(m, DPLLM_ESHAPE, "batch %d outside [1,%d]", B, DPLLM_MAX_BATCH);
  if (k >= 0) {
    if (k < lin->L.kmin || k > lin->L.p) return fail(m, DPLLM_ERANGE, "k=%d outside [%d,%d]", k, lin->L.kmin, lin->L.p);
    return launch_gemv(m, *lin, k, k, nullptr, x_dev, y_dev, B, (hipStream_t)stream);
  }
  if (!k_dev) return fail(m, DPLLM_EINVAL, "k < 0 needs k_dev");
  if (lin->active < 0) return fail(m, DPLLM_ESTATE, "linear %d has no active pair", id);
  const Selector& s = lin->sel[lin->active];
  return launch_gemv(m, *lin, s.l, s.h, k_dev, x_dev, y_dev, B, (hipStream_t)stream);
}

int dpllm_decode_step(dpllm_model* m, const void* const* xs, void* const* ys, int32_t* k_dev, float* e_dev,
                      void* stream) {
  if (!m) return DPLLM_EINVAL;
  if (!xs || !ys || !k_dev || !e_dev) return fail(m, DPLLM_EINVAL, "null pointer");
  const int n = (int)m->linears.size();
  for (int id = 0; id < n; ++id) {
    const Linear& lin = m->linears[id];
    if (!lin.loaded) return fail(m, DPLLM_ESTATE, "linear %d is not loaded", id);
    if (lin.active < 0) return fail(m, DPLLM_ESTATE, "linear %d has no selector", id);
    if (!xs[id] || !ys[id]) return fail(m, DPLLM_EINVAL, "null x or y for linear %d", id);
    if ((uintptr_t)xs[id] % 16) return fail(m, DPLLM_EINVAL, "x of linear %d not 16-byte aligned", id);
  }
  hipStream_t st = (hipStream_t)stream;
  for (int id = 0; id < n; ++id) {
    const Linear& lin = m->linears[id];
    const Selector& s = lin.sel[lin.active];
    int rc = launch_selector(m, lin, s, xs[id], e_dev + id, k_dev + id, st);
    if (rc != DPLLM_OK) return rc;
    rc = launch_gemv(m, lin, s.l, s.h, k_dev + id, xs[id], ys[id], 1, st);
    if (rc != DPLLM_OK) return rc;
  }
  return DPLLM_OK;
}

int dpllm_debug_unpack(dpllm_model* m, int id, int k, uint8_t* idx_dev, void* stream) {
  int rc = DPLLM_OK;
  Linear* lin = get_linear(m, id, &rc);
  if (!lin) return rc;
  if (!idx_dev) return fail(m, DPLLM_EINVAL, "null pointer");
  if (k < 1 || k > lin->L.p) return fail(m, DPLLM_ERANGE, "k=%d outside [1,%d]", k, lin->L.p);
  size_t n = (size_t)lin->L.out * lin->L.ncw;
  hipLaunchKernelGGL(debug_unpack_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, (hipStream_t)stream,
                     lin->planes(), lin->L.plane_bytes / 16, lin->L.p, k, lin->L.out, lin->L.ncw, idx_dev);
  HIP_TRY(m, hipGetLastError());
  return DPLLM_OK;
}

}  // extern "C"
