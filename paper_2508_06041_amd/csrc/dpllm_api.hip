// Host side of the C boundary declared in include/dpllm.h: argument checks, the model object,
// load-time re-tiling, launch planning and kernel launches.  No kernel arithmetic lives here.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "../../include/dpllm.h"
#include "aux_kernels.hpp"
#include "gemv_kernels.hpp"
#include "gemv_lane.hpp"
#include "layout.hpp"
#include "selector_kernels.hpp"

using namespace dpllm;

// Scratch of dpllm_estimate_noalloc: the partial dot products of one projection selector (rank up to
// kStaticMaxRank, every column chunking) or its sum x^2.  Every GPU the library runs on holds its own copy of the
// array until the process ends.  In host code the name is only a stand-in: the device address comes from
// hipGetSymbolAddress, once per device (static_scratch_ptr), and only that pointer is handed to kernels.
constexpr int kStaticMaxRank = 256;
constexpr size_t kStaticScratchSlots = (size_t)kSelMaxChunks * kStaticMaxRank;
static __device__ __align__(256) double scratch[kStaticScratchSlots];

namespace {

struct Pair {
  bool set = false;
  int l = 0, h = 0, kind = DPLLM_SEL_NONE, r = 0;
  const uint16_t* G = nullptr;
  float alpha = 0.f, beta = 0.f, T = 0.f;
};

struct TargetEntry {   // what a linear runs under one of the targets 1 .. DPLLM_MAX_TARGETS - 1
  bool set = false;
  int slot = 0;
  float T = 0.f;
};

struct Linear {
  bool loaded = false;
  LinearLayout L;
  char* arena = nullptr;
  Pair sel[DPLLM_MAX_PAIRS];
  int active = -1;                     // the pair of target 0
  TargetEntry tgt[DPLLM_MAX_TARGETS];  // [0] unused
  const void* sel_input = nullptr;     // decode step: the selector reads this vector instead of the linear's input
  int find_pair(int l, int h) const {
    for (int i = 0; i < DPLLM_MAX_PAIRS; ++i)
      if (sel[i].set && sel[i].l == l && sel[i].h == h) return i;
    return -1;
  }
  // what the launches are sized for: the properties of all pairs the linear holds, whichever is in use
  int max_rowgroups() const {
    int g = 0;
    for (const Pair& s : sel)
      if (s.set) g = std::max(g, sel_rowgroups_of(s.kind, s.r));
    return g;
  }
  int part_k() const {   // the bitwidth the work of a step launch is cut for: the larger one of the pair of target 0
    return active >= 0 ? sel[active].h : L.p;
  }
  bool streaming() const {   // every bitwidth its selectors can ask for has a decode scheme in the streaming kernel
    for (const Pair& s : sel)
      if (s.set && (s.l < kFastKMin || s.h > kFastKMax)) return false;
    return true;
  }
};

// A decode step is cut into phases: maximal runs of consecutive linears none of which reads or overwrites
// what an earlier linear of the run writes.  Inside a phase all selectors run in one launch and all GEMVs
// in another; phases run one after the other on the stream, so the result equals running the linears strictly
// in order.
struct Phase {
  int sel_first = 0, sel_count = 0;     // slice of the device selector job table
  int part_first = 0, part_count = 0;   // slice of the device selector part table
  int member_first = 0;                 // slice of the device table of group members
  int gemv_first = 0, gemv_count = 0;   // slice of the device GEMV job table (streaming kernel, one launch)
  int blocks = 0;                       // workgroups of that launch
  int block_first = 0;                  // slice of the device workgroup-to-job table
  std::vector<int> plain;               // linears served by the plain kernel, one launch each
  bool estimators = true;               // under some target a job of the selector launch has an estimator (else the launch is skipped)
  bool decide = false;                  // a linear of the selector launch is served by the plain kernel, which reads its
                                        // bitwidth from k_dev: the decisions of this launch are taken by a launch of their own
};
constexpr int kLanePoolRows = 8192;     // row blocks x splits of the column-split launches that may be in flight
constexpr size_t kSelOneSlots = (size_t)kSelMaxChunks * kSelMaxRank;

struct StepPlan {
  bool valid = false;
  uint64_t version = 0;
  std::vector<const void*> xs;
  std::vector<void*> ys;
  int32_t* k_dev = nullptr;
  float* e_dev = nullptr;
  std::vector<Phase> phases;
};

// The caller's workspace, carved once by dpllm_set_workspace.  Offsets in bytes, every region 256-byte aligned.
struct Workspace {
  char* base = nullptr;
  size_t bytes = 0;
  size_t lane_ws = 0, lane_cnt = 0;          // column-split pool: kLanePoolRows x 64 fp32, kLanePoolRows counters
  size_t est_ws = 0;                         // dpllm_estimate: kSelOneSlots fp64
  size_t target = 0;                         // the number of the active target
  size_t sel_params = 0;                     // SelParams [DPLLM_MAX_TARGETS][n]
  size_t sel_jobs = 0, sel_members = 0;      // SelJob [n], int32 [n]
  size_t sel_parts = 0, sel_parts_cap = 0;   // SelPart [cap]
  size_t sel_ws = 0, sel_ws_cap = 0;         // fp64 [cap]
  size_t gemv_jobs = 0;                      // GemvJob [n]
  size_t block_jobs = 0, block_jobs_cap = 0; // int32 [cap]
  size_t total = 0;
  template <class T>
  T* at(size_t off) const { return reinterpret_cast<T*>(base + off); }
};

}  // namespace

struct dpllm_model {
  std::vector<Linear> linears;
  std::string err;
  uint64_t version = 1;            // bumped by every call that changes what the launch plan depends on
  bool params_dirty = true;        // the device table of selector parameters is behind the host's
  StepPlan plan;
  Workspace ws;
  // host copies of what the plan puts into the workspace (kept so that the asynchronous copies have a source)
  std::vector<SelJob> h_sel_jobs;
  std::vector<SelPart> h_sel_parts;
  std::vector<int32_t> h_sel_members;
  std::vector<GemvJob> h_gemv_jobs;
  std::vector<int32_t> h_block_jobs;
  std::vector<SelParams> h_params;
  int device = 0;
};

namespace {

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

// ---- workspace ------------------------------------------------------------------------------------------------
// Sized for any launch plan over the linears as they stand (shapes, pairs): the caps are upper bounds.
Workspace carve_workspace(const dpllm_model* m) {
  Workspace w;
  const size_t n = m->linears.size();
  size_t parts = 0, slots = 0, blocks = 0;
  for (const Linear& lin : m->linears) {
    if (!lin.loaded) continue;
    const size_t rg = (size_t)std::max(1, lin.max_rowgroups());
    parts += rg * kSelMaxChunks + 1;
    slots += rg * kSelPartRows * kSelMaxChunks;
    blocks += (size_t)lin.L.nrq * 8;
  }
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, kAlign); return o; };
  w.lane_ws = take(sizeof(float) * 64 * kLanePoolRows);
  w.lane_cnt = take(sizeof(uint32_t) * kLanePoolRows);
  w.est_ws = take(sizeof(double) * kSelOneSlots);
  w.target = take(sizeof(int32_t));
  w.sel_params = take(sizeof(SelParams) * DPLLM_MAX_TARGETS * n);
  w.sel_jobs = take(sizeof(SelJob) * n);
  w.sel_members = take(sizeof(int32_t) * n);
  w.sel_parts_cap = parts;
  w.sel_parts = take(sizeof(SelPart) * parts);
  w.sel_ws_cap = slots;
  w.sel_ws = take(sizeof(double) * slots);
  w.gemv_jobs = take(sizeof(GemvJob) * n);
  w.block_jobs_cap = blocks;
  w.block_jobs = take(sizeof(int32_t) * blocks);
  w.total = off;
  return w;
}

// ---- selector ---------------------------------------------------------------------------------------------
SelParams make_params(const Pair& s, float T) {
  SelParams P;
  P.G = s.G;
  P.T = T; P.alpha = s.alpha; P.beta = s.beta;
  P.r = s.r; P.l = s.l; P.h = s.h; P.kind = s.kind;
  P.pad = 0;
  return P;
}

// launch_rowgroups: groups of 16 rows of G over all jobs of the launch.  A launch with fewer of them than
// would fill the chip cuts the columns into chunks (multiples of 512 columns) as well.
SelJob make_sel_job(const Linear& lin, int linear, int rowgroups, const void* x, float* e_dev, int32_t* k_dev, long launch_rowgroups) {
  SelJob j;
  j.x = (const uint16_t*)x;
  j.e_out = e_dev;
  j.k_out = k_dev;
  j.ws = nullptr;
  j.in = lin.L.in;
  j.linear = linear;
  j.nchunks = 1;
  j.chunk_cols = lin.L.in;
  if (rowgroups > 0) {
    // long rows are cut as well, so that the parts of a launch are of similar size (7B step: 32.5 -> 30.7 us)
    constexpr long max_cols = 4096;
    long want = std::min<long>(kSelMaxChunks, 1152 / std::max<long>(1, launch_rowgroups));   // 1280 parts run at once
    want = std::max<long>(want, std::min<long>(kSelMaxChunks, (lin.L.in + max_cols - 1) / max_cols));
    if (want > 1) {
      j.chunk_cols = (int)((lin.L.in + want - 1) / want + kSelChunkStep - 1) / kSelChunkStep * kSelChunkStep;   // <= want chunks
      j.nchunks = (lin.L.in + j.chunk_cols - 1) / j.chunk_cols;
    }
  }
  j.ws_rows = std::max(1, rowgroups) * kSelPartRows;
  j.pad = 0;
  return j;
}

// ---- GEMV -------------------------------------------------------------------------------------------------
GemvJob make_gemv_job(const Linear& lin, int k, const int32_t* k_dev, const void* x, void* y) {
  GemvJob j;
  j.arena = lin.arena;
  j.x = (const uint16_t*)x;
  j.y = (uint16_t*)y;
  j.k_dev = k_dev;
  j.has_fin = 0;
  j.fin = SelFinish{};
  j.plane_stride_u4 = (uint32_t)(lin.L.plane_bytes / 16);
  for (int kk = kFastKMin; kk <= kFastKMax; ++kk)
    j.lut_off[kk - kFastKMin] = (kk >= lin.L.kmin && kk <= lin.L.p) ? (uint32_t)lin.L.lut_offset[kk] : 0u;
  j.k = k;
  j.kmin = lin.L.kmin; j.p = lin.L.p;
  j.out = lin.L.out; j.ncw = lin.L.ncw; j.nrq = lin.L.nrq; j.ncc = lin.L.ncc;
  j.nblocks = lin.L.nrq;
  j.block_start = 0;
  j.nsamples = 1;
  j.nsplit = 1;
  j.ws = nullptr;
  j.cnt = nullptr;
  return j;
}

// Blocks of 64 rows one workgroup (eight wavefronts) streams.  A workgroup should run for the better part of a
// hundred microseconds (about 1 MiB of planes): shorter ones pay their start-up (job record, tables, first
// loads: a few microseconds of an otherwise idle slot) too often, longer ones leave the chip half empty at the
// end of the launch (measured on the 7B step: 0.25 MiB 496 us, 0.375 MiB 480, 0.75 MiB 471, 1 MiB 468, 2 MiB
// 477, 4 MiB 546); and a launch wants at least a few workgroups per compute unit.
constexpr long kLaneGroupBytes = 1048576;
// GEMV launches below this many workgroups take their selectors' decisions themselves; larger ones get a launch
// of its own for the decisions (measured on a 7B step of 3094 workgroups: 509 against 514 us)
constexpr int kFoldMaxBlocks = 1536;
constexpr int kLaneSplitBlocks = 256;   // a launch that splits columns aims at one workgroup per compute unit
int pick_blocks_per_group(const LinearLayout& L, int k, long total_blocks, long group_bytes = kLaneGroupBytes) {
  const long bytes_per_block = 64L * L.in * k / 8;
  long r = std::min<long>(16, std::max<long>(1, group_bytes / std::max<long>(1, bytes_per_block)));
  while (r > 1 && total_blocks / r < 1024) --r;
  return (int)r;
}

// Launches with fewer workgroups than compute units (a workgroup is tied to 64 rows): the workgroups that share
// a block of rows.  Measured on 4096 .. 28672 rows x 4096 .. 14336 columns: splitting pays only below about one
// workgroup per compute unit (64 blocks of rows: 23 -> 12 us at 14336 columns) and costs above it (172 blocks:
// 9 -> 12 us), since every split builds the tables again and runs fewer tiles per wavefront.
// workgroups = those of the whole launch before splitting; rows = blocks of rows x samples per pass x groups of
// the job; pool = what is left of the partial-sum pool.
int pick_lane_split(const LinearLayout& L, long workgroups, long rows, long pool) {
  long s = std::min<long>(8, kLaneSplitBlocks / std::max<long>(1, workgroups));
  s = std::min<long>(s, L.ncc / kLaneWaves);   // at least one tile per wavefront
  while (s > 1 && rows * s > pool) --s;
  return (int)std::max<long>(1, s);
}

template <int B>
void launch_plain_t(const GemvArgs& a, hipStream_t st) {
  hipLaunchKernelGGL(gemv_plain_kernel<B>, dim3((a.out + 15) / 16), dim3(256), 0, st, a);
}

int launch_plain(dpllm_model* m, const Linear& lin, int k, const int32_t* k_dev, const void* x, void* y, int B, hipStream_t st) {
  GemvArgs a;
  a.arena = lin.arena;
  a.plane_bytes = lin.L.plane_bytes;
  for (int kk = 0; kk <= 8; ++kk) a.lut_off[kk] = (kk >= lin.L.kmin && kk <= lin.L.p) ? (uint32_t)lin.L.lut_offset[kk] : 0u;
  a.k = k;
  a.k_dev = k_dev;
  a.kmin = lin.L.kmin; a.p = lin.L.p;
  a.x = (const uint16_t*)x;
  a.y = (uint16_t*)y;
  a.out = lin.L.out; a.in = lin.L.in; a.ncw = lin.L.ncw; a.ncc = lin.L.ncc;
  switch (B) {
    case 1: launch_plain_t<1>(a, st); break;
    case 2: launch_plain_t<2>(a, st); break;
    case 3: launch_plain_t<3>(a, st); break;
    case 4: launch_plain_t<4>(a, st); break;
    case 5: launch_plain_t<5>(a, st); break;
    case 6: launch_plain_t<6>(a, st); break;
    case 7: launch_plain_t<7>(a, st); break;
    case 8: launch_plain_t<8>(a, st); break;
    default: return fail(m, DPLLM_ESHAPE, "batch %d outside [1, %d]", B, DPLLM_MAX_BATCH);
  }
  HIP_TRY(m, hipGetLastError());
  return DPLLM_OK;
}

// one linear, B right-hand sides: a batch runs in groups of four samples that share one pass over the planes
int launch_gemv(dpllm_model* m, const Linear& lin, int k, const int32_t* k_dev, const void* x, void* y, int B, hipStream_t st) {
  const bool streaming = k_dev ? lin.L.kmin >= kFastKMin : (k >= kFastKMin && k <= kFastKMax);
  if (!streaming) return launch_plain(m, lin, k, k_dev, x, y, B, st);
  GemvJob j = make_gemv_job(lin, k, k_dev, x, y);
  const int rpb = pick_blocks_per_group(lin.L, k_dev ? lin.L.p : k, lin.L.nrq);
  j.nblocks = (lin.L.nrq + rpb - 1) / rpb;
  const long groups = B > 1 ? (B + 3) / 4 : 1, per_pass = B > 1 ? 4 : 1;
  if (m->ws.base) {   // without a workspace there is no pool for partial sums: no column split
    j.nsplit = pick_lane_split(lin.L, j.nblocks * groups, (long)lin.L.nrq * per_pass * groups, kLanePoolRows);
    j.nblocks *= j.nsplit;
    j.ws = m->ws.at<float>(m->ws.lane_ws);
    j.cnt = m->ws.at<uint32_t>(m->ws.lane_cnt);
  }
  if (B > 1)
    hipLaunchKernelGGL((gemv_lane_kernel<4>), dim3(j.nblocks * (unsigned)groups), dim3(kLaneThreads), 0, st, (const GemvJob*)nullptr,
                       (const int32_t*)nullptr, B, j, (const SelParams*)nullptr, (const int32_t*)nullptr, 0);
  else
    hipLaunchKernelGGL((gemv_lane_kernel<1>), dim3(j.nblocks), dim3(kLaneThreads), 0, st, (const GemvJob*)nullptr,
                       (const int32_t*)nullptr, 1, j, (const SelParams*)nullptr, (const int32_t*)nullptr, 0);
  HIP_TRY(m, hipGetLastError());
  return DPLLM_OK;
}

// ---- decode-step planning ------------------------------------------------------------------------------------
bool overlap(const void* a, size_t an, const void* b, size_t bn) {
  uintptr_t a0 = (uintptr_t)a, b0 = (uintptr_t)b;
  return a0 < b0 + bn && b0 < a0 + an;
}

// the table of selector parameters: row t = what every linear runs under target t (rows of targets that hold no
// entry of their own for a linear repeat target 0)
void fill_params(dpllm_model* m) {
  const size_t n = m->linears.size();
  m->h_params.assign((size_t)DPLLM_MAX_TARGETS * n, SelParams{});
  for (size_t i = 0; i < n; ++i) {
    const Linear& lin = m->linears[i];
    if (!lin.loaded || lin.active < 0) continue;
    const Pair& base = lin.sel[lin.active];
    for (int t = 0; t < DPLLM_MAX_TARGETS; ++t) {
      const TargetEntry& e = lin.tgt[t];
      const bool own = t > 0 && e.set && lin.sel[e.slot].set;
      m->h_params[(size_t)t * n + i] = own ? make_params(lin.sel[e.slot], e.T) : make_params(base, base.T);
    }
  }
}

int upload_params(dpllm_model* m, hipStream_t st) {
  fill_params(m);
  // a selector launch none of whose linears has an estimator under any target has nothing to compute
  const size_t n = m->linears.size();
  for (Phase& ph : m->plan.phases) {
    ph.estimators = false;
    for (int j = ph.sel_first; j < ph.sel_first + ph.sel_count && !ph.estimators; ++j)
      for (int t = 0; t < DPLLM_MAX_TARGETS && !ph.estimators; ++t)
        ph.estimators = m->h_params[(size_t)t * n + m->h_sel_jobs[j].linear].kind != DPLLM_SEL_NONE;
  }
  HIP_TRY(m, hipMemcpyAsync(m->ws.at<SelParams>(m->ws.sel_params), m->h_params.data(), sizeof(SelParams) * m->h_params.size(),
                            hipMemcpyHostToDevice, st));
  m->params_dirty = false;
  return DPLLM_OK;
}

int build_plan(dpllm_model* m, const void* const* xs, void* const* ys, int32_t* k_dev, float* e_dev, hipStream_t st) {
  const int n = (int)m->linears.size();
  const Workspace& W = m->ws;
  StepPlan& P = m->plan;
  P.valid = false;
  P.xs.assign(xs, xs + n);
  P.ys.assign(ys, ys + n);
  P.k_dev = k_dev;
  P.e_dev = e_dev;
  P.phases.clear();
  std::vector<SelJob>& sel_jobs = m->h_sel_jobs;
  std::vector<SelPart>& sel_parts = m->h_sel_parts;
  std::vector<int32_t>& sel_members = m->h_sel_members;
  sel_members.clear();
  std::vector<GemvJob>& gemv_jobs = m->h_gemv_jobs;
  std::vector<int32_t>& block_jobs = m->h_block_jobs;
  sel_jobs.clear(); sel_parts.clear(); gemv_jobs.clear(); block_jobs.clear();
  size_t ws_slots = 0;
  // phases: maximal runs of consecutive linears that do not depend on one another
  std::vector<std::pair<int, int>> bounds;
  std::vector<int> phase_of(n, 0);
  for (int id = 0; id < n;) {
    int end = id + 1;
    for (; end < n; ++end) {  // extend the phase while linear `end` is independent of all of [id, end)
      const Linear& le = m->linears[end];
      bool dep = false;
      for (int j = id; j < end && !dep; ++j) {
        const Linear& lj = m->linears[j];
        dep = overlap(xs[end], (size_t)le.L.in * 2, ys[j], (size_t)lj.L.out * 2) ||
              (le.sel_input && overlap(le.sel_input, (size_t)le.L.in * 2, ys[j], (size_t)lj.L.out * 2)) ||
              (lj.sel_input && overlap(ys[end], (size_t)le.L.out * 2, lj.sel_input, (size_t)lj.L.in * 2)) ||
              overlap(ys[end], (size_t)le.L.out * 2, xs[j], (size_t)lj.L.in * 2) ||
              overlap(ys[end], (size_t)le.L.out * 2, ys[j], (size_t)lj.L.out * 2);
      }
      if (dep) break;
    }
    for (int j = id; j < end; ++j) phase_of[j] = (int)bounds.size();
    bounds.emplace_back(id, end);
    id = end;
  }
  // A selector that reads its own input buffer (asynchronous estimation, Sec. 5.2) does not have to run right
  // before its linear: any phase from which on nothing writes that buffer before the linear runs will do.  It
  // joins the latest such phase that launches selectors anyway (for linears that estimate from their immediate
  // input), so that its own phase starts with the GEMV launch; without such a phase it stays where it is.
  std::vector<char> has_selectors(bounds.size(), 0);
  for (int j = 0; j < n; ++j)
    if (!m->linears[j].sel_input) has_selectors[phase_of[j]] = 1;
  std::vector<std::vector<int>> sel_of_phase(bounds.size());
  for (int j = 0; j < n; ++j) {
    const Linear& lin = m->linears[j];
    int q = phase_of[j];
    if (lin.sel_input) {
      int first = q;   // earliest phase the selector may run in
      while (first > 0) {
        bool written = false;
        for (int i = bounds[first - 1].first; i < bounds[first - 1].second && !written; ++i)
          written = overlap(lin.sel_input, (size_t)lin.L.in * 2, ys[i], (size_t)m->linears[i].L.out * 2);
        if (written) break;
        --first;
      }
      while (q > first && !has_selectors[q]) --q;
      if (!has_selectors[q]) q = phase_of[j];
      has_selectors[q] = 1;
    }
    sel_of_phase[q].push_back(j);
  }
  std::vector<int> sel_job_of(n, -1);   // index of every linear's selector job (it sits in its own phase or an earlier one)
  for (size_t pi = 0; pi < bounds.size(); ++pi) {
    long pool_used = 0;   // phases follow one another on the stream: each may use the whole partial-sum pool
    const int id = bounds[pi].first, end = bounds[pi].second;
    Phase ph;
    ph.sel_first = (int)sel_jobs.size();
    ph.sel_count = (int)sel_of_phase[pi].size();
    ph.part_first = (int)sel_parts.size();
    long launch_rowgroups = 0;
    for (int j : sel_of_phase[pi]) launch_rowgroups += m->linears[j].max_rowgroups();
    for (size_t local = 0; local < sel_of_phase[pi].size(); ++local) {
      const int j = sel_of_phase[pi][local];
      const Linear& lin = m->linears[j];
      const int rowgroups = lin.max_rowgroups();
      SelJob sj = make_sel_job(lin, j, rowgroups, lin.sel_input ? lin.sel_input : xs[j], e_dev + j, k_dev + j, launch_rowgroups);
      for (int part = 0; part < rowgroups * sj.nchunks; ++part) sel_parts.push_back(SelPart{(int)local, part, j, 0, 0, 0});
      sj.ws = W.at<double>(W.sel_ws) + ws_slots;
      ws_slots += (size_t)sj.ws_rows * sj.nchunks;
      sel_job_of[j] = (int)sel_jobs.size();
      if (!lin.streaming()) ph.decide = true;
      sel_jobs.push_back(sj);
    }
    // groups of jobs that read the same vector: one more part each, which adds up x^2 once for the members whose
    // estimator is the linear regression
    ph.member_first = (int)sel_members.size();
    for (int a = 0; a < ph.sel_count; ++a) {
      const SelJob& ja = sel_jobs[ph.sel_first + a];
      bool head = true;
      for (int b = 0; b < a && head; ++b) head = sel_jobs[ph.sel_first + b].x != ja.x || sel_jobs[ph.sel_first + b].in != ja.in;
      if (!head) continue;
      const int first = (int)sel_members.size() - ph.member_first;
      for (int b = a; b < ph.sel_count; ++b) {
        const SelJob& jb = sel_jobs[ph.sel_first + b];
        if (jb.x == ja.x && jb.in == ja.in) sel_members.push_back(b);
      }
      sel_parts.push_back(SelPart{a, -1, ja.linear, (int)sel_members.size() - ph.member_first - first, first, 0});
    }
    ph.part_count = (int)sel_parts.size() - ph.part_first;
    // GEMV jobs of the phase: one launch of the streaming kernel for all linears it serves
    ph.gemv_first = (int)gemv_jobs.size();
    ph.block_first = (int)block_jobs.size();
    long total_rq = 0, lane_groups = 0;
    for (int j = id; j < end; ++j)
      if (m->linears[j].streaming()) total_rq += m->linears[j].L.nrq;
    // The chip runs 512 workgroups at a time.  A launch of a few such rounds loses the unfilled part of its last
    // round (2.7 rounds cost 3): the work per workgroup is scaled, between half and one and a half times the
    // usual megabyte, to the value with the smallest estimate of rounds x (start-up + work of a workgroup).
    long base_bytes = kLaneGroupBytes;
    {
      double best = 1e300;
      for (int pct = 50; pct <= 150; pct += 5) {
        const long gb = kLaneGroupBytes * pct / 100;
        long groups = 0;
        for (int j = id; j < end; ++j) {
          const Linear& lin = m->linears[j];
          if (!lin.streaming()) continue;
          const int rpb = pick_blocks_per_group(lin.L, lin.part_k(), total_rq, gb);
          groups += (lin.L.nrq + rpb - 1) / rpb;
        }
        const double rounds = std::ceil(groups / 512.0);
        const double est = rounds * (4.0 + 85.0 * pct / 100) * (1.0 + 0.0005 * std::abs(pct - 100));   // ties: the usual size
        if (est < best) { best = est; base_bytes = gb; lane_groups = groups; }
      }
    }
    std::vector<long> bytes_after(end - id, 0);   // plane bytes of the launch that follow linear j
    {
      long acc = 0;
      for (int j = end - 1; j >= id; --j) {
        const Linear& lin = m->linears[j];
        if (!lin.streaming()) continue;
        bytes_after[j - id] = acc;
        acc += (long)lin.L.nrq * 64 * lin.L.in * lin.part_k() / 8;
      }
    }
    // Large launches: the linears dispatched last (one round of workgroups: two on each of 256 compute units)
    // get workgroups of half the usual work, so that the chip drains in less time at the end of the launch
    // (measured on the 7B step: 0.5 - 0.8 % of the launch; quarters and eighths did not add to that).
    const bool taper = lane_groups >= 2048;
    int blocks = 0;
    for (int j = id; j < end; ++j) {
      const Linear& lin = m->linears[j];
      if (!lin.streaming()) { ph.plain.push_back(j); continue; }
      GemvJob gj = make_gemv_job(lin, 0, k_dev + j, xs[j], ys[j]);
      gj.has_fin = 1;
      gj.fin = sel_finish_of(sel_jobs[sel_job_of[j]]);
      long group_bytes = base_bytes;
      if (taper && bytes_after[j - id] < 512 * base_bytes) group_bytes /= 2;
      const int rpb = pick_blocks_per_group(lin.L, lin.part_k(), total_rq, group_bytes);
      gj.nblocks = (lin.L.nrq + rpb - 1) / rpb;
      gj.nsplit = pick_lane_split(lin.L, lane_groups, lin.L.nrq, kLanePoolRows - pool_used);
      if (gj.nsplit > 1) {
        gj.nblocks *= gj.nsplit;
        gj.ws = W.at<float>(W.lane_ws) + pool_used * 64;
        gj.cnt = W.at<uint32_t>(W.lane_cnt) + pool_used;
        pool_used += (long)lin.L.nrq * gj.nsplit;
      }
      gj.block_start = blocks;
      blocks += gj.nblocks;
      block_jobs.insert(block_jobs.end(), gj.nblocks, (int32_t)(gemv_jobs.size() - ph.gemv_first));
      gemv_jobs.push_back(gj);
    }
    ph.gemv_count = (int)gemv_jobs.size() - ph.gemv_first;
    ph.blocks = blocks;
    P.phases.push_back(ph);
  }
  if (sel_parts.size() > W.sel_parts_cap || ws_slots > W.sel_ws_cap || block_jobs.size() > W.block_jobs_cap)
    return fail(m, DPLLM_ESTATE, "workspace too small for this step (set after the model changed?): call dpllm_workspace_bytes and "
                                 "dpllm_set_workspace again");
  // The tables may still be read by a step enqueued earlier on this stream: the copies are ordered behind it.
  if (!sel_parts.empty())
    HIP_TRY(m, hipMemcpyAsync(W.at<SelPart>(W.sel_parts), sel_parts.data(), sizeof(SelPart) * sel_parts.size(), hipMemcpyHostToDevice, st));
  if (!block_jobs.empty())
    HIP_TRY(m, hipMemcpyAsync(W.at<int32_t>(W.block_jobs), block_jobs.data(), sizeof(int32_t) * block_jobs.size(), hipMemcpyHostToDevice, st));
  HIP_TRY(m, hipMemcpyAsync(W.at<SelJob>(W.sel_jobs), sel_jobs.data(), sizeof(SelJob) * sel_jobs.size(), hipMemcpyHostToDevice, st));
  HIP_TRY(m, hipMemcpyAsync(W.at<int32_t>(W.sel_members), sel_members.data(), sizeof(int32_t) * sel_members.size(), hipMemcpyHostToDevice, st));
  if (!gemv_jobs.empty())
    HIP_TRY(m, hipMemcpyAsync(W.at<GemvJob>(W.gemv_jobs), gemv_jobs.data(), sizeof(GemvJob) * gemv_jobs.size(), hipMemcpyHostToDevice, st));
  P.version = m->version;
  P.valid = true;
  m->params_dirty = true;   // the phases' estimator flags are worked out with the parameter table
  return DPLLM_OK;
}

// device address of `scratch` on the current device, looked up on the first call on that device
constexpr int kMaxDevices = 64;
int static_scratch_ptr(dpllm_model* m, double** out) {
  static double* ptr[kMaxDevices] = {};
  int dev = 0;
  HIP_TRY(m, hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return fail(m, DPLLM_EINVAL, "device %d outside [0,%d)", dev, kMaxDevices);
  if (!ptr[dev]) {
    void* p = nullptr;
    HIP_TRY(m, hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return fail(m, DPLLM_EHIP, "hipGetSymbolAddress returned a null address");
    ptr[dev] = (double*)p;
  }
  *out = ptr[dev];
  return DPLLM_OK;
}

bool capturing(hipStream_t st) {
  hipStreamCaptureStatus s = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing(st, &s) != hipSuccess) { (void)hipGetLastError(); return false; }
  return s != hipStreamCaptureStatusNone;
}

}  // namespace

extern "C" {

int dpllm_model_create(dpllm_model** out, int n_linears) {
  if (!out || n_linears < 1) return DPLLM_EINVAL;
  *out = nullptr;
  dpllm_model* m = new (std::nothrow) dpllm_model();
  if (!m) return DPLLM_EINVAL;
  m->linears.resize(n_linears);
  if (hipGetDevice(&m->device) != hipSuccess) {
    (void)hipGetLastError();
    delete m;
    return DPLLM_EHIP;
  }
  *out = m;
  return DPLLM_OK;
}

void dpllm_model_destroy(dpllm_model* m) { delete m; }

const char* dpllm_last_error(const dpllm_model* m) { return m ? m->err.c_str() : "null model"; }

int dpllm_linear_device_bytes(int out, int in, int p, int kmin, size_t* bytes) {
  if (!bytes) return DPLLM_EINVAL;
  int rc = check_shape(out, in, p, kmin);
  if (rc != DPLLM_OK) return rc;
  *bytes = LinearLayout::make(out, in, p, kmin).total_bytes;
  return DPLLM_OK;
}

int dpllm_debug_locate(int out, int in, int p, int kmin, int plane, int row, int col, size_t* byte_offset, int* bit) {
  if (!byte_offset || !bit) return DPLLM_EINVAL;
  int rc = check_shape(out, in, p, kmin);
  if (rc != DPLLM_OK) return rc;
  if (plane < 0 || plane >= p || row < 0 || row >= out || col < 0 || col >= in) return DPLLM_ERANGE;
  const LinearLayout L = LinearLayout::make(out, in, p, kmin);
  // the word of the tile, the column's position inside it, and the rotation of plane b (see layout_device.hpp)
  const size_t word = plane_word_index(row, col / 32, L.ncc);
  *byte_offset = (size_t)plane * L.plane_bytes + word * 4;
  *bit = ((col_to_pos(col % 32) - plane) % 32 + 32) % 32;
  return DPLLM_OK;
}

int dpllm_workspace_bytes(const dpllm_model* m, size_t* bytes) {
  if (!m || !bytes) return DPLLM_EINVAL;
  *bytes = carve_workspace(m).total;
  return DPLLM_OK;
}

int dpllm_set_workspace(dpllm_model* m, void* ws_dev, size_t bytes, void* stream) {
  if (!m) return DPLLM_EINVAL;
  if (!ws_dev) return fail(m, DPLLM_EINVAL, "null workspace");
  if ((uintptr_t)ws_dev % kAlign) return fail(m, DPLLM_EINVAL, "workspace not %zu-byte aligned", kAlign);
  Workspace w = carve_workspace(m);
  if (bytes < w.total) return fail(m, DPLLM_ESTATE, "workspace holds %zu bytes, %zu needed", bytes, w.total);
  w.base = (char*)ws_dev;
  w.bytes = bytes;
  hipStream_t st = (hipStream_t)stream;
  // counters and the target word start at zero; everything else is written before it is read
  struct { size_t off, words; } zero[] = {{w.lane_cnt, (size_t)kLanePoolRows}, {w.target, 1}};
  for (const auto& z : zero)
    hipLaunchKernelGGL(fill_u32_kernel, dim3((unsigned)((z.words + 255) / 256)), dim3(256), 0, st, w.at<uint32_t>(z.off), z.words, 0u);
  HIP_TRY(m, hipGetLastError());
  m->ws = w;
  m->params_dirty = true;
  m->version++;
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
  if (!src_on_device) {   // host sources pass through a device staging buffer that lives for the length of this call
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
    size_t n = (size_t)L.nrq * L.ncc * 64 * p;
    hipLaunchKernelGGL(retile_planes_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, d_planes,
                       (uint4*)dev_arena, p, out, L.ncw, L.ncc, L.nrq, L.plane_bytes / 16);
  }
  const char* lsrc = staging ? (const char*)staging + plane_words * 4 : nullptr;
  for (int k = kmin; k <= p; ++k) {
    const uint16_t* src = staging ? (const uint16_t*)lsrc : luts[k - kmin];
    size_t n = (size_t)L.rows_padded << k;
    hipLaunchKernelGGL(copy_lut_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, src,
                       (uint16_t*)((char*)dev_arena + L.lut_offset[k]), out, L.rows_padded, 1 << k);
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
  m->version++;
  m->params_dirty = true;
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
  Pair& s = lin->sel[slot];
  // the launch plan is sized by the ranks and bitwidths of all pairs of the linear: it survives a change of G,
  // alpha, beta or T
  const bool same_shape = s.set && lin->active == slot && s.kind == kind && sel_rowgroups_of(s.kind, s.r) == sel_rowgroups_of(kind, r);
  s.set = true; s.l = l; s.h = h; s.kind = kind; s.r = kind == DPLLM_SEL_PROJ ? r : 0; s.G = (const uint16_t*)G_dev;
  s.alpha = alpha; s.beta = beta; s.T = T;
  lin->active = slot;
  if (!same_shape) m->version++;
  m->params_dirty = true;
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
  m->params_dirty = true;
  return DPLLM_OK;
}

int dpllm_set_active_pair(dpllm_model* m, int id, int l, int h) {
  int rc = DPLLM_OK;
  Linear* lin = get_linear(m, id, &rc);
  if (!lin) return rc;
  int slot = lin->find_pair(l, h);
  if (slot < 0) return fail(m, DPLLM_ESTATE, "pair (%d,%d) not set on linear %d", l, h, id);
  if (lin->active < 0 || lin->sel[lin->active].h != lin->sel[slot].h) m->version++;   // the step's work is cut for h
  lin->active = slot;
  m->params_dirty = true;
  return DPLLM_OK;
}

int dpllm_set_target_entry(dpllm_model* m, int target, int id, int l, int h, float T) {
  int rc = DPLLM_OK;
  Linear* lin = get_linear(m, id, &rc);
  if (!lin) return rc;
  if (target < 1 || target >= DPLLM_MAX_TARGETS) return fail(m, DPLLM_EINVAL, "target %d outside [1,%d]", target, DPLLM_MAX_TARGETS - 1);
  if (std::isnan(T)) return fail(m, DPLLM_EINVAL, "threshold is NaN");
  int slot = lin->find_pair(l, h);
  if (slot < 0) return fail(m, DPLLM_ESTATE, "pair (%d,%d) not set on linear %d", l, h, id);
  lin->tgt[target].set = true;
  lin->tgt[target].slot = slot;
  lin->tgt[target].T = T;
  m->params_dirty = true;
  return DPLLM_OK;
}

int dpllm_set_target(dpllm_model* m, int target, void* stream) {
  if (!m) return DPLLM_EINVAL;
  if (target < 0 || target >= DPLLM_MAX_TARGETS) return fail(m, DPLLM_EINVAL, "target %d outside [0,%d]", target, DPLLM_MAX_TARGETS - 1);
  if (!m->ws.base) return fail(m, DPLLM_ESTATE, "no workspace set");
  hipLaunchKernelGGL(fill_u32_kernel, dim3(1), dim3(64), 0, (hipStream_t)stream, m->ws.at<uint32_t>(m->ws.target), (size_t)1,
                     (uint32_t)target);
  HIP_TRY(m, hipGetLastError());
  return DPLLM_OK;
}

int dpllm_set_selector_input(dpllm_model* m, int id, const void* xsel_dev) {
  int rc = DPLLM_OK;
  Linear* lin = get_linear(m, id, &rc);
  if (!lin) return rc;
  if ((uintptr_t)xsel_dev % 16) return fail(m, DPLLM_EINVAL, "selector input not 16-byte aligned");
  lin->sel_input = xsel_dev;
  m->version++;
  return DPLLM_OK;
}

// the two launches of a lone estimate: the parts leave their partial results in `slots`, the decide kernel finishes
static int launch_estimate(dpllm_model* m, const Linear& lin, int id, const Pair& sel, const void* x_dev, float* e_dev, int32_t* k_dev,
                           double* slots, hipStream_t st) {
  const int rowgroups = sel_rowgroups_of(sel.kind, sel.r);
  SelJob j = make_sel_job(lin, id, rowgroups, x_dev, e_dev, k_dev, rowgroups);
  j.ws = slots;
  const SelParams P = make_params(sel, sel.T);
  const int blocks = sel.kind == DPLLM_SEL_PROJ ? rowgroups * j.nchunks : sel.kind == DPLLM_SEL_LINREG ? 1 : 0;
  if (blocks > 0)
    hipLaunchKernelGGL(selector_part_kernel, dim3(blocks), dim3(kSelPartThreads), 0, st, (const SelJob*)nullptr,
                       (const SelPart*)nullptr, (const int32_t*)nullptr, (const SelParams*)nullptr, (const int32_t*)nullptr, 0, j, P);
  hipLaunchKernelGGL(selector_decide_kernel, dim3(1), dim3(kSelDecideThreads), 0, st, (const SelJob*)nullptr,
                     (const SelParams*)nullptr, (const int32_t*)nullptr, 0, j, P);
  HIP_TRY(m, hipGetLastError());
  return DPLLM_OK;
}

static int check_estimate_args(dpllm_model* m, int id, int l, int h, const void* x_dev, float* e_dev, int32_t* k_dev, Linear** lin,
                               int* slot) {
  int rc = DPLLM_OK;
  *lin = get_linear(m, id, &rc);
  if (!*lin) return rc;
  if (!x_dev || !e_dev || !k_dev) return fail(m, DPLLM_EINVAL, "null pointer");
  if ((uintptr_t)x_dev % 16) return fail(m, DPLLM_EINVAL, "x not 16-byte aligned");
  *slot = (*lin)->find_pair(l, h);
  if (*slot < 0) return fail(m, DPLLM_ESTATE, "pair (%d,%d) not set on linear %d", l, h, id);
  return DPLLM_OK;
}

int dpllm_estimate(dpllm_model* m, int id, int l, int h, const void* x_dev, float* e_dev, int32_t* k_dev,
                   void* stream) {
  Linear* lin = nullptr;
  int slot = -1;
  int rc = check_estimate_args(m, id, l, h, x_dev, e_dev, k_dev, &lin, &slot);
  if (rc != DPLLM_OK) return rc;
  if (!m->ws.base) return fail(m, DPLLM_ESTATE, "no workspace set");
  return launch_estimate(m, *lin, id, lin->sel[slot], x_dev, e_dev, k_dev, m->ws.at<double>(m->ws.est_ws), (hipStream_t)stream);
}

int dpllm_estimate_noalloc(dpllm_model* m, int id, int l, int h, const void* x_dev, float* e_dev, int32_t* k_dev,
                           void* stream) {
  Linear* lin = nullptr;
  int slot = -1;
  int rc = check_estimate_args(m, id, l, h, x_dev, e_dev, k_dev, &lin, &slot);
  if (rc != DPLLM_OK) return rc;
  const Pair& sel = lin->sel[slot];
  if (sel.kind == DPLLM_SEL_PROJ && sel.r > kStaticMaxRank)
    return fail(m, DPLLM_ERANGE, "rank %d beyond the static scratch (at most %d): use dpllm_estimate with a workspace", sel.r, kStaticMaxRank);
  double* slots = nullptr;
  rc = static_scratch_ptr(m, &slots);
  if (rc != DPLLM_OK) return rc;
  // nothing in the scratch has to start at zero: every slot the decide kernel reads is written by the parts of
  // this call first (the previous call's contents are never read)
  return launch_estimate(m, *lin, id, sel, x_dev, e_dev, k_dev, slots, (hipStream_t)stream);
}

int dpllm_gemv(dpllm_model* m, int id, int k, const int32_t* k_dev, const void* x_dev, void* y_dev, int B,
               void* stream) {
  int rc = DPLLM_OK;
  Linear* lin = get_linear(m, id, &rc);
  if (!lin) return rc;
  if (!x_dev || !y_dev) return fail(m, DPLLM_EINVAL, "null pointer");
  if ((uintptr_t)x_dev % 16) return fail(m, DPLLM_EINVAL, "x not 16-byte aligned");
  if (B < 1 || B > DPLLM_MAX_BATCH) return fail(m, DPLLM_ESHAPE, "batch %d outside [1,%d]", B, DPLLM_MAX_BATCH);
  if (overlap(x_dev, (size_t)B * lin->L.in * 2, y_dev, (size_t)B * lin->L.out * 2)) return fail(m, DPLLM_EINVAL, "x and y overlap");
  if (k >= 0) {
    if (k < lin->L.kmin || k > lin->L.p) return fail(m, DPLLM_ERANGE, "k=%d outside [%d,%d]", k, lin->L.kmin, lin->L.p);
    return launch_gemv(m, *lin, k, nullptr, x_dev, y_dev, B, (hipStream_t)stream);
  }
  if (!k_dev) return fail(m, DPLLM_EINVAL, "k < 0 needs k_dev");
  return launch_gemv(m, *lin, 0, k_dev, x_dev, y_dev, B, (hipStream_t)stream);
}

int dpllm_decode_step_parts(dpllm_model* m, const void* const* xs, void* const* ys, int32_t* k_dev, float* e_dev,
                            int parts, void* stream) {
  if (!m) return DPLLM_EINVAL;
  if (parts < 1 || parts > (DPLLM_STEP_SELECT | DPLLM_STEP_GEMV)) return fail(m, DPLLM_EINVAL, "bad parts %d", parts);
  if (!xs || !ys || !k_dev || !e_dev) return fail(m, DPLLM_EINVAL, "null pointer");
  if (!m->ws.base) return fail(m, DPLLM_ESTATE, "no workspace set");
  const int n = (int)m->linears.size();
  hipStream_t st = (hipStream_t)stream;
  StepPlan& P = m->plan;
  bool reuse = P.valid && P.version == m->version && P.k_dev == k_dev && P.e_dev == e_dev &&
               std::equal(xs, xs + n, P.xs.begin()) && std::equal(ys, ys + n, P.ys.begin());
  if ((!reuse || m->params_dirty) && capturing(st))
    return fail(m, DPLLM_ESTATE, "the model changed since its last step: run one step outside stream capture first");
  if (!reuse) {
    for (int id = 0; id < n; ++id) {
      const Linear& lin = m->linears[id];
      if (!lin.loaded) return fail(m, DPLLM_ESTATE, "linear %d is not loaded", id);
      if (lin.active < 0) return fail(m, DPLLM_ESTATE, "linear %d has no selector", id);
      if (!xs[id] || !ys[id]) return fail(m, DPLLM_EINVAL, "null x or y for linear %d", id);
      if ((uintptr_t)xs[id] % 16) return fail(m, DPLLM_EINVAL, "x of linear %d not 16-byte aligned", id);
      if (overlap(xs[id], (size_t)lin.L.in * 2, ys[id], (size_t)lin.L.out * 2)) return fail(m, DPLLM_EINVAL, "x and y of linear %d overlap", id);
    }
    int rc = build_plan(m, xs, ys, k_dev, e_dev, st);
    if (rc != DPLLM_OK) return rc;
  }
  if (m->params_dirty) {
    int rc = upload_params(m, st);
    if (rc != DPLLM_OK) return rc;
  }
  const Workspace& W = m->ws;
  SelJob none{};
  GemvJob gnone{};
  SelParams pnone{};
  const SelParams* d_params = W.at<SelParams>(W.sel_params);
  const int32_t* d_target = W.at<int32_t>(W.target);
  const bool both = parts == (DPLLM_STEP_SELECT | DPLLM_STEP_GEMV);
  for (const Phase& ph : P.phases) {
    const bool fold = both && !ph.decide && ph.blocks < kFoldMaxBlocks;
    if ((parts & DPLLM_STEP_SELECT) && ph.sel_count > 0) {
      const SelJob* jobs = W.at<SelJob>(W.sel_jobs) + ph.sel_first;
      if (ph.estimators)
        hipLaunchKernelGGL(selector_part_kernel, dim3(ph.part_count), dim3(kSelPartThreads), 0, st, jobs,
                           (const SelPart*)(W.at<SelPart>(W.sel_parts) + ph.part_first),
                           (const int32_t*)(W.at<int32_t>(W.sel_members) + ph.member_first), d_params, d_target, n, none, pnone);
      // Whole step: the GEMV workgroups take the decisions of their linears themselves (one launch fewer per
      // dependency level).  Selectors alone, a linear on the plain kernel, or a GEMV launch of so many workgroups
      // that repeating the decision in each of them costs more than a launch: a launch that finishes every job of
      // this selector launch.
      if (!fold)
        hipLaunchKernelGGL(selector_decide_kernel, dim3(ph.sel_count), dim3(kSelDecideThreads), 0, st, jobs, d_params, d_target, n, none, pnone);
    }
    if (!(parts & DPLLM_STEP_GEMV)) continue;
    if (ph.gemv_count > 0)
      hipLaunchKernelGGL((gemv_lane_kernel<1>), dim3(ph.blocks), dim3(kLaneThreads), 0, st,
                         (const GemvJob*)(W.at<GemvJob>(W.gemv_jobs) + ph.gemv_first), (const int32_t*)(W.at<int32_t>(W.block_jobs) + ph.block_first),
                         ph.gemv_count, gnone, fold ? d_params : (const SelParams*)nullptr, d_target, n);
    for (int j : ph.plain) {
      int rc = launch_plain(m, m->linears[j], 0, k_dev + j, xs[j], ys[j], 1, st);
      if (rc != DPLLM_OK) return rc;
    }
  }
  HIP_TRY(m, hipGetLastError());
  return DPLLM_OK;
}

int dpllm_decode_step(dpllm_model* m, const void* const* xs, void* const* ys, int32_t* k_dev, float* e_dev,
                      void* stream) {
  return dpllm_decode_step_parts(m, xs, ys, k_dev, e_dev, DPLLM_STEP_SELECT | DPLLM_STEP_GEMV, stream);
}

int dpllm_debug_unpack(dpllm_model* m, int id, int k, uint8_t* idx_dev, void* stream) {
  int rc = DPLLM_OK;
  Linear* lin = get_linear(m, id, &rc);
  if (!lin) return rc;
  if (!idx_dev) return fail(m, DPLLM_EINVAL, "null pointer");
  if (k < 1 || k > lin->L.p) return fail(m, DPLLM_ERANGE, "k=%d outside [1,%d]", k, lin->L.p);
  size_t n = (size_t)lin->L.out * lin->L.ncw;
  hipLaunchKernelGGL(debug_unpack_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, (hipStream_t)stream,
                     (const uint32_t*)lin->arena, lin->L.plane_bytes / 4, lin->L.p, k, lin->L.out, lin->L.ncw, lin->L.ncc, idx_dev);
  HIP_TRY(m, hipGetLastError());
  return DPLLM_OK;
}

int dpllm_debug_copy(void* dst_dev, const void* src_dev, size_t bytes, void* stream) {
  if (!dst_dev || !src_dev || bytes % 16 || ((uintptr_t)dst_dev | (uintptr_t)src_dev) % 16) return DPLLM_EINVAL;
  hipLaunchKernelGGL(plain_copy_kernel, dim3(256 * 16), dim3(256), 0, (hipStream_t)stream, (const uint4*)src_dev,
                     (uint4*)dst_dev, bytes / 16);
  return hipGetLastError() == hipSuccess ? DPLLM_OK : DPLLM_EHIP;
}

int dpllm_debug_read(const void* src_dev, size_t bytes, void* sink_dev, void* stream) {
  if (!src_dev || !sink_dev || bytes % 16 || ((uintptr_t)src_dev | (uintptr_t)sink_dev) % 16) return DPLLM_EINVAL;
  hipLaunchKernelGGL(plain_read_kernel, dim3(256 * 8), dim3(256), 0, (hipStream_t)stream, (const uint4*)src_dev,
                     bytes / 16, (uint4*)sink_dev);
  return hipGetLastError() == hipSuccess ? DPLLM_OK : DPLLM_EHIP;
}

}  // extern "C"
