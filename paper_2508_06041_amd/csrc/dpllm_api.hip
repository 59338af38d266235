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
#include "gemv_fast.hpp"
#include "gemv_kernels.hpp"
#include "gemv_lane.hpp"
#include "layout.hpp"
#include "selector_kernels.hpp"

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
  const void* sel_input = nullptr;   // decode step: the selector reads this vector instead of the linear's input
  const uint4* planes() const { return reinterpret_cast<const uint4*>(arena); }
  const uint16_t* lut(int k) const { return reinterpret_cast<const uint16_t*>(arena + L.lut_offset[k]); }
  int find_pair(int l, int h) const {
    for (int i = 0; i < DPLLM_MAX_PAIRS; ++i)
      if (sel[i].set && sel[i].l == l && sel[i].h == h) return i;
    return -1;
  }
};

// A decode step is cut into phases: maximal runs of consecutive linears none of which reads or overwrites
// what an earlier linear of the run writes.  Inside a phase all selectors run in one launch and all GEMVs
// of one candidate pair in another; phases run one after the other on the stream, so the result equals
// running the linears strictly in order.
struct GemvLaunch {
  int ka, kb;          // kernel instance; ka == kb == 0: the plain kernel, one launch per job
  int mode;            // arrangement of the planes of the linears in this launch
  int first, count;    // slice of the device job table
  int blocks;          // workgroups of the launch
  int block_first;     // slice of the device workgroup-to-job table
};
struct Phase {
  int sel_first, sel_count;     // slice of the device selector job table
  int part_first, part_count;   // slice of the device selector part table
  std::vector<GemvLaunch> gemv;
};
constexpr int kLanePoolRows = 8192;
constexpr size_t kSelOneSlots = (size_t)kSelMaxChunks * kSelMaxRank;

struct StepPlan {
  bool valid = false;
  uint64_t version = 0;
  std::vector<const void*> xs;
  std::vector<void*> ys;
  int32_t* k_dev = nullptr;
  float* e_dev = nullptr;
  std::vector<Phase> phases;
  std::vector<GemvJob> gemv_jobs;   // host copies (also used for plain launches)
  std::vector<int> gemv_ids;        // linear id of every gemv job
};

}  // namespace

struct dpllm_model {
  std::vector<Linear> linears;
  std::string err;
  uint64_t version = 1;            // bumped by every call that changes what a plan depends on
  int layout = kLayoutRowLane;     // arrangement given to linears loaded from now on
  // decode-step plan and its device tables
  StepPlan plan;
  SelJob* d_sel_jobs = nullptr;
  SelPart* d_sel_parts = nullptr;
  size_t sel_parts_cap = 0;
  double* d_sel_ws = nullptr;       // the workspace slots of every selector job of the plan
  size_t sel_ws_cap = 0;
  double* d_sel_ws_one = nullptr;   // kSelMaxChunks x kSelMaxRank slots for dpllm_estimate, then its arrival counter
  uint32_t* d_sel_tickets = nullptr;  // one arrival counter per linear of the plan, zero between launches
  GemvJob* d_gemv_jobs = nullptr;
  int32_t* d_block_jobs = nullptr;   // for every workgroup of every multi-job GEMV launch of the plan: its job
  size_t block_jobs_cap = 0;
  // column-split launches of the row-per-lane kernel: partial sums (kLanePoolRows x 64 fp32) and arrival counters
  // (kLanePoolRows, zero whenever no launch is running); one launch at a time uses them
  float* d_lane_ws = nullptr;
  uint32_t* d_lane_cnt = nullptr;
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

// ---- selector ---------------------------------------------------------------------------------------------
// launch_rowgroups: groups of 16 rows of G over all jobs of the launch.  A launch with fewer of them than
// would fill the chip cuts the columns into chunks (multiples of 512 columns) as well.
SelJob make_sel_job(const Linear& lin, const Selector& s, const void* x, float* e_dev, int32_t* k_dev, long launch_rowgroups) {
  SelJob j;
  j.G = s.G;
  j.x = (const uint16_t*)x;
  j.e_out = e_dev;
  j.k_out = k_dev;
  j.T = s.T; j.alpha = s.alpha; j.beta = s.beta;
  j.in = lin.L.in; j.r = s.r;
  j.l = s.l; j.h = s.h; j.kind = s.kind;
  j.nchunks = 1;
  j.chunk_cols = lin.L.in;
  if (s.kind == 1) {
    // long rows are cut as well, so that the parts of a launch are of similar size (7B step: 32.5 -> 30.7 us)
    constexpr long max_cols = 4096;
    long want = std::min<long>(kSelMaxChunks, 512 / std::max<long>(1, launch_rowgroups));
    want = std::max<long>(want, std::min<long>(kSelMaxChunks, (lin.L.in + max_cols - 1) / max_cols));
    if (want > 1) {
      j.chunk_cols = (int)((lin.L.in + want - 1) / want + kSelChunkStep - 1) / kSelChunkStep * kSelChunkStep;   // <= want chunks
      j.nchunks = (lin.L.in + j.chunk_cols - 1) / j.chunk_cols;
    }
  }
  j.nparts = sel_rowgroups_of(s.kind, s.r) * j.nchunks;
  j.ws = nullptr;
  j.ticket = nullptr;
  return j;
}

// ---- GEMV -------------------------------------------------------------------------------------------------
// Kernel instances: a fixed bitwidth k (k, k) and the adjacent candidate pairs (k, k + 1), k >= 3.  Anything
// else (k < 3, non-adjacent pairs) is served by the plain kernel.  A batch of B right-hand sides runs in
// groups of two (B = 2) or four samples inside one launch; a group decodes every weight once and multiplies it
// with each of its samples.
bool has_fast_kernel(int ka, int kb) { return ka >= 3 && kb <= 8 && (kb == ka || kb == ka + 1); }

// Right-hand sides that share one pass over the planes.  A batch B runs as ceil(B / group) groups.
template <int KA, int KB, int NB>
void launch_group_t(int njobs, const GemvJob& one, hipStream_t st) {
  const int groups = (njobs + NB - 1) / NB;
  hipLaunchKernelGGL((gemv_kernel<KA, KB, NB>), dim3(one.nblocks * groups), dim3(64), 0, st, (const GemvJob*)nullptr,
                     (const int32_t*)nullptr, njobs, one);
}

template <int KA, int KB>
void launch_fast_t(const GemvJob* d_jobs, const int32_t* d_block_jobs, int njobs, const GemvJob& one, int blocks, hipStream_t st) {
  if (d_jobs == nullptr && njobs > 1) {
    // measured on 8B shapes: two samples per pass are fastest for B = 2, four per pass from B = 3 on
    if (njobs == 2) launch_group_t<KA, KB, 2>(njobs, one, st);
    else launch_group_t<KA, KB, 4>(njobs, one, st);
  } else {
    hipLaunchKernelGGL((gemv_kernel<KA, KB, 1>), dim3(blocks), dim3(64), 0, st, d_jobs, d_block_jobs, njobs, one);
  }
}

// row-per-lane arrangement: a batch runs in groups of two samples that share one pass over the planes
template <int KA, int KB>
void launch_lane_t(const GemvJob* d_jobs, const int32_t* d_block_jobs, int njobs, const GemvJob& one, int blocks, hipStream_t st) {
  if (d_jobs == nullptr && njobs > 1)
    hipLaunchKernelGGL((gemv_lane_kernel<KA, KB, 2>), dim3(one.nblocks * ((njobs + 1) / 2)), dim3(kLaneThreads), 0, st, d_jobs,
                       d_block_jobs, njobs, one);
  else
    hipLaunchKernelGGL((gemv_lane_kernel<KA, KB, 1>), dim3(d_jobs == nullptr ? one.nblocks : blocks), dim3(kLaneThreads), 0, st,
                       d_jobs, d_block_jobs, njobs, one);
}

// d_jobs != nullptr: a table of jobs, d_block_jobs[b] = index in it of the job workgroup b works for
void launch_fast(int mode, int ka, int kb, const GemvJob* d_jobs, const int32_t* d_block_jobs, int njobs, const GemvJob& one,
                 int blocks, hipStream_t st) {
#define DPLLM_CASE(A, B)                                                            \
  case (A) * 16 + (B):                                                              \
    if (mode == kLayoutRowLane) launch_lane_t<A, B>(d_jobs, d_block_jobs, njobs, one, blocks, st); \
    else launch_fast_t<A, B>(d_jobs, d_block_jobs, njobs, one, blocks, st);                       \
    break;
  switch (ka * 16 + kb) {
    DPLLM_CASE(3, 3) DPLLM_CASE(4, 4) DPLLM_CASE(5, 5) DPLLM_CASE(6, 6) DPLLM_CASE(7, 7) DPLLM_CASE(8, 8)
    DPLLM_CASE(3, 4) DPLLM_CASE(4, 5) DPLLM_CASE(5, 6) DPLLM_CASE(6, 7) DPLLM_CASE(7, 8)
    default: break;
  }
#undef DPLLM_CASE
}

GemvJob make_gemv_job(const Linear& lin, int ka, int kb, const int32_t* k_dev, const void* x, void* y) {
  GemvJob j;
  j.arena = lin.arena;
  j.x = (const uint16_t*)x;
  j.y = (uint16_t*)y;
  j.k_dev = k_dev;
  j.plane_stride_u4 = (uint32_t)(lin.L.plane_bytes / 16);
  j.lut_off_a = (uint32_t)lin.L.lut_offset[ka];
  j.lut_off_b = (uint32_t)lin.L.lut_offset[kb];
  j.ka = ka; j.kb = kb;
  j.out = lin.L.out; j.ncw = lin.L.ncw; j.nrq = lin.L.nrq; j.ncc = lin.L.ncc;
  j.nblocks = lin.L.nrq;
  j.block_start = 0;
  j.nsamples = 1;
  j.nsplit = 1;
  j.ws = nullptr;
  j.cnt = nullptr;
  return j;
}

// row quads one wavefront streams (workgroup b of a job takes row quads b, b + nblocks, ...): enough
// wavefronts to fill the chip several times over, long enough runs to amortise the pipeline fill
int pick_rq_per_block(long total_rq) {
  long r = total_rq / 8192;
  return (int)std::min<long>(8, std::max<long>(1, r));
}

// Row-per-lane arrangement: blocks of 64 rows one workgroup (eight wavefronts) streams.  A workgroup should
// run for the better part of a hundred microseconds (about 1 MiB of planes): shorter ones pay their start-up
// (job record, tables, first loads: a few microseconds of an otherwise idle slot) too often, longer ones leave
// the chip half empty at the end of the launch (measured on the 7B step: 0.25 MiB 496 us, 0.375 MiB 480,
// 0.75 MiB 471, 1 MiB 468, 2 MiB 477, 4 MiB 546); and a launch wants at least a few workgroups per compute unit.
constexpr long kLaneGroupBytes = 1048576;
int pick_blocks_per_group(const LinearLayout& L, int k, long total_blocks, long group_bytes = kLaneGroupBytes) {
  const long bytes_per_block = 64L * L.in * k / 8;
  long r = std::min<long>(16, std::max<long>(1, group_bytes / std::max<long>(1, bytes_per_block)));
  while (r > 1 && total_blocks / r < 1024) --r;
  return (int)r;
}

// Row-per-lane arrangement, launches with fewer workgroups than compute units (a workgroup is tied to 64 rows):
// the workgroups that share a block of rows.  Measured on 4096 .. 28672 rows x 4096 .. 14336 columns: splitting
// pays only below about one workgroup per compute unit (64 blocks of rows: 23 -> 12 us at 14336 columns) and costs
// above it (172 blocks: 9 -> 12 us), since every split builds the tables again and runs fewer tiles per wavefront.
// workgroups = those of the whole launch before splitting; rows = blocks of rows x samples per pass x groups of
// the job; pool = what is left of the partial-sum pool.
int pick_lane_split(const LinearLayout& L, long workgroups, long rows, long pool) {
  long s = std::min<long>(8, 320 / std::max<long>(1, workgroups));
  s = std::min<long>(s, L.ncc / kLaneWaves);   // at least one tile per wavefront
  while (s > 1 && rows * s > pool) --s;
  return (int)std::max<long>(1, s);
}

template <int B>
void launch_plain_t(const GemvArgs& a, hipStream_t st) {
  hipLaunchKernelGGL(gemv_plain_kernel<B>, dim3((a.nrq + 3) / 4), dim3(256), 0, st, a);
}

int launch_plain(dpllm_model* m, const Linear& lin, int ka, int kb, const int32_t* k_dev, const void* x, void* y,
                 int B, hipStream_t st) {
  GemvArgs a;
  a.planes = (const uint32_t*)lin.arena;
  a.plane_stride_u32 = lin.L.plane_bytes / 4;
  a.ka = ka; a.kb = kb;
  a.lut_a = lin.lut(ka);
  a.lut_b = k_dev ? lin.lut(kb) : nullptr;
  a.k_dev = k_dev;
  a.x = (const uint16_t*)x;
  a.y = (uint16_t*)y;
  a.out = lin.L.out; a.in = lin.L.in; a.ncw = lin.L.ncw; a.nrq = (lin.L.out + 3) / 4;
  a.ncc = lin.L.ncc; a.row_lane = lin.L.mode == kLayoutRowLane;
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

int launch_gemv(dpllm_model* m, const Linear& lin, int ka, int kb, const int32_t* k_dev, const void* x, void* y,
                int B, hipStream_t st) {
  if (!has_fast_kernel(ka, kb)) return launch_plain(m, lin, ka, kb, k_dev, x, y, B, st);
  GemvJob j = make_gemv_job(lin, ka, kb, k_dev, x, y);
  const int rpb = lin.L.mode == kLayoutRowLane ? pick_blocks_per_group(lin.L, kb, lin.L.nrq) : pick_rq_per_block(lin.L.nrq);
  j.nblocks = (lin.L.nrq + rpb - 1) / rpb;
  if (lin.L.mode == kLayoutRowLane) {
    const long groups = B > 1 ? (B + 1) / 2 : 1, per_pass = B > 1 ? 2 : 1;
    j.nsplit = pick_lane_split(lin.L, j.nblocks * groups, (long)lin.L.nrq * per_pass * groups, kLanePoolRows);
    j.nblocks *= j.nsplit;
    j.ws = m->d_lane_ws;
    j.cnt = m->d_lane_cnt;
  }
  launch_fast(lin.L.mode, ka, kb, nullptr, nullptr, B, j, j.nblocks * B, st);
  HIP_TRY(m, hipGetLastError());
  return DPLLM_OK;
}

// ---- decode-step planning ------------------------------------------------------------------------------------
bool overlap(const void* a, size_t an, const void* b, size_t bn) {
  uintptr_t a0 = (uintptr_t)a, b0 = (uintptr_t)b;
  return a0 < b0 + bn && b0 < a0 + an;
}

int build_plan(dpllm_model* m, const void* const* xs, void* const* ys, int32_t* k_dev, float* e_dev,
               hipStream_t st) {
  const int n = (int)m->linears.size();
  StepPlan& P = m->plan;
  P.valid = false;
  P.xs.assign(xs, xs + n);
  P.ys.assign(ys, ys + n);
  P.k_dev = k_dev;
  P.e_dev = e_dev;
  P.phases.clear();
  P.gemv_jobs.clear();
  P.gemv_ids.clear();
  if (!m->d_sel_jobs) {
    HIP_TRY(m, hipMalloc((void**)&m->d_sel_jobs, sizeof(SelJob) * n));
    HIP_TRY(m, hipMalloc((void**)&m->d_gemv_jobs, sizeof(GemvJob) * n));
    HIP_TRY(m, hipMalloc((void**)&m->d_sel_tickets, sizeof(uint32_t) * n));
    HIP_TRY(m, hipMemset(m->d_sel_tickets, 0, sizeof(uint32_t) * n));
  }
  std::vector<SelJob> sel_jobs;
  std::vector<SelPart> sel_parts;
  std::vector<int32_t> block_jobs;
  std::vector<size_t> ws_offset;
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
  for (size_t pi = 0; pi < bounds.size(); ++pi) {
    const int id = bounds[pi].first, end = bounds[pi].second;
    Phase ph;
    ph.sel_first = (int)sel_jobs.size();
    ph.sel_count = (int)sel_of_phase[pi].size();
    ph.part_first = (int)sel_parts.size();
    long launch_rowgroups = 0;
    for (int j : sel_of_phase[pi]) {
      const Selector& s = m->linears[j].sel[m->linears[j].active];
      launch_rowgroups += sel_rowgroups_of(s.kind, s.r);
    }
    for (size_t local = 0; local < sel_of_phase[pi].size(); ++local) {
      const int j = sel_of_phase[pi][local];
      const Linear& lin = m->linears[j];
      const Selector& s = lin.sel[lin.active];
      SelJob sj = make_sel_job(lin, s, lin.sel_input ? lin.sel_input : xs[j], e_dev + j, k_dev + j, launch_rowgroups);
      for (int part = 0; part < sj.nparts; ++part) sel_parts.push_back(SelPart{(int)local, part});
      ws_offset.push_back(ws_slots);
      ws_slots += (size_t)sel_slots_of(s.kind, s.r, sj.nchunks);
      sel_jobs.push_back(sj);
    }
    ph.part_count = (int)sel_parts.size() - ph.part_first;
    // GEMV jobs of the phase, grouped by kernel instance (bitwidth pair, arrangement) in order of first appearance
    struct Cls { int ka, kb, mode; bool operator==(const Cls& o) const { return ka == o.ka && kb == o.kb && mode == o.mode; } };
    auto cls_of = [&](int j) {
      const Linear& lj = m->linears[j];
      const Selector& s = lj.sel[lj.active];
      return has_fast_kernel(s.l, s.h) ? Cls{s.l, s.h, lj.L.mode} : Cls{0, 0, 0};
    };
    std::vector<Cls> classes;
    for (int j = id; j < end; ++j) {
      Cls c = cls_of(j);
      if (std::find(classes.begin(), classes.end(), c) == classes.end()) classes.push_back(c);
    }
    for (const Cls& c : classes) {
      GemvLaunch gl;
      gl.ka = c.ka; gl.kb = c.kb; gl.mode = c.mode;
      gl.first = (int)P.gemv_jobs.size();
      gl.block_first = (int)block_jobs.size();
      long total_rq = 0;
      for (int j = id; j < end; ++j)
        if (cls_of(j) == c) total_rq += m->linears[j].L.nrq;
      const int rpb_quad = pick_rq_per_block(total_rq);
      long lane_groups = 0;   // workgroups of the launch in the row-per-lane arrangement, before any split
      if (c.mode == kLayoutRowLane)
        for (int j = id; j < end; ++j)
          if (cls_of(j) == c) {
            const LinearLayout& L = m->linears[j].L;
            const int rpb = pick_blocks_per_group(L, c.kb, total_rq);
            lane_groups += (L.nrq + rpb - 1) / rpb;
          }
      std::vector<long> bytes_after(end - id, 0);   // plane bytes of the launch that follow linear j
      {
        long acc = 0;
        for (int j = end - 1; j >= id; --j) {
          if (!(cls_of(j) == c)) continue;
          bytes_after[j - id] = acc;
          const LinearLayout& L = m->linears[j].L;
          acc += (long)L.nrq * 64 * L.in * (c.ka + c.kb) / 16;
        }
      }
      // Large launches: the linears dispatched last (one round of workgroups: two on each of 256 compute units)
      // get workgroups of half the usual work, so that the chip drains in less time at the end of the launch
      // (measured on the 7B step: 0.5 - 0.8 % of the launch; quarters and eighths did not add to that).
      const bool taper = c.mode == kLayoutRowLane && lane_groups >= 2048;
      long pool_used = 0;
      int blocks = 0;
      for (int j = id; j < end; ++j) {
        if (!(cls_of(j) == c)) continue;
        const Linear& lin = m->linears[j];
        const Selector& s = lin.sel[lin.active];
        GemvJob gj = make_gemv_job(lin, s.l, s.h, s.l == s.h ? nullptr : k_dev + j, xs[j], ys[j]);
        long group_bytes = kLaneGroupBytes;
        if (taper && bytes_after[j - id] < 512 * kLaneGroupBytes) group_bytes /= 2;
        const int rpb = c.mode == kLayoutRowLane ? pick_blocks_per_group(lin.L, s.h, total_rq, group_bytes) : rpb_quad;
        gj.nblocks = (lin.L.nrq + rpb - 1) / rpb;
        if (c.mode == kLayoutRowLane) {
          gj.nsplit = pick_lane_split(lin.L, lane_groups, lin.L.nrq, kLanePoolRows - pool_used);
          gj.nblocks *= gj.nsplit;
          gj.ws = m->d_lane_ws + pool_used * 64;
          gj.cnt = m->d_lane_cnt + pool_used;
          pool_used += (long)lin.L.nrq * gj.nsplit;
        }
        gj.block_start = blocks;
        blocks += gj.nblocks;
        block_jobs.insert(block_jobs.end(), gj.nblocks, (int32_t)(P.gemv_jobs.size() - gl.first));
        P.gemv_jobs.push_back(gj);
        P.gemv_ids.push_back(j);
      }
      gl.count = (int)P.gemv_jobs.size() - gl.first;
      gl.blocks = blocks;
      ph.gemv.push_back(gl);
    }
    P.phases.push_back(ph);
  }
  // The tables may still be read by a step enqueued earlier: drain the stream before replacing them.
  HIP_TRY(m, hipStreamSynchronize(st));
  if (sel_parts.size() > m->sel_parts_cap) {
    if (m->d_sel_parts) (void)hipFree(m->d_sel_parts);
    m->d_sel_parts = nullptr; m->sel_parts_cap = 0;
    HIP_TRY(m, hipMalloc((void**)&m->d_sel_parts, sizeof(SelPart) * sel_parts.size()));
    m->sel_parts_cap = sel_parts.size();
  }
  if (block_jobs.size() > m->block_jobs_cap) {
    if (m->d_block_jobs) (void)hipFree(m->d_block_jobs);
    m->d_block_jobs = nullptr; m->block_jobs_cap = 0;
    HIP_TRY(m, hipMalloc((void**)&m->d_block_jobs, sizeof(int32_t) * block_jobs.size()));
    m->block_jobs_cap = block_jobs.size();
  }
  if (!block_jobs.empty())
    HIP_TRY(m, hipMemcpy(m->d_block_jobs, block_jobs.data(), sizeof(int32_t) * block_jobs.size(), hipMemcpyHostToDevice));
  if (ws_slots > m->sel_ws_cap) {
    if (m->d_sel_ws) (void)hipFree(m->d_sel_ws);
    m->d_sel_ws = nullptr; m->sel_ws_cap = 0;
    HIP_TRY(m, hipMalloc((void**)&m->d_sel_ws, sizeof(double) * ws_slots));
    m->sel_ws_cap = ws_slots;
  }
  for (size_t i = 0; i < sel_jobs.size(); ++i) {
    sel_jobs[i].ws = m->d_sel_ws + ws_offset[i];
    sel_jobs[i].ticket = m->d_sel_tickets + i;
  }
  if (!sel_parts.empty())
    HIP_TRY(m, hipMemcpy(m->d_sel_parts, sel_parts.data(), sizeof(SelPart) * sel_parts.size(), hipMemcpyHostToDevice));
  HIP_TRY(m, hipMemcpy(m->d_sel_jobs, sel_jobs.data(), sizeof(SelJob) * sel_jobs.size(), hipMemcpyHostToDevice));
  HIP_TRY(m, hipMemcpy(m->d_gemv_jobs, P.gemv_jobs.data(), sizeof(GemvJob) * P.gemv_jobs.size(),
                       hipMemcpyHostToDevice));
  P.version = m->version;
  P.valid = true;
  return DPLLM_OK;
}

void free_device(dpllm_model* m) {
  if (m->d_sel_jobs) (void)hipFree(m->d_sel_jobs);
  if (m->d_sel_parts) (void)hipFree(m->d_sel_parts);
  if (m->d_sel_ws) (void)hipFree(m->d_sel_ws);
  if (m->d_sel_ws_one) (void)hipFree(m->d_sel_ws_one);
  if (m->d_sel_tickets) (void)hipFree(m->d_sel_tickets);
  if (m->d_gemv_jobs) (void)hipFree(m->d_gemv_jobs);
  if (m->d_block_jobs) (void)hipFree(m->d_block_jobs);
  if (m->d_lane_ws) (void)hipFree(m->d_lane_ws);
  if (m->d_lane_cnt) (void)hipFree(m->d_lane_cnt);
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
    free_device(m);
    delete m;
    return DPLLM_EHIP;
  }
  if (hipMalloc((void**)&m->d_lane_ws, sizeof(float) * 64 * kLanePoolRows) != hipSuccess ||
      hipMalloc((void**)&m->d_lane_cnt, sizeof(uint32_t) * kLanePoolRows) != hipSuccess ||
      hipMemset(m->d_lane_cnt, 0, sizeof(uint32_t) * kLanePoolRows) != hipSuccess ||
      hipDeviceSynchronize() != hipSuccess) {
    (void)hipGetLastError();
    free_device(m);
    delete m;
    return DPLLM_EHIP;
  }
  *out = m;
  return DPLLM_OK;
}

void dpllm_model_destroy(dpllm_model* m) {
  if (!m) return;
  free_device(m);
  delete m;
}

const char* dpllm_last_error(const dpllm_model* m) { return m ? m->err.c_str() : "null model"; }

int dpllm_linear_device_bytes(int out, int in, int p, int kmin, size_t* bytes) {
  if (!bytes) return DPLLM_EINVAL;
  int rc = check_shape(out, in, p, kmin);
  if (rc != DPLLM_OK) return rc;
  // enough for either arrangement of the planes
  *bytes = std::max(LinearLayout::make(out, in, p, kmin, kLayoutRowQuad).total_bytes,
                    LinearLayout::make(out, in, p, kmin, kLayoutRowLane).total_bytes);
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
  LinearLayout L = LinearLayout::make(out, in, p, kmin, m->layout);
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
    const int row_lane = L.mode == kLayoutRowLane;
    size_t n = (row_lane ? (size_t)L.nrq * L.ncc * 64 : (size_t)L.nrq * L.ncw) * p;
    hipLaunchKernelGGL(retile_planes_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, d_planes,
                       (uint4*)dev_arena, p, out, L.ncw, L.ncc, L.nrq, row_lane, L.plane_bytes / 16);
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
  m->version++;
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
  m->version++;
  return DPLLM_OK;
}

int dpllm_set_active_pair(dpllm_model* m, int id, int l, int h) {
  int rc = DPLLM_OK;
  Linear* lin = get_linear(m, id, &rc);
  if (!lin) return rc;
  int slot = lin->find_pair(l, h);
  if (slot < 0) return fail(m, DPLLM_ESTATE, "pair (%d,%d) not set on linear %d", l, h, id);
  lin->active = slot;
  m->version++;
  return DPLLM_OK;
}

int dpllm_model_set_layout(dpllm_model* m, int layout) {
  if (!m) return DPLLM_EINVAL;
  if (layout != DPLLM_LAYOUT_ROWQUAD && layout != DPLLM_LAYOUT_ROWLANE) return fail(m, DPLLM_EINVAL, "unknown layout %d", layout);
  m->layout = layout == DPLLM_LAYOUT_ROWLANE ? kLayoutRowLane : kLayoutRowQuad;
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

int dpllm_estimate(dpllm_model* m, int id, int l, int h, const void* x_dev, float* e_dev, int32_t* k_dev,
                   void* stream) {
  int rc = DPLLM_OK;
  Linear* lin = get_linear(m, id, &rc);
  if (!lin) return rc;
  if (!x_dev || !e_dev || !k_dev) return fail(m, DPLLM_EINVAL, "null pointer");
  if ((uintptr_t)x_dev % 16) return fail(m, DPLLM_EINVAL, "x not 16-byte aligned");
  int slot = lin->find_pair(l, h);
  if (slot < 0) return fail(m, DPLLM_ESTATE, "pair (%d,%d) not set on linear %d", l, h, id);
  const Selector& sel = lin->sel[slot];
  SelJob j = make_sel_job(*lin, sel, x_dev, e_dev, k_dev, sel_rowgroups_of(sel.kind, sel.r));
  if (!m->d_sel_ws_one) {
    HIP_TRY(m, hipMalloc((void**)&m->d_sel_ws_one, sizeof(double) * (kSelOneSlots + 1)));
    HIP_TRY(m, hipMemset(m->d_sel_ws_one + kSelOneSlots, 0, sizeof(double)));
    HIP_TRY(m, hipDeviceSynchronize());
  }
  j.ws = m->d_sel_ws_one;
  j.ticket = reinterpret_cast<uint32_t*>(m->d_sel_ws_one + kSelOneSlots);
  hipLaunchKernelGGL(selector_part_kernel, dim3(j.nparts), dim3(kSelPartThreads), 0, (hipStream_t)stream,
                     (const SelJob*)nullptr, (const SelPart*)nullptr, j);
  HIP_TRY(m, hipGetLastError());
  return DPLLM_OK;
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
  return launch_gemv(m, *lin, s.l, s.h, s.l == s.h ? nullptr : k_dev, x_dev, y_dev, B, (hipStream_t)stream);
}

int dpllm_decode_step_parts(dpllm_model* m, const void* const* xs, void* const* ys, int32_t* k_dev, float* e_dev,
                            int parts, void* stream) {
  if (!m) return DPLLM_EINVAL;
  if (parts < 1 || parts > (DPLLM_STEP_SELECT | DPLLM_STEP_GEMV)) return fail(m, DPLLM_EINVAL, "bad parts %d", parts);
  if (!xs || !ys || !k_dev || !e_dev) return fail(m, DPLLM_EINVAL, "null pointer");
  const int n = (int)m->linears.size();
  StepPlan& P = m->plan;
  bool reuse = P.valid && P.version == m->version && P.k_dev == k_dev && P.e_dev == e_dev &&
               std::equal(xs, xs + n, P.xs.begin()) && std::equal(ys, ys + n, P.ys.begin());
  if (!reuse) {
    for (int id = 0; id < n; ++id) {
      const Linear& lin = m->linears[id];
      if (!lin.loaded) return fail(m, DPLLM_ESTATE, "linear %d is not loaded", id);
      if (lin.active < 0) return fail(m, DPLLM_ESTATE, "linear %d has no selector", id);
      if (!xs[id] || !ys[id]) return fail(m, DPLLM_EINVAL, "null x or y for linear %d", id);
      if ((uintptr_t)xs[id] % 16) return fail(m, DPLLM_EINVAL, "x of linear %d not 16-byte aligned", id);
    }
    int rc = build_plan(m, xs, ys, k_dev, e_dev, (hipStream_t)stream);
    if (rc != DPLLM_OK) return rc;
  }
  hipStream_t st = (hipStream_t)stream;
  SelJob none{};
  GemvJob gnone{};
  for (const Phase& ph : P.phases) {
    if (parts & DPLLM_STEP_SELECT) {
      const SelJob* jobs = m->d_sel_jobs + ph.sel_first;
      if (ph.part_count > 0)
        hipLaunchKernelGGL(selector_part_kernel, dim3(ph.part_count), dim3(kSelPartThreads), 0, st, jobs,
                           (const SelPart*)(m->d_sel_parts + ph.part_first), none);
    }
    if (!(parts & DPLLM_STEP_GEMV)) continue;
    for (const GemvLaunch& gl : ph.gemv) {
      if (gl.ka != 0) {
        launch_fast(gl.mode, gl.ka, gl.kb, m->d_gemv_jobs + gl.first, m->d_block_jobs + gl.block_first, gl.count, gnone,
                    gl.blocks, st);
      } else {
        for (int i = gl.first; i < gl.first + gl.count; ++i) {
          const GemvJob& j = P.gemv_jobs[i];
          int rc = launch_plain(m, m->linears[P.gemv_ids[i]], j.ka, j.kb, j.k_dev, j.x, j.y, 1, st);
          if (rc != DPLLM_OK) return rc;
        }
      }
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
                     (const uint32_t*)lin->arena, lin->L.plane_bytes / 4, lin->L.p, k, lin->L.out, lin->L.ncw, lin->L.ncc,
                     (int)(lin->L.mode == kLayoutRowLane), idx_dev);
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
