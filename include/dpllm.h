/*
 * dpllm.h — C boundary of the MI355X (gfx950) DP-LLM decode hot path.
 *
 * The library serves one multi-scale ("any-precision") weight-only-quantised model:
 * every linear keeps a parent p-bit code per weight, stored as p bitplanes, and a
 * per-row table of 2^k fp16 centroids for every k <= p, so that the k-bit model is
 * read from the top k planes only (paper Sec. 2.2: variants of 3..n bits overlaid in
 * the memory of one n-bit model).  Each linear carries a precision selector (paper
 * Sec. 3 and Sec. 5.1) that estimates the relative error ||(W_h - W_l) x|| from the
 * current input and picks h when the estimate exceeds the layer's threshold T, else l.
 *
 * Conventions
 *   - Every function returns DPLLM_OK (0) or a negative DPLLM_E* code; nothing throws
 *     or aborts.  dpllm_last_error() gives the text of the last failure on a model.
 *   - "host" / "device" on a pointer says where the memory lives.  The caller owns all
 *     device memory: the weight arenas, G, x, y, k, e, and one workspace per model
 *     (partial results of the selectors and of column-split GEMV launches, arrival
 *     counters, job and parameter tables: a few MiB, see dpllm_workspace_bytes) that it
 *     hands over with dpllm_set_workspace.  Everything is borrowed until the model is
 *     destroyed (a linear's memory: until it is loaded again).  No call allocates device
 *     memory, except dpllm_load_linear from host pointers (a staging buffer it frees
 *     before it returns).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All work
 *     is enqueued on it; only dpllm_load_linear synchronises it.
 *   - One model may be driven from one stream at a time (the workspace is shared by
 *     the calls of a model; calls that overlap on one model race).  The calls that
 *     configure a model (load, set_selector, set_threshold, set_active_pair,
 *     set_target_entry, set_selector_input, set_workspace) take effect for the work
 *     enqueued after them and must not run while a step of the model is being captured
 *     into a graph; dpllm_set_target is the call for switching while steps are in flight.
 *   - fp16 values cross the boundary as IEEE binary16 bit patterns (uint16_t).
 *
 * Canonical host layout of a linear with `out` rows and `in` columns (in % 32 == 0):
 *   planes : uint32_t [p][out][in/32]; plane 0 = most significant bit of the p-bit
 *            code; column c is bit (c % 32) of word c / 32.
 *   luts   : luts[k - kmin] -> uint16_t [out][2^k] for k = kmin..p; the k-bit code of a
 *            weight is the top k bits of its p-bit code.
 * The library re-tiles the planes into a private, plane-separable device layout inside
 * the caller's arena; dpllm_debug_unpack returns canonical codes for checking it.
 */
#ifndef DPLLM_H
#define DPLLM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DPLLM_OK 0
#define DPLLM_EINVAL (-1) /* null pointer, bad id, bad flag, NaN threshold            */
#define DPLLM_ESHAPE (-2) /* in % 32 != 0, out < 1, batch outside [1, DPLLM_MAX_BATCH] */
#define DPLLM_ERANGE (-3) /* bitwidth outside [kmin, p] or p outside [1, 8]           */
#define DPLLM_ESTATE (-4) /* linear not loaded, selector not set, arena too small     */
#define DPLLM_EHIP (-5)   /* a HIP runtime call failed                                 */

#define DPLLM_MAX_BITS 8
#define DPLLM_MAX_BATCH 8
#define DPLLM_MAX_PAIRS 8   /* (l,h) candidate pairs kept per linear                    */
#define DPLLM_MAX_TARGETS 8 /* target precisions (sets of pairs and thresholds) resident */
#define DPLLM_MAX_RANK 1024 /* projection rank r                                        */

#define DPLLM_SEL_NONE 0   /* no estimator: always l                                     */
#define DPLLM_SEL_PROJ 1   /* random projection: e = ||G x||_2      (paper Sec. 5.1)    */
#define DPLLM_SEL_LINREG 2 /* linear regression: e = alpha ||x||_2 + beta (Sec. 5.1)    */

typedef struct dpllm_model dpllm_model; /* opaque host object */

/* Creates a model with room for n_linears linears (ids 0..n_linears-1), on the current
 * HIP device.  *out receives the handle.  Errors: EINVAL, EHIP. */
int dpllm_model_create(dpllm_model** out, int n_linears);

/* Frees the handle.  Caller-owned device memory (arenas, G, the workspace) is not
 * touched.  NULL is accepted. */
void dpllm_model_destroy(dpllm_model* m);

/* Text of the last error on m (owned by m, valid until the next failing call). */
const char* dpllm_last_error(const dpllm_model* m);

/* Bytes of device arena one linear needs (planes + tables, 256-byte aligned parts).
 * Errors: EINVAL (bytes NULL), ESHAPE, ERANGE. */
int dpllm_linear_device_bytes(int out, int in, int p, int kmin, size_t* bytes);

/* "Load a parent p-bit bitplane model with per-row LUTs for every k <= p" (Sec. 2.2).
 * Copies linear `id` from the canonical layout into dev_arena (device, caller-owned,
 * 256-byte aligned, >= dpllm_linear_device_bytes) in the private device layout.
 * src_on_device = 0: planes and every luts[i] are host pointers;
 * src_on_device = 1: they are device pointers (the array `luts` itself is always host).
 * Synchronises `stream` before returning.  Reloading an id replaces it and drops its
 * selectors.  Errors: EINVAL, ESHAPE, ERANGE, ESTATE (arena too small), EHIP. */
int dpllm_load_linear(dpllm_model* m, int id, int out, int in, int p, int kmin,
                      const uint32_t* planes, const uint16_t* const* luts, int src_on_device,
                      void* dev_arena, size_t arena_bytes, void* stream);

/* Bytes of workspace the model needs as it stands (linears loaded, pairs set): enough for every entry point and
 * every order of the linears' buffers.  Ask again after loading more linears or attaching pairs of higher rank.
 * Errors: EINVAL. */
int dpllm_workspace_bytes(const dpllm_model* m, size_t* bytes);

/* Hands the model its workspace: ws_dev (device, caller-owned, 256-byte aligned, >= dpllm_workspace_bytes), which
 * the model uses until it is destroyed or given another.  Enqueues the clearing of its counters on `stream`.
 * dpllm_estimate, dpllm_decode_step(_parts) and dpllm_set_target need a workspace; dpllm_gemv runs without one
 * (it then never splits the columns of a linear over several workgroups).
 * Errors: EINVAL, ESTATE (too small), EHIP. */
int dpllm_set_workspace(dpllm_model* m, void* ws_dev, size_t bytes, void* stream);

/* Attaches the precision selector of candidate pair (l, h), kmin <= l <= h <= p, to a
 * loaded linear and makes it the active pair (Sec. 3: two candidate precisions per
 * layer; Sec. 5.1: one G per pair).  kind = DPLLM_SEL_PROJ: G_dev is a device pointer
 * to fp16 [r][in] (row-major, borrowed), G = A (W_h - W_l) precomputed by the caller,
 * 1 <= r <= DPLLM_MAX_RANK.  kind = DPLLM_SEL_LINREG uses alpha, beta.  kind =
 * DPLLM_SEL_NONE needs l == h.  T may be +inf (always l) or -inf (always h), not NaN.
 * Setting an existing pair replaces it.  The pair becomes the linear's pair under target 0.
 * Errors: EINVAL, ERANGE, ESTATE. */
int dpllm_set_selector(dpllm_model* m, int id, int l, int h, int kind, const void* G_dev, int r,
                       float alpha, float beta, float T);

/* Replaces the threshold an existing pair has under target 0 and in dpllm_estimate.
 * Errors: EINVAL (NaN), ESTATE (pair not set). */
int dpllm_set_threshold(dpllm_model* m, int id, int l, int h, float T);

/* Chooses which of a linear's pairs is its pair under target 0.  Errors: ESTATE. */
int dpllm_set_active_pair(dpllm_model* m, int id, int l, int h);

/* Run-time adaptation (Sec. 2.1: the target precision changes from query to query; Algorithm 1: one threshold
 * list per target precision; Sec. 5.1: one G per candidate pair, all resident).  A model holds
 * DPLLM_MAX_TARGETS targets.  Target 0 is what dpllm_set_selector / dpllm_set_threshold / dpllm_set_active_pair
 * describe.  dpllm_set_target_entry says that under target t (1 <= t < DPLLM_MAX_TARGETS) linear id runs pair
 * (l, h), which must have been attached with dpllm_set_selector, with threshold T; a linear without an entry
 * for t runs as under target 0.  Errors: EINVAL, ESTATE (pair not set). */
int dpllm_set_target_entry(dpllm_model* m, int target, int id, int l, int h, float T);

/* Switches the whole model to `target` with one word written on the device, enqueued on `stream`: the steps
 * enqueued behind it (also replays of graphs captured earlier, and it can be captured itself) run every linear
 * under that target's pair and threshold.  No launch plan is rebuilt and nothing is synchronised.
 * Errors: EINVAL, ESTATE (no workspace), EHIP. */
int dpllm_set_target(dpllm_model* m, int target, void* stream);

/* Asynchronous estimation (Sec. 5.2): the selector of a layer fed by the residual stream may read the
 * previous residual vector instead of the layer's immediate input, which takes the estimate off the critical
 * path.  xsel_dev (device fp16 [in], 16-byte aligned, borrowed) replaces the input of linear id's selector in
 * dpllm_decode_step / dpllm_decode_step_parts; the GEMV still reads xs[id].  NULL restores the immediate
 * input.  The step keeps sequential semantics: a selector input written by an earlier linear of the step is
 * read after that linear has run, and when (earlier in the step) such a selector runs is the library's
 * choice.  Reloading the linear clears it.  Errors: EINVAL, ESTATE. */
int dpllm_set_selector_input(dpllm_model* m, int id, const void* xsel_dev);

/* "Estimate the relative error for (layer, x)" (Sec. 5.1) and select (Sec. 3):
 * e_dev[0] = estimate (fp32, rounded from the fp64 the decision is taken in),
 * k_dev[0] = h if estimate > T else l, for pair (l, h) of the linear and the threshold it has under target 0.
 * x_dev: device fp16 [in].  e_dev, k_dev: device.
 * Errors: EINVAL, ESTATE (pair not set, no workspace), EHIP. */
int dpllm_estimate(dpllm_model* m, int id, int l, int h, const void* x_dev, float* e_dev,
                   int32_t* k_dev, void* stream);

/* dpllm_estimate for callers that cannot allocate or hand over a workspace (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): same arguments, same result bit for bit, but the partial
 * products of the selector travel through a fixed array in the library's own device image (64 KiB per GPU, held
 * until the process ends) instead of the model's workspace.  It allocates nothing, needs no workspace, and
 * enqueues two kernels on `stream`.  Limit: projection rank r <= 256 (ERANGE beyond).  All calls on one GPU, from
 * any model or stream, share the array: calls that overlap in time on one GPU race, calls that follow one another
 * on one stream do not.  Errors: EINVAL, ERANGE, ESTATE (pair not set), EHIP. */
int dpllm_estimate_noalloc(dpllm_model* m, int id, int l, int h, const void* x_dev, float* e_dev,
                           int32_t* k_dev, void* stream);

/* "Run the GEMV at bitwidth k": y[b][o] = sum_c LUT_k[o][code_k(o,c)] * x[b][c], fp32
 * accumulation, fp16 result.  k >= 0: that bitwidth.  k < 0: the bitwidth is read on the
 * device from k_dev[0] (the hand-over from dpllm_estimate without a host round trip); a
 * value there that the linear does not serve (outside [kmin, p]) leaves y_dev untouched.
 * x_dev: device fp16 [B][in]; y_dev: device fp16 [B][out], not overlapping x_dev;
 * 1 <= B <= DPLLM_MAX_BATCH; one bitwidth serves the whole batch.
 * Errors: EINVAL, ESHAPE, ERANGE, ESTATE, EHIP. */
int dpllm_gemv(dpllm_model* m, int id, int k, const int32_t* k_dev, const void* x_dev, void* y_dev,
               int B, void* stream);

/* "Run a whole decode step under per-layer thresholds" (Sec. 3, every linear operation
 * of every Transformer block carries a selector): for id = 0..n_linears-1 in order,
 * estimate on xs[id] with the linear's pair and threshold under the active target, then
 * the GEMV at the selected bitwidth into ys[id], batch 1, all on `stream` with no host
 * synchronisation.  xs, ys: host arrays of n_linears device pointers (fp16 [in_id], fp16
 * [out_id]; xs[id] and ys[id] must not overlap).  k_dev, e_dev: device arrays of n_linears
 * entries receiving every linear's bitwidth and estimate.  Results equal those of running
 * the linears one after another: consecutive linears that do not touch each other's
 * inputs and outputs share launches, dependent ones are ordered on the stream.
 * The first call, and a call after the pointers, the linears or the shapes of their pairs
 * changed, rebuilds the launch plan and copies its tables into the workspace; a call after
 * thresholds, pairs in use or target entries changed copies the parameter table.  Both are
 * asynchronous copies on `stream` (nothing is synchronised, nothing allocated) but cannot
 * be captured into a graph: ESTATE then.  Every other call only enqueues kernels.
 * A graph that holds captured steps reads these tables when it is replayed: it follows later changes of
 * thresholds, pairs in use, target entries and the target (that is the point of keeping them on the device),
 * and it must not be replayed after a call that rebuilt the launch plan for other pointers or shapes.
 * Errors: EINVAL, ESTATE, ESHAPE, EHIP. */
int dpllm_decode_step(dpllm_model* m, const void* const* xs, void* const* ys, int32_t* k_dev,
                      float* e_dev, void* stream);

/* The two halves of dpllm_decode_step, for callers that schedule them apart (Sec. 5.2:
 * selectors fed by an earlier activation can run ahead of the GEMVs they steer) or time
 * them apart.  parts = DPLLM_STEP_SELECT: every selector writes k_dev / e_dev.  parts =
 * DPLLM_STEP_GEMV: every GEMV runs at the bitwidth k_dev already holds (l or h of the
 * linear's active pair).  Both bits = dpllm_decode_step.  Same arguments, plan and errors. */
#define DPLLM_STEP_SELECT 1
#define DPLLM_STEP_GEMV 2
int dpllm_decode_step_parts(dpllm_model* m, const void* const* xs, void* const* ys, int32_t* k_dev,
                            float* e_dev, int parts, void* stream);

/* Parity aid: writes the canonical k-bit codes of linear `id`, uint8 [out][in], read back
 * from the private device layout, to idx_dev (device).  Errors: EINVAL, ERANGE, ESTATE, EHIP. */
int dpllm_debug_unpack(dpllm_model* m, int id, int k, uint8_t* idx_dev, void* stream);

/* Parity aid (host only, touches no device): where the private device layout keeps the plane-`plane` bit of the
 * weight (row, col) of a linear of this shape: *byte_offset from the start of the arena (a multiple of 4: the
 * 32-bit word), *bit inside that word.  Errors: EINVAL, ESHAPE, ERANGE. */
int dpllm_debug_locate(int out, int in, int p, int kmin, int plane, int row, int col, size_t* byte_offset, int* bit);

/* Measurement aid: a plain 128-bit copy kernel, bytes % 16 == 0, both pointers device and 16-byte
 * aligned.  Its known traffic (bytes read + bytes written) scales the HBM byte counters that the
 * profiles report for the GEMV.  Errors: EINVAL, EHIP. */
int dpllm_debug_copy(void* dst_dev, const void* src_dev, size_t bytes, void* stream);

/* Measurement aid: a plain 128-bit non-temporal streaming read of `bytes` (bytes % 16 == 0, pointers device and
 * 16-byte aligned; sink_dev: 16 writable bytes, practically never written).  Its rate over >= 1 GiB is the
 * measured HBM read ceiling the GEMV's rate is reported against.  Errors: EINVAL, EHIP. */
int dpllm_debug_read(const void* src_dev, size_t bytes, void* sink_dev, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* DPLLM_H */
