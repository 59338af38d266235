"""Benchmark of the DP-LLM decode hot path on one MI355X.

A "step" is one whole decode step of a Llama-7B-shaped model (32 blocks x 7 linears, parent p = 8
bitplanes): for every linear the rank-64 selector estimates ||G x||, compares it with the layer's
threshold and hands the bitwidth (3 or 4) to the any-precision GEMV on the device.  Inputs are
synthetic (see synth.py) and resident in HBM before the timed region.

Prints ONE JSON line: whole-step algorithmic GB/s (`value`), microseconds per decode step, the
realised average bitwidth, the roofline of the dominant kernel (the GEMV launch), a per-k sweep with
the bitwidth pinned by +/-inf-style fixed selectors (the paper's latency protocol), and the CPU oracle
timed on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0     # MI355X published HBM3E bandwidth
RANK = 64                  # projection rank used for every linear (paper Sec. 5.1)


def gemv_bytes(out, in_, k, B=1):
    """Algorithmic bytes of one any-precision GEMV: top-k planes + the k-bit table + x + y."""
    return out * in_ * k / 8 + out * (1 << k) * 2 + B * in_ * 2 + B * out * 2


def selector_bytes(in_, r=RANK):
    return r * in_ * 2 + in_ * 2 + 8


def build_model(dp, synth, torch, shapes, n_blocks, p, l, h, n_x, seed=1234, keep_blocks=(0,), log=None,
                quantile=None, layout=None):
    """Loads n_blocks x len(shapes) linears generated on the GPU and attaches one projection selector each.
    Returns (model, meta) where meta carries shapes, thresholds, G, the activation sets and host copies of
    the linears of `keep_blocks` for the oracle.  Thresholds: tau ~ U[0.05, 0.3] times the median of
    ||W_h x|| (default), or the `quantile` of the calibration estimates."""
    import numpy as np
    n = n_blocks * len(shapes)
    model = dp.Model(n, layout=layout)
    ins = sorted({in_ for _, _, in_ in shapes})
    xs_by_in = {in_: synth.make_x(in_, n_x, seed=seed + in_, device="cuda") for in_ in ins}
    rng = np.random.default_rng(seed)
    taus = rng.uniform(0.05, 0.3, size=n)
    meta = {"shapes": [], "T": [], "G": [], "xs_by_in": xs_by_in, "host": {}, "est": []}
    t0 = time.time()
    for b in range(n_blocks):
        for j, (name, out, in_) in enumerate(shapes):
            i = b * len(shapes) + j
            lin = synth.make_linear(out, in_, p, 3, seed=seed + 7919 * i, device="cuda", keep_codes=True)
            model.dpllm_load_linear(i, lin["planes"], lin["luts"], 3)
            G = synth.make_G(lin, l, h, RANK, seed=seed + 104729 * i + 1)
            est = synth.estimates_fp64(G, xs_by_in[in_])
            if quantile is None:
                T = synth.thresholds_from_tau(lin, h, xs_by_in[in_], float(taus[i]))
            else:   # Phase-3 style: the rho-quantile of the calibration estimates
                T = synth.quantile_threshold(est, quantile)
            T = synth.nudge_threshold(T, est, band=1e-6)
            model.dpllm_set_selector(i, l, h, dp.DPLLM_SEL_PROJ, G=G, T=T)
            meta["shapes"].append((out, in_))
            meta["T"].append(T)
            meta["G"].append(G)
            meta["est"].append(est)
            if b in keep_blocks:
                meta["host"][i] = {"planes": synth.planes_np(lin["planes"]),
                                   "luts": {k: synth.lut_np(v) for k, v in lin["luts"].items()},
                                   "selector": {"l": l, "h": h, "kind": 1, "G": synth.lut_np(G), "T": T}}
            del lin
        if log and (b % 8 == 7 or b == n_blocks - 1):
            log("built block %d/%d (%.0f s)" % (b + 1, n_blocks, time.time() - t0))
    return model, meta


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--model", choices=["7b", "8b", "70b"], default="7b",
                    help="shape of the linears: Llama-7B (the headline workload), Llama-3-8B, or 70B with p = 6 planes")
    ap.add_argument("--blocks", type=int, default=None, help="Transformer blocks (default: 32 for 7b and 8b, 80 for 70b)")
    ap.add_argument("--no-sweep", action="store_true", help="skip the per-k sweep")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle timing")
    ap.add_argument("--no-graph", action="store_true", help="time eager launches only (no HIP graph replay)")
    ap.add_argument("--chained", action="store_true",
                    help="also time the step with the buffers chained as in a Transformer block (many small launches "
                         "of the same kernels: kept out of the default run so that its kernel trace stays one workload)")
    ap.add_argument("--layout", choices=["rowlane", "rowquad"], default="rowlane",
                    help="arrangement of the planes: one row per lane (default; fastest for a whole step) or four rows per lane")
    ap.add_argument("--copy-yardstick", action="store_true",
                    help="also run a plain 1 GiB copy kernel (for scaling hardware byte counters under rocprofv3 --pmc)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)")

    import numpy as np
    import torch

    import synth
    import paper_2508_06041_amd as dp

    def log(msg):
        print("[bench] " + msg, file=sys.stderr, flush=True)

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.copy_yardstick:
        src = torch.ones(1 << 28, dtype=torch.int32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dp.dpllm_debug_copy(dst, src)
        torch.cuda.synchronize()
        del src, dst
    shapes, p = {"7b": (synth.LLAMA_7B, 8), "8b": (synth.LLAMA3_8B, 8), "70b": (synth.LLAMA_70B, 6)}[args.model]
    l, h, n_x = 3, 4, 256
    if args.blocks is None:
        args.blocks = 80 if args.model == "70b" else 32
    if args.model == "70b":
        n_x = 32   # the calibration pass over the activations is what takes time at this size
    layout = dp.DPLLM_LAYOUT_ROWLANE if args.layout == "rowlane" else dp.DPLLM_LAYOUT_ROWQUAD
    model, meta = build_model(dp, synth, torch, shapes, args.blocks, p, l, h, n_x, log=log, layout=layout)
    gemv_name = "gemv_lane_kernel<3,4,1>" if args.layout == "rowlane" else "gemv_kernel<3,4,1>"
    n = len(meta["shapes"])
    ins = sorted(meta["xs_by_in"])
    # the activation vectors of a step sit in one buffer (one copy per step); 128-byte aligned slices
    offs, tot = {}, 0
    for in_ in ins:
        offs[in_] = tot
        tot += (in_ + 63) // 64 * 64
    xall = torch.zeros(tot, dtype=torch.float16, device="cuda")
    xbuf = {in_: xall[offs[in_]:offs[in_] + in_] for in_ in ins}
    xsteps = torch.zeros((n_x, tot), dtype=torch.float16, device="cuda")
    for in_ in ins:
        xsteps[:, offs[in_]:offs[in_] + in_] = meta["xs_by_in"][in_][:n_x]
    xs = [xbuf[in_] for _, in_ in meta["shapes"]]
    ys = [torch.empty(out, dtype=torch.float16, device="cuda") for out, _ in meta["shapes"]]
    x_tensors, y_tensors = xs, ys                     # keep the tensors alive; the calls take pointer arrays
    xs, ys = model.pointers(x_tensors), model.pointers(y_tensors)
    k_dev = torch.zeros(n, dtype=torch.int32, device="cuda")
    e_dev = torch.zeros(n, dtype=torch.float32, device="cuda")

    def set_inputs(t):
        xall.copy_(xsteps[t % n_x])

    def timed(fn, steps, warmup):
        for t in range(warmup):
            fn(t)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for t in range(steps):
            fn(warmup + t)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / steps   # ms per call

    # ---- the decode step under thresholds (selectors + GEMVs) ------------------------------------------
    ks_hist = []

    def full_step(t):
        set_inputs(t)
        model.dpllm_decode_step(xs, ys, k_dev, e_dev)

    ms_step_eager = timed(full_step, args.steps, args.warmup)
    ms_step, launch_mode = ms_step_eager, "eager launches"
    if not args.no_graph:
        # the same K steps recorded once in a HIP graph (per step: one input copy + two kernels) and replayed:
        # what a serving loop does to shed launch gaps.  The replay's final state is checked against eager.
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for t in range(args.steps):
                full_step(args.warmup + t)
        graph.replay()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        graph.replay()
        e1.record()
        torch.cuda.synchronize()
        ms_graph = e0.elapsed_time(e1) / args.steps
        k_graph, y_graph = k_dev.clone(), y_tensors[-1].clone()
        full_step(args.warmup + args.steps - 1)
        torch.cuda.synchronize()
        if torch.equal(k_graph, k_dev) and torch.equal(y_graph, y_tensors[-1]):
            ms_step, launch_mode = ms_graph, "one HIP graph of the K steps"
        else:
            log("graph replay differs from eager: reporting the eager time")
    # realised bitwidths over the activation set (untimed pass)
    params = np.array([o * i for o, i in meta["shapes"]], dtype=np.float64)
    step_bytes = []
    for t in range(min(n_x, 64)):
        set_inputs(t)
        model.dpllm_decode_step(xs, ys, k_dev, e_dev)
        ks = k_dev.cpu().numpy()
        ks_hist.append(float((ks * params).sum() / params.sum()))
        step_bytes.append(sum(gemv_bytes(o, i, int(k)) + selector_bytes(i) for (o, i), k in zip(meta["shapes"], ks)))
    eff_bits = float(np.mean(ks_hist))
    bytes_step = float(np.mean(step_bytes))

    # ---- the two kernels apart: HIP events on the launch stream around each half ------------------------
    set_inputs(0)
    model.dpllm_decode_step(xs, ys, k_dev, e_dev)
    ks0 = k_dev.cpu().numpy()
    gemv_bytes0 = sum(gemv_bytes(o, i, int(k)) for (o, i), k in zip(meta["shapes"], ks0))
    ms_gemv = timed(lambda t: model.dpllm_decode_step_parts(xs, ys, k_dev, e_dev, dp.DPLLM_STEP_GEMV), args.steps, 5)
    ms_sel = timed(lambda t: model.dpllm_decode_step_parts(xs, ys, k_dev, e_dev, dp.DPLLM_STEP_SELECT), args.steps, 5)
    sel_bytes = sum(selector_bytes(i) for _, i in meta["shapes"])
    roof_achieved = gemv_bytes0 / (ms_gemv * 1e-3) / 1e9
    # HBM traffic per GEMV launch from the committed counter summary (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
    # scaled by a plain copy kernel); it belongs to the default 32-block workload only
    traffic = None
    counters = os.path.join(ROOT, "profiles", "decode_step_7b_hbm_counters.txt")
    if args.model == "7b" and args.blocks == 32 and os.path.exists(counters):
        for line in open(counters):
            if line.startswith("gemv_traffic_bytes_per_launch"):
                traffic = float(line.split()[1])

    # ---- measured ceiling: a plain non-temporal streaming read of 2 GiB on the same box ----------------------
    rbuf = torch.ones(1 << 29, dtype=torch.int32, device="cuda")
    rsink = torch.zeros(4, dtype=torch.int32, device="cuda")
    ms_read = timed(lambda t: dp.dpllm_debug_read(rbuf, rsink), 100, 100)
    read_ceiling = rbuf.numel() * 4 / (ms_read * 1e-3) / 1e9
    del rbuf

    # ---- per-k sweep, bitwidth pinned for every layer (the paper fixes it with +/-inf thresholds) -------
    per_k = {}
    if not args.no_sweep:
        for k in range(3, p + 1):
            for i in range(n):
                model.dpllm_set_selector(i, k, k, dp.DPLLM_SEL_NONE)
            ms_k = timed(lambda t: model.dpllm_decode_step_parts(xs, ys, k_dev, e_dev, dp.DPLLM_STEP_GEMV),
                         max(10, args.steps // 4), 3)
            bk = sum(gemv_bytes(o, i, k) for o, i in meta["shapes"])
            per_k[str(k)] = {"us_per_step": round(ms_k * 1e3, 1), "GBps": round(bk / (ms_k * 1e-3) / 1e9, 1),
                             "frac_of_peak": round(bk / (ms_k * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)}
            log("k=%d: %.1f us/step, %.0f GB/s" % (k, ms_k * 1e3, per_k[str(k)]["GBps"]))
        for i in range(n):
            model.dpllm_set_active_pair(i, l, h)

    # ---- the same linears with their buffers chained the way a Transformer block chains them ---------------------
    # (q, k, v read the residual; o reads v's output; gate and up read o's output; down reads gate's output and
    # writes the next residual): four dependent groups per block, each a selector launch and a GEMV launch of a
    # few linears.  Reported beside the headline figure, which runs all linears of the step as one group.
    chained = None
    if args.chained and all(shapes[i][1:] == shapes[0][1:] and shapes[0][1] == shapes[0][2] for i in range(4)):   # q, k, v, o square and alike
        d, f = shapes[0][2], shapes[4][1]
        res = [torch.zeros(d, dtype=torch.float16, device="cuda") for _ in range(args.blocks + 1)]
        res[0].copy_(meta["xs_by_in"][d][0] / 1024)
        cx, cy = [], []
        for b in range(args.blocks):
            q, k_, v, o = (torch.empty(d, dtype=torch.float16, device="cuda") for _ in range(4))
            g, u = (torch.empty(f, dtype=torch.float16, device="cuda") for _ in range(2))
            cx += [res[b], res[b], res[b], v, o, o, g]
            cy += [q, k_, v, o, g, u, res[b + 1]]
        cxp, cyp = model.pointers(cx), model.pointers(cy)
        ms_chain = timed(lambda t: model.dpllm_decode_step(cxp, cyp, k_dev, e_dev), 20, 20)
        chained = {"us_per_step": round(ms_chain * 1e3, 1), "dependent_groups": 4 * args.blocks,
                   "launches_per_step": 8 * args.blocks}
        # asynchronous estimation (Sec. 5.2): the selectors of the layers fed by the residual stream read the
        # previous residual vector (q, k, v: the attention output of the block before; gate, up: the block's
        # input), so they ride in the selector launches of o and down and two of the four groups start with
        # their GEMV launch
        for b in range(args.blocks):
            for j in (0, 1, 2):
                if b > 0:
                    model.dpllm_set_selector_input(7 * b + j, cy[7 * (b - 1) + 3])
            for j in (4, 5):
                model.dpllm_set_selector_input(7 * b + j, res[b])
        ms_async = timed(lambda t: model.dpllm_decode_step(cxp, cyp, k_dev, e_dev), 20, 20)
        chained["us_per_step_async_estimation"] = round(ms_async * 1e3, 1)
        for i in range(n):
            model.dpllm_set_selector_input(i, None)
        model.dpllm_decode_step(xs, ys, k_dev, e_dev)   # back to the plan of the headline run
        torch.cuda.synchronize()

    # ---- CPU oracle on a bounded sample: the 7 linears of block 0, one step -------------------------------
    cpu = None
    if not args.no_cpu:
        import oracle
        ids = sorted(meta["host"])
        refs = [meta["host"][i] for i in ids]
        x_np = [synth.lut_np(meta["xs_by_in"][meta["shapes"][i][1]][0]) for i in ids]
        oracle.decode_step(refs[:1], x_np[:1])       # warm the library
        reps = 2
        t0 = time.perf_counter()
        for _ in range(reps):
            _, rk, _ = oracle.decode_step(refs, x_np)
        dt = (time.perf_counter() - t0) / reps
        b = sum(gemv_bytes(*meta["shapes"][i], int(k)) + selector_bytes(meta["shapes"][i][1]) for i, k in zip(ids, rk))
        cpu = {"value": round(b / dt / 1e9, 3), "unit": "GB/s", "cores": oracle.threads(), "kind": "oracle",
               "sample": "block 0 of %d (7 linears, %.0f M weights), 1 step x %d repetitions; %.1f ms per block, "
                         "scaled x%d = %.0f us per decode step" % (args.blocks, sum(o * i for o, i in [meta["shapes"][j] for j in ids]) / 1e6,
                                                                    reps, dt * 1e3, args.blocks, dt * 1e6 * args.blocks)}

    out = {
        "metric": "any-precision GEMV HBM GB/s (whole decode step at ~3.5 average bits, selectors included)",
        "value": round(bytes_step / (ms_step * 1e-3) / 1e9, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": "Llama-%s-shaped decode step: %d blocks x 7 linears, p=%d bitplanes, (l,h)=(3,4), "
                               "rank-64 projection selectors, thresholds tau~U[0.05,0.3] x median||W_h x||, "
                               "%d outlier-fp16 activation vectors, batch 1" % (args.model.upper(), args.blocks, p, n_x),
                   "linears": n, "layout": args.layout, "frac_of_hbm_peak": round(bytes_step / (ms_step * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)},
        "us_per_decode_step": round(ms_step * 1e3, 1),
        "us_per_decode_step_eager": round(ms_step_eager * 1e3, 1),
        "launch": launch_mode,
        "effective_bits": round(eff_bits, 4),
        "bytes_per_step": int(bytes_step),
        "selector": {"us_per_step": round(ms_sel * 1e3, 1), "GBps": round(sel_bytes / (ms_sel * 1e-3) / 1e9, 1),
                     "share_of_step": round(ms_sel / (ms_sel + ms_gemv), 4)},
        "per_k": per_k,
        "chained_step": chained,
        "roofline": {"bound": "hbm", "kernel": gemv_name, "achieved": round(roof_achieved, 1),
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(roof_achieved / HBM_PEAK_GBPS, 4),
                     "us_per_launch": round(ms_gemv * 1e3, 1), "algorithmic_bytes": int(gemv_bytes0),
                     "measured_read_ceiling": round(read_ceiling, 1),
                     "frac_of_measured_ceiling": round(roof_achieved / read_ceiling, 4),
                     "traffic": traffic},
        "cpu_baseline": cpu,
    }
    print(json.dumps(out), flush=True)
    model.close()


if __name__ == "__main__":
    main()
