"""Benchmark of the DP-LLM decode hot path on one MI355X.

A "step" is one whole decode step of a Llama-7B-shaped model (32 blocks x 7 linears, parent p = 8
bitplanes): for every linear the rank-64 selector estimates ||G x||, compares it with the layer's
threshold and hands the bitwidth (3 or 4) to the any-precision GEMV on the device.  Inputs are
synthetic (see synth.py) and resident in HBM before the timed region.

Prints ONE JSON line.  `value` is the whole step's algorithmic GB/s with all linears of the step in one
group (streaming throughput); beside it:
  roofline      the dominant kernel (the GEMV launch of the step) against the HBM peak, HIP events
  per_k         the same launch with every layer pinned to one bitwidth (the paper's +/-inf protocol)
  chained_step  the same linears with their buffers chained as a Transformer block chains them (a selector and a
                GEMV launch per dependency level), with and without asynchronous estimation (Sec. 5.2), and the
                selector overhead against the same step with the bitwidths pinned (the paper's overhead table)
  selector      the selector launch alone; with --hybrid also projection-only / hybrid / hybrid + asynchronous
  per_layer     us per layer and GB/s per (shape, k): streaming over >= 1 GiB of distinct copies, an isolated
                launch, and the CPU oracle on the same layer
  batch         8B-shaped linears at B = 1, 2, 4, 8 for the bitwidths of the pairs (3,4) (4,5) (5,6)
  cpu_baseline  the CPU oracle on whole steps of the same workload
`--sections` limits the run to some of them (the profiles under profiles/ are taken with `--sections step`, so
that their kernel trace holds one workload).
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0     # MI355X published HBM3E bandwidth
RANK = 64                  # projection rank used for every linear (paper Sec. 5.1)
MIN_TIMED_MS = 50.0        # the chip's clocks settle over tens of milliseconds: no timed region is shorter
ALL_SECTIONS = ["step", "per_k", "chained", "per_layer", "batch", "cpu"]


def gemv_bytes(out, in_, k, B=1):
    """Algorithmic bytes of one any-precision GEMV: top-k planes + the k-bit table + x + y."""
    return out * in_ * k / 8 + out * (1 << k) * 2 + B * in_ * 2 + B * out * 2


def selector_bytes(in_, kind=1, r=RANK):
    return (r * in_ * 2 if kind == 1 else 0) + in_ * 2 + 8


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--model", choices=["7b", "8b", "70b"], default="7b",
                    help="shape of the linears: Llama-7B (the headline workload), Llama-3-8B, or 70B with p = 6 planes")
    ap.add_argument("--blocks", type=int, default=None, help="Transformer blocks (default: 32 for 7b and 8b, 80 for 70b)")
    ap.add_argument("--quantile", type=float, default=None,
                    help="thresholds = this quantile of the calibration estimates (0.75: the 3.25-bit target) instead of tau-based ones")
    ap.add_argument("--hybrid", action="store_true",
                    help="every second linear takes the linear-regression estimator (Sec. 5.1: about half the layers)")
    ap.add_argument("--pin-k", type=int, default=None,
                    help="every layer pinned to this bitwidth for the whole run (no estimator: the paper's +/-inf protocol); "
                         "used with --sections step for per-bitwidth counter profiles")
    ap.add_argument("--sections", default=",".join(ALL_SECTIONS), help="comma list of " + ", ".join(ALL_SECTIONS))
    ap.add_argument("--no-graph", action="store_true", help="time eager launches only (no HIP graph replay)")
    ap.add_argument("--sustain", type=float, default=3.0,
                    help="seconds of back-to-back graph replays behind the 'sustained' figure (0: skip)")
    ap.add_argument("--copy-yardstick", action="store_true",
                    help="also run a plain 1 GiB copy kernel (for scaling hardware byte counters under rocprofv3 --pmc)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)")
    sections = set(s for s in args.sections.split(",") if s)
    assert sections <= set(ALL_SECTIONS), sections

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
    want_cpu = "cpu" in sections
    keep = tuple(range(args.blocks)) if want_cpu and args.model != "70b" else ((0,) if want_cpu else ())
    model, meta = synth.build_model(dp, shapes, args.blocks, p, [(l, h)], n_x, log=log, quantile=args.quantile,
                                    keep_blocks=keep, linreg_every=2 if args.hybrid else 0)
    sel = meta["sel"][(l, h)]
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
    x_tensors = [xbuf[in_] for _, in_ in meta["shapes"]]
    y_tensors = [torch.empty(out, dtype=torch.float16, device="cuda") for out, _ in meta["shapes"]]
    xs, ys = model.pointers(x_tensors), model.pointers(y_tensors)
    k_dev = torch.zeros(n, dtype=torch.int32, device="cuda")
    e_dev = torch.zeros(n, dtype=torch.float32, device="cuda")

    def set_inputs(t):
        xall.copy_(xsteps[t % n_x])

    def timed(fn, steps, warmup, min_ms=MIN_TIMED_MS):
        """ms per call of fn(t) over `steps` calls, repeated until the timed region lasts min_ms."""
        for t in range(warmup):
            fn(t)
        torch.cuda.synchronize()
        total, calls = 0.0, 0
        while calls == 0 or total < min_ms:
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for t in range(steps):
                fn(warmup + calls + t)
            e1.record()
            torch.cuda.synchronize()
            total += e0.elapsed_time(e1)
            calls += steps
        return total / calls

    def timed_graph(fn, steps, min_ms=MIN_TIMED_MS, sustain_s=0.0):
        """ms per call with `steps` calls of fn recorded once in a HIP graph and the graph replayed.  sustain_s > 0:
        also replays for that many seconds and returns the ms per call over the last third of them (the chip's
        clocks depend on how long it has been under load), else None."""
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for t in range(steps):
                fn(t)
        graph.replay()
        torch.cuda.synchronize()
        total, reps = 0.0, 0
        while reps == 0 or total < min_ms:
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            graph.replay()
            e1.record()
            torch.cuda.synchronize()
            total += e0.elapsed_time(e1)
            reps += 1
        sustained = None
        if sustain_s > 0:
            per_replay = total / reps
            n_all = max(3, int(sustain_s * 1e3 / per_replay))
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            for r in range(n_all):
                if r == n_all - n_all // 3:
                    e0.record()
                graph.replay()
            e1.record()
            torch.cuda.synchronize()
            sustained = e0.elapsed_time(e1) / ((n_all // 3) * steps)
        return total / (reps * steps), reps, sustained

    if args.pin_k is not None:
        for i in range(n):
            model.dpllm_set_selector(i, args.pin_k, args.pin_k, dp.DPLLM_SEL_NONE)
        l = h = args.pin_k
        for s_ in sel:
            s_["kind"] = 0
    out = {}
    # ---- the decode step under thresholds (selectors + GEMVs), all linears one group -------------------------
    def full_step(t):
        set_inputs(t)
        model.dpllm_decode_step(xs, ys, k_dev, e_dev)

    full_step(0)
    torch.cuda.synchronize()
    ms_step_eager = timed(full_step, args.steps, args.warmup)
    ms_step, launch_mode, timed_steps, ms_sustained = ms_step_eager, "eager launches", args.steps, None
    if not args.no_graph:
        # the same K steps recorded once in a HIP graph (per step: one input copy + two kernels) and replayed:
        # what a serving loop does to shed launch gaps.  The replay's final state is checked against eager.
        ms_graph, reps, _ = timed_graph(lambda t: full_step(args.warmup + t), args.steps)
        k_graph, y_graph = k_dev.clone(), y_tensors[-1].clone()
        full_step(args.warmup + args.steps - 1)
        torch.cuda.synchronize()
        if torch.equal(k_graph, k_dev) and torch.equal(y_graph, y_tensors[-1]):
            ms_step, launch_mode, timed_steps = ms_graph, "one HIP graph of the K steps, replayed %d times" % reps, args.steps * reps
        else:
            log("graph replay differs from eager: reporting the eager time")
    # realised bitwidths over the activation set (untimed pass)
    params = np.array([o * i for o, i in meta["shapes"]], dtype=np.float64)
    ks_hist, step_bytes = [], []
    for t in range(min(n_x, 64)):
        set_inputs(t)
        model.dpllm_decode_step(xs, ys, k_dev, e_dev)
        ks = k_dev.cpu().numpy()
        ks_hist.append(float((ks * params).sum() / params.sum()))
        step_bytes.append(sum(gemv_bytes(o, i, int(k)) + selector_bytes(i, s["kind"])
                              for (o, i), k, s in zip(meta["shapes"], ks, sel)))
    eff_bits = float(np.mean(ks_hist))
    bytes_step = float(np.mean(step_bytes))

    # ---- the two kernels apart: HIP events on the launch stream around each half ------------------------
    set_inputs(0)
    model.dpllm_decode_step(xs, ys, k_dev, e_dev)
    ks0 = k_dev.cpu().numpy().copy()
    gemv_bytes0 = sum(gemv_bytes(o, i, int(k)) for (o, i), k in zip(meta["shapes"], ks0))
    ms_gemv = timed(lambda t: model.dpllm_decode_step_parts(xs, ys, k_dev, e_dev, dp.DPLLM_STEP_GEMV), args.steps, 5)
    ms_sel = timed(lambda t: model.dpllm_decode_step_parts(xs, ys, k_dev, e_dev, dp.DPLLM_STEP_SELECT), args.steps, 5)
    sel_bytes = sum(selector_bytes(i, s["kind"]) for (_, i), s in zip(meta["shapes"], sel))
    roof_achieved = gemv_bytes0 / (ms_gemv * 1e-3) / 1e9
    # HBM traffic per GEMV launch: from the committed counter summary (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs
    # of this program, scaled by a plain copy kernel); counters cannot be read inside this run
    traffic, traffic_source = None, None
    counters = os.path.join(ROOT, "profiles", "decode_step_7b_hbm_counters.txt")
    if args.model == "7b" and args.blocks == 32 and not args.hybrid and args.quantile is None and os.path.exists(counters):
        for line in open(counters):
            if line.startswith("gemv_traffic_bytes_per_launch"):
                traffic = float(line.split()[1])
                traffic_source = "profiles/decode_step_7b_hbm_counters.txt (separate rocprofv3 --pmc runs of this workload, not this run)"

    # ---- measured ceiling: a plain non-temporal streaming read of 2 GiB on the same box ----------------------
    rbuf = torch.ones(1 << 29, dtype=torch.int32, device="cuda")
    rsink = torch.zeros(4, dtype=torch.int32, device="cuda")
    ms_read = timed(lambda t: dp.dpllm_debug_read(rbuf, rsink), 100, 100)
    read_ceiling = rbuf.numel() * 4 / (ms_read * 1e-3) / 1e9
    del rbuf

    def pin_all(k_of):
        """Every layer pinned to one bitwidth (no estimator: the paper fixes it with +/-inf thresholds)."""
        for i in range(n):
            model.dpllm_set_selector(i, int(k_of(i)), int(k_of(i)), dp.DPLLM_SEL_NONE)

    def unpin_all():
        for i in range(n):
            model.dpllm_set_active_pair(i, l, h)

    # ---- per-k sweep ------------------------------------------------------------------------------------------
    per_k = {}
    if "per_k" in sections:
        for k in range(3, p + 1):
            pin_all(lambda i: k)
            model.dpllm_decode_step(xs, ys, k_dev, e_dev)      # the selector launch writes the pinned bitwidths
            ms_k = timed(lambda t: model.dpllm_decode_step_parts(xs, ys, k_dev, e_dev, dp.DPLLM_STEP_GEMV), 25, 3)
            bk = sum(gemv_bytes(o, i, k) for o, i in meta["shapes"])
            per_k[str(k)] = {"us_per_step": round(ms_k * 1e3, 1), "GBps": round(bk / (ms_k * 1e-3) / 1e9, 1),
                             "frac_of_peak": round(bk / (ms_k * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)}
            log("k=%d: %.1f us/step, %.0f GB/s" % (k, ms_k * 1e3, per_k[str(k)]["GBps"]))
        unpin_all()
        model.dpllm_decode_step(xs, ys, k_dev, e_dev)

    # ---- the same linears with their buffers chained the way a Transformer block chains them ---------------------
    # (q, k, v read the residual; o reads v's output; gate and up read o's output; down reads gate's output and
    # writes the next residual): four dependent groups per block, each a selector launch and a GEMV launch of a
    # few linears.  Reported beside the headline figure, which runs all linears of the step as one group.
    chained = None
    if "chained" in sections and all(shapes[i][1:] == shapes[0][1:] and shapes[0][1] == shapes[0][2] for i in range(4)):
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

        def chain_step(t):
            model.dpllm_decode_step(cxp, cyp, k_dev, e_dev)

        def chain_time():
            chain_step(0)
            torch.cuda.synchronize()
            return timed(chain_step, 20, 10) if args.no_graph else timed_graph(chain_step, 10)[0]

        ms_chain = chain_time()
        kc = k_dev.cpu().numpy().copy()
        chain_bytes = sum(gemv_bytes(o, i, int(k)) + selector_bytes(i, s["kind"]) for (o, i), k, s in zip(meta["shapes"], kc, sel))
        # the same step with every layer pinned to the bitwidth it just chose and no estimator: the static model the
        # paper's overhead figures compare with
        pin_all(lambda i: kc[i])
        ms_static = chain_time()
        unpin_all()
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
        ms_async = chain_time()
        for i in range(n):
            model.dpllm_set_selector_input(i, None)
        chained = {"us_per_step": round(ms_chain * 1e3, 1), "dependent_groups": 4 * args.blocks,
                   "frac_of_hbm_peak": round(chain_bytes / (ms_chain * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                   "us_per_step_async_estimation": round(ms_async * 1e3, 1),
                   "frac_of_hbm_peak_async_estimation": round(chain_bytes / (ms_async * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                   "us_per_step_selectors_off": round(ms_static * 1e3, 1),
                   "selector_overhead_pct": round(100 * (ms_chain - ms_static) / ms_static, 2),
                   "selector_overhead_pct_async_estimation": round(100 * (ms_async - ms_static) / ms_static, 2),
                   "launch": "eager" if args.no_graph else "HIP graph"}
        model.dpllm_decode_step(xs, ys, k_dev, e_dev)   # back to the plan of the headline run
        torch.cuda.synchronize()
        log("chained: %s" % json.dumps(chained))

    # ---- per layer: streaming over >= 1 GiB of distinct copies, isolated launches, the oracle -----------------
    def layer_sweep(layer_shapes, lp, ks, batches, with_oracle):
        res = {}
        for name, o, i in layer_shapes:
            copies = max(8, int(math.ceil((1 << 30) / (o * i * min(ks) / 8))))
            m2 = dp.Model(copies)
            host = None
            for c in range(copies):
                lin = synth.make_linear(o, i, lp, 3, seed=90000 + 131 * c + o + 7 * i, device="cuda", keep_codes=False)
                m2.dpllm_load_linear(c, lin["planes"], lin["luts"], 3)
                if c == 0 and with_oracle:
                    host = {"planes": synth.planes_np(lin["planes"]), "luts": {k: synth.lut_np(v) for k, v in lin["luts"].items()}}
                del lin
            X = synth.make_x(i, max(batches), seed=4242 + i, device="cuda")
            xv = [X[0].contiguous()] * copies
            yv = [torch.empty(o, dtype=torch.float16, device="cuda") for _ in range(copies)]
            xp, yp = m2.pointers(xv), m2.pointers(yv)
            kd = torch.zeros(copies, dtype=torch.int32, device="cuda")
            ed = torch.zeros(copies, dtype=torch.float32, device="cuda")
            ybatch = torch.empty((max(batches), o), dtype=torch.float16, device="cuda")
            for k in ks:
                entry = {"copies": copies}
                if 1 in batches:
                    for c in range(copies):
                        m2.dpllm_set_selector(c, k, k, dp.DPLLM_SEL_NONE)
                    m2.dpllm_decode_step(xp, yp, kd, ed)
                    ms = timed(lambda t: m2.dpllm_decode_step_parts(xp, yp, kd, ed, dp.DPLLM_STEP_GEMV), 5, 2)
                    entry["us_streaming"] = round(ms * 1e3 / copies, 3)
                    entry["GBps_streaming"] = round(gemv_bytes(o, i, k) * copies / (ms * 1e-3) / 1e9, 1)
                    entry["frac_of_peak"] = round(entry["GBps_streaming"] / HBM_PEAK_GBPS, 4)
                for B in batches:
                    xb = X[0].contiguous() if B == 1 else X[:B].contiguous()
                    yb = ybatch[0] if B == 1 else ybatch[:B]
                    ms = timed_graph(lambda t: m2.dpllm_gemv(t % copies, k, xb, y=yb), copies)[0]
                    key = "us_isolated" if B == 1 else "us_B%d" % B
                    entry[key] = round(ms * 1e3, 3)
                    entry["GBps_isolated" if B == 1 else "GBps_B%d" % B] = round(gemv_bytes(o, i, k, B) / (ms * 1e-3) / 1e9, 1)
                if with_oracle:
                    import oracle
                    xh = synth.lut_np(X[0])
                    t0 = time.perf_counter()
                    oracle.gemv(host["planes"], k, host["luts"][k], xh)
                    entry["us_oracle"] = round((time.perf_counter() - t0) * 1e6, 0)
                res["%s %dx%d k=%d" % (name, o, i, k)] = entry
            m2.close()
            del m2, yv, xv
            torch.cuda.empty_cache()
            log("per-layer %s %dx%d done" % (name, o, i))
        return res

    per_layer = None
    if "per_layer" in sections:
        distinct = []
        for s in shapes:
            if s[1:] not in [d_[1:] for d_ in distinct]:
                distinct.append(s)
        per_layer = layer_sweep(distinct, p, list(range(3, p + 1)), [1], want_cpu)
    batch = None
    if "batch" in sections:
        distinct = []
        for s in synth.LLAMA3_8B:
            if s[1:] not in [d_[1:] for d_ in distinct]:
                distinct.append(s)
        batch = layer_sweep(distinct, 8, [3, 4, 5, 6], [1, 2, 4, 8], False)

    # ---- CPU oracle: whole steps of the same workload on the host cores (a bounded sample for the 70B shape) ----
    cpu = None
    if want_cpu:
        import oracle
        ids = sorted(meta["host"])
        refs = [dict(meta["host"][i], selector=synth.oracle_selector(meta, (l, h), i)) for i in ids]
        oracle.decode_step(refs[:1], [synth.lut_np(meta["xs_by_in"][meta["shapes"][ids[0]][1]][0])])       # warm the library
        reps = 2 if len(ids) == n else 4
        t0 = time.perf_counter()
        b = 0.0
        for rep in range(reps):
            x_np = [synth.lut_np(meta["xs_by_in"][meta["shapes"][i][1]][rep]) for i in ids]
            _, rk, _ = oracle.decode_step(refs, x_np)
            b += sum(gemv_bytes(*meta["shapes"][i], int(k)) + selector_bytes(meta["shapes"][i][1], sel[i]["kind"]) for i, k in zip(ids, rk))
        dt = time.perf_counter() - t0
        whole = len(ids) == n
        cpu = {"value": round(b / dt / 1e9, 3), "unit": "GB/s", "cores": oracle.threads(), "kind": "oracle",
               "us_per_decode_step": round(dt / reps * 1e6 * (1 if whole else args.blocks), 0),
               "sample": ("%d whole decode steps (all %d linears), %.1f s of CPU time" % (reps, n, dt)) if whole else
                         ("block 0 of %d (7 linears), %d steps, %.1f s; us_per_decode_step is that x %d" % (args.blocks, reps, dt, args.blocks))}

    # ---- last, so that nothing else is measured on a chip it has warmed up: the step's graph replayed for seconds --
    if args.sustain > 0 and not args.no_graph and "step" in sections:
        full_step(0)                                   # back to the plan of the unchained step
        torch.cuda.synchronize()
        ms_sustained = timed_graph(lambda t: full_step(args.warmup + t), args.steps, min_ms=0.0, sustain_s=args.sustain)[2]
        log("sustained: %.1f us/step over the last third of %.1f s" % (ms_sustained * 1e3, args.sustain))
    out = {
        "metric": "any-precision GEMV HBM GB/s (whole decode step at ~%.2f average bits, selectors included)" % eff_bits,
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
                               "rank-64 projection selectors%s, thresholds %s, %d outlier-fp16 activation vectors, batch 1, "
                               "all linears of the step in one dependency group"
                               % (args.model.upper(), args.blocks, p,
                                  (" (every second linear: linear regression)" if args.hybrid else "") +
                                  (" REPLACED by every layer pinned to k=%d" % args.pin_k if args.pin_k is not None else ""),
                                  "tau~U[0.05,0.3] x median||W_h x||" if args.quantile is None else "= %.2f-quantile of the calibration estimates" % args.quantile,
                                  n_x),
                   "linears": n, "frac_of_hbm_peak": round(bytes_step / (ms_step * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                   "timed_steps": timed_steps},
        "us_per_decode_step": round(ms_step * 1e3, 1),
        "us_per_decode_step_eager": round(ms_step_eager * 1e3, 1),
        "launch": launch_mode,
        "sustained": None if ms_sustained is None else {
            "us_per_decode_step": round(ms_sustained * 1e3, 1), "seconds": args.sustain,
            "note": "the same graph replayed back to back for this long, timed over the last third"},
        "effective_bits": round(eff_bits, 4),
        "bytes_per_step": int(bytes_step),
        "selector": {"us_per_step": round(ms_sel * 1e3, 1), "GBps": round(sel_bytes / (ms_sel * 1e-3) / 1e9, 1),
                     "frac_of_peak": round(sel_bytes / (ms_sel * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                     "share_of_step": round(ms_sel / (ms_sel + ms_gemv), 4),
                     "linears_on_linear_regression": sum(1 for s in sel if s["kind"] == 2)},
        "per_k": per_k,
        "chained_step": chained,
        "per_layer": per_layer,
        "batch": batch,
        "roofline": {"bound": "hbm", "kernel": "gemv_lane_kernel<1>", "achieved": round(roof_achieved, 1),
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(roof_achieved / HBM_PEAK_GBPS, 4),
                     "us_per_launch": round(ms_gemv * 1e3, 1), "algorithmic_bytes": int(gemv_bytes0),
                     "measured_read_ceiling": round(read_ceiling, 1),
                     "frac_of_measured_ceiling": round(roof_achieved / read_ceiling, 4),
                     "traffic": traffic, "traffic_source": traffic_source},
        "cpu_baseline": cpu,
    }
    print(json.dumps(out), flush=True)
    model.close()


if __name__ == "__main__":
    main()
