"""GPU parity: the HIP library, called through its C boundary, against the CPU oracle on the
same seeded inputs.  Integer work (codes, bitwidth decisions) must be bit-exact; GEMV outputs
must be within 2e-3 relative L2 (fp32 accumulation, fp16 result)."""
import math

import numpy as np
import pytest
import torch

import oracle
import synth

pytestmark = pytest.mark.gpu

REL_L2 = 2e-3          # tolerance of the GEMV output stated for this path
DECISION_BAND = 1e-9   # decisions must agree wherever |e - T| exceeds this relative band


@pytest.fixture(scope="module")
def dp():
    """The binding (importing it loads the HIP library; there is no other path)."""
    import paper_2508_06041_amd as dp
    assert torch.cuda.is_available()
    return dp


def rel_l2(got, ref):
    ref = np.asarray(ref, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    n = np.linalg.norm(ref)
    return np.linalg.norm(got - ref) / (n if n > 0 else 1.0)


def load(dp, lins):
    model = dp.Model(len(lins))
    for i, lin in enumerate(lins):
        model.dpllm_load_linear(i, synth.planes_np(lin["planes"]),
                                {k: synth.lut_np(v) for k, v in lin["luts"].items()}, lin["kmin"])
    return model


# ----------------------------------------------------------------------------- T1 codes
@pytest.mark.parametrize("p", range(1, 9))
def test_unpack_bit_exact_all_p_k(dp, p):
    rng = np.random.default_rng(p)
    for out, in_ in [(1, 32), (33, 96), (7, 2080), (130, 4096 + 32)]:
        planes = rng.integers(0, 2 ** 32, size=(p, out, in_ // 32), dtype=np.uint32)
        luts = {k: np.zeros((out, 1 << k), dtype=np.uint16) for k in range(1, p + 1)}
        model = dp.Model(1)
        model.dpllm_load_linear(0, planes, luts, 1)
        ref_p = oracle.unpack(planes)
        for k in range(1, p + 1):
            got = model.dpllm_debug_unpack(0, k).cpu().numpy()
            assert (got == oracle.index_k(ref_p, p, k)).all(), (p, k, out, in_)
        model.close()


def test_load_from_device_pointers_matches_host_load(dp):
    lin = synth.make_linear(40, 160, 6, 3, seed=5)
    a = load(dp, [lin])
    b = dp.Model(1)
    b.dpllm_load_linear(0, lin["planes"].cuda(), {k: v.cuda() for k, v in lin["luts"].items()}, 3)
    x = synth.make_x(160, 1, seed=6)[0].cuda()
    for k in range(3, 7):
        assert torch.equal(a.dpllm_debug_unpack(0, k), b.dpllm_debug_unpack(0, k))
        assert torch.equal(a.dpllm_gemv(0, k, x), b.dpllm_gemv(0, k, x))


# ----------------------------------------------------------------------------- T3 GEMV
TINY = [(2, 32, 4, 3), (7, 64, 8, 3), (33, 96, 5, 3), (5, 160, 3, 1), (257, 2048 + 64, 8, 3), (64, 11008, 6, 3)]


@pytest.mark.parametrize("out,in_,p,kmin", TINY)
def test_gemv_small_shapes_all_k(dp, out, in_, p, kmin):
    lin = synth.make_linear(out, in_, p, kmin, seed=out + in_)
    model = load(dp, [lin])
    x = synth.make_x(in_, 1, seed=out)[0]
    planes = synth.planes_np(lin["planes"])
    for k in range(kmin, p + 1):
        ref = oracle.gemv(planes, k, synth.lut_np(lin["luts"][k]), synth.lut_np(x))
        got = model.dpllm_gemv(0, k, x.cuda()).float().cpu().numpy()
        assert rel_l2(got, ref) <= REL_L2, (k, rel_l2(got, ref))
    model.close()


def test_gemv_special_inputs(dp):
    lin = synth.make_linear(48, 256, 6, 3, seed=77)
    model = load(dp, [lin])
    planes = synth.planes_np(lin["planes"])
    codes = oracle.unpack(planes)
    for c in (0, 31, 32, 100, 255):       # x = e_c returns column c of W_k exactly
        e = torch.zeros(256, dtype=torch.float16)
        e[c] = 1.0
        for k in (3, 6):
            got = model.dpllm_gemv(0, k, e.cuda()).cpu().numpy()
            lut = synth.to_np(lin["luts"][k])
            assert (got == lut[np.arange(48), codes[:, c] >> (6 - k)]).all()
    zero = torch.zeros(256, dtype=torch.float16, device="cuda")
    assert (model.dpllm_gemv(0, 4, zero) == 0).all()
    model.close()


def test_gemv_config0_1024(dp):
    lin = synth.make_linear(1024, 1024, 4, 3, seed=0)
    x = synth.make_x(1024, 1, seed=0, outliers=False)[0]
    model = load(dp, [lin])
    for k in (3, 4):
        ref = oracle.gemv(synth.planes_np(lin["planes"]), k, synth.lut_np(lin["luts"][k]), synth.lut_np(x))
        got = model.dpllm_gemv(0, k, x.cuda()).float().cpu().numpy()
        assert rel_l2(got, ref) <= REL_L2
    model.close()


@pytest.mark.parametrize("out,in_", [(4096, 4096), (11008, 4096), (4096, 11008)])
def test_gemv_llama7b_shapes_k3_to_8(dp, out, in_):
    lin = synth.make_linear(out, in_, 8, 3, seed=out * 7 + in_, device="cuda", keep_codes=False)
    model = dp.Model(1)
    model.dpllm_load_linear(0, lin["planes"], lin["luts"], 3)
    x = synth.make_x(in_, 1, seed=3)[0]
    planes = synth.planes_np(lin["planes"])
    for k in range(3, 9):
        ref = oracle.gemv(planes, k, synth.lut_np(lin["luts"][k]), synth.lut_np(x))
        got = model.dpllm_gemv(0, k, x.cuda()).float().cpu().numpy()
        assert rel_l2(got, ref) <= REL_L2, (k, rel_l2(got, ref))
    model.close()


@pytest.mark.parametrize("B", [2, 3, 4, 5, 7, 8])
def test_gemv_small_batch(dp, B):
    """Groups of up to four samples share one pass over the planes; ragged last group, ragged last tile."""
    in_ = 4096 + 96
    lin = synth.make_linear(260, in_, 8, 3, seed=B)
    model = load(dp, [lin])
    X = synth.make_x(in_, B, seed=10 + B)
    planes = synth.planes_np(lin["planes"])
    for k in range(3, 9):
        ref = oracle.gemv(planes, k, synth.lut_np(lin["luts"][k]), synth.lut_np(X))
        got = model.dpllm_gemv(0, k, X.cuda()).float().cpu().numpy()
        assert got.shape == (B, 260)
        for b in range(B):
            assert rel_l2(got[b], ref[b]) <= REL_L2, (k, b)
    # bitwidth of a candidate pair read on the device, whole batch at that bitwidth
    model.dpllm_set_selector(0, 4, 5, dp.DPLLM_SEL_LINREG, alpha=0.0, beta=1.0, T=0.5)
    for k_sel in (4, 5):
        k_dev = torch.tensor([k_sel], dtype=torch.int32, device="cuda")
        got = model.dpllm_gemv(0, -1, X.cuda(), k_dev=k_dev).float().cpu().numpy()
        ref = oracle.gemv(planes, k_sel, synth.lut_np(lin["luts"][k_sel]), synth.lut_np(X))
        assert rel_l2(got, ref) <= REL_L2, k_sel
    model.close()


# ----------------------------------------------------------------------------- T4-T6 selector
def test_estimate_matches_oracle_and_hands_k_over(dp):
    lin = synth.make_linear(96, 4096 + 256, 5, 3, seed=21)
    model = load(dp, [lin])
    planes = synth.planes_np(lin["planes"])
    for r in (1, 16, 64, 256):
        G = synth.make_G(lin, 3, 4, r, seed=22 + r)
        xs = synth.make_x(lin["in"], 6, seed=23)
        est = [oracle.estimate(synth.lut_np(G), synth.lut_np(x)) for x in xs]
        T = synth.nudge_threshold(float(np.median(est)), torch.tensor(est))
        model.dpllm_set_selector(0, 3, 4, dp.DPLLM_SEL_PROJ, G=G.cuda(), T=T)
        for x, e_ref in zip(xs, est):
            e, k = model.dpllm_estimate(0, 3, 4, x.cuda())
            k_ref = oracle.decide(e_ref, T, 3, 4)
            assert abs(e_ref - T) > DECISION_BAND * max(abs(T), e_ref)
            assert int(k) == k_ref
            assert float(e) == float(np.float32(e_ref)) or math.isclose(float(e), e_ref, rel_tol=3e-7)
            y = model.dpllm_gemv(0, -1, x.cuda(), k_dev=k)      # bitwidth read on the device
            ref = oracle.gemv(planes, k_ref, synth.lut_np(lin["luts"][k_ref]), synth.lut_np(x))
            assert rel_l2(y.float().cpu().numpy(), ref) <= REL_L2
            assert torch.equal(y, model.dpllm_gemv(0, k_ref, x.cuda()))
    model.close()


def test_degenerate_thresholds_and_kinds(dp):
    lin = synth.make_linear(64, 512, 6, 3, seed=31)
    model = load(dp, [lin])
    G = synth.make_G(lin, 4, 5, 64, seed=32).cuda()
    x = synth.make_x(512, 1, seed=33)[0]
    model.dpllm_set_selector(0, 4, 5, dp.DPLLM_SEL_PROJ, G=G, T=float("inf"))
    assert int(model.dpllm_estimate(0, 4, 5, x.cuda())[1]) == 4
    model.dpllm_set_threshold(0, 4, 5, float("-inf"))
    assert int(model.dpllm_estimate(0, 4, 5, x.cuda())[1]) == 5
    model.dpllm_set_threshold(0, 4, 5, -1.0)
    assert int(model.dpllm_estimate(0, 4, 5, x.cuda())[1]) == 5
    e_ref = oracle.estimate(synth.lut_np(G.cpu()), synth.lut_np(x))
    model.dpllm_set_threshold(0, 4, 5, float(np.float32(e_ref)) * 2)
    assert int(model.dpllm_estimate(0, 4, 5, x.cuda())[1]) == 4
    # linear-regression estimator
    alpha, beta = 0.375, 0.5
    model.dpllm_set_selector(0, 3, 4, dp.DPLLM_SEL_LINREG, alpha=alpha, beta=beta, T=0.0)
    e, k = model.dpllm_estimate(0, 3, 4, x.cuda())
    assert math.isclose(float(e), oracle.linreg_estimate(synth.lut_np(x), alpha, beta), rel_tol=3e-7)
    assert int(k) == 4
    # no estimator: l == h
    model.dpllm_set_selector(0, 6, 6, dp.DPLLM_SEL_NONE)
    e, k = model.dpllm_estimate(0, 6, 6, x.cuda())
    assert int(k) == 6 and float(e) == 0.0
    model.close()


def _step_model(dp, shapes, p, l, h, r, n_steps, seed, mode):
    """Builds a model with one selector per linear; returns everything the comparison needs."""
    lins, refs = [], []
    model = dp.Model(len(shapes))
    xs_by_in = {in_: synth.make_x(in_, n_steps, seed=seed + in_) for _, in_ in shapes}
    for i, (out, in_) in enumerate(shapes):
        lin = synth.make_linear(out, in_, p, 3, seed=seed + 13 * i)
        G = synth.make_G(lin, l, h, r, seed=seed + 17 * i + 1)
        est = synth.estimates_fp64(G, xs_by_in[in_])
        if mode == "inf":
            T = float("inf")
        elif mode == "-inf":
            T = float("-inf")
        else:
            T = synth.nudge_threshold(synth.quantile_threshold(est, 0.5), est, band=1e-6)
        model.dpllm_load_linear(i, synth.planes_np(lin["planes"]),
                                {k: synth.lut_np(v) for k, v in lin["luts"].items()}, 3)
        model.dpllm_set_selector(i, l, h, dp.DPLLM_SEL_PROJ, G=G.cuda(), T=T)
        refs.append({"planes": synth.planes_np(lin["planes"]),
                     "luts": {k: synth.lut_np(v) for k, v in lin["luts"].items()},
                     "selector": {"l": l, "h": h, "kind": 1, "G": synth.lut_np(G), "T": T}})
        lins.append(lin)
    return model, refs, xs_by_in


@pytest.mark.parametrize("mode", ["mixed", "inf", "-inf"])
def test_decode_step_matches_oracle(dp, mode):
    shapes = [(128, 256), (128, 256), (64, 256), (128, 128), (320, 256), (320, 256), (256, 320)]
    n_steps = 12
    model, refs, xs_by_in = _step_model(dp, shapes, 5, 3, 4, 64, n_steps, seed=900, mode=mode)
    n = len(shapes)
    k_dev = torch.zeros(n, dtype=torch.int32, device="cuda")
    e_dev = torch.zeros(n, dtype=torch.float32, device="cuda")
    seen = set()
    for t in range(n_steps):
        xs = [xs_by_in[in_][t].cuda() for _, in_ in shapes]
        ys = [torch.empty(out, dtype=torch.float16, device="cuda") for out, _ in shapes]
        model.dpllm_decode_step(xs, ys, k_dev, e_dev)
        torch.cuda.synchronize()
        ry, rk, re = oracle.decode_step(refs, [synth.lut_np(xs_by_in[in_][t]) for _, in_ in shapes])
        for ref, e in zip(refs, re):
            T = ref["selector"]["T"]
            if np.isfinite(T):
                assert abs(e - T) > DECISION_BAND * max(abs(T), e)
        assert k_dev.cpu().numpy().tolist() == rk.tolist()
        assert np.allclose(e_dev.cpu().numpy(), re, rtol=3e-7)
        for y, r in zip(ys, ry):
            assert rel_l2(y.float().cpu().numpy(), r) <= REL_L2
        seen.update(rk.tolist())
    assert seen == ({3, 4} if mode == "mixed" else {3} if mode == "inf" else {4})
    model.close()



def test_decode_step_with_selector_inputs(dp):
    """Asynchronous estimation (Sec. 5.2): some selectors read another vector (the previous residual); the
    decisions follow that vector, the GEMVs still read the immediate inputs."""
    shapes = [(128, 256), (64, 256), (320, 256), (256, 320)]
    n_steps = 6
    model, refs, xs_by_in = _step_model(dp, shapes, 5, 3, 4, 64, n_steps, seed=6100, mode="mixed")
    n = len(shapes)
    k_dev = torch.zeros(n, dtype=torch.int32, device="cuda")
    e_dev = torch.zeros(n, dtype=torch.float32, device="cuda")
    prev = {in_: torch.zeros(in_, dtype=torch.float16, device="cuda") for in_ in xs_by_in}
    for i in (0, 2):
        model.dpllm_set_selector_input(i, prev[shapes[i][1]])
    flips = 0
    for t in range(1, n_steps):
        for in_ in prev:
            prev[in_].copy_(xs_by_in[in_][t - 1])
        xs = [xs_by_in[in_][t].cuda() for _, in_ in shapes]
        ys = [torch.empty(out, dtype=torch.float16, device="cuda") for out, _ in shapes]
        model.dpllm_decode_step(xs, ys, k_dev, e_dev)
        torch.cuda.synchronize()
        x_np = [synth.lut_np(xs_by_in[in_][t]) for _, in_ in shapes]
        xsel_np = [synth.lut_np(xs_by_in[in_][t - 1]) if i in (0, 2) else None for i, (_, in_) in enumerate(shapes)]
        ry, rk, re = oracle.decode_step(refs, x_np, xsel_np)
        _, rk_now, _ = oracle.decode_step(refs, x_np)
        flips += int((rk != rk_now).sum())
        assert k_dev.cpu().numpy().tolist() == rk.tolist()
        assert np.allclose(e_dev.cpu().numpy(), re, rtol=3e-7)
        for y, r in zip(ys, ry):
            assert rel_l2(y.float().cpu().numpy(), r) <= REL_L2
    assert flips > 0      # the two inputs really lead to different decisions somewhere
    model.dpllm_set_selector_input(0, None)
    model.dpllm_set_selector_input(2, None)
    xs = [xs_by_in[in_][0].cuda() for _, in_ in shapes]
    ys = [torch.empty(out, dtype=torch.float16, device="cuda") for out, _ in shapes]
    model.dpllm_decode_step(xs, ys, k_dev, e_dev)
    _, rk, _ = oracle.decode_step(refs, [synth.lut_np(xs_by_in[in_][0]) for _, in_ in shapes])
    assert k_dev.cpu().numpy().tolist() == rk.tolist()
    model.close()


def test_decode_step_chained_buffers_run_in_order(dp):
    """Linears that read what earlier ones write (o <- v, gate/up <- o, down <- gate) are ordered by the
    library: the result equals running them one after the other.  Bitwidths are pinned (alternating +/-inf) so
    that the comparison does not hinge on estimates of slightly different inputs; the oracle chains its own
    fp16-rounded outputs."""
    shapes = [(128, 256), (128, 256), (256, 256), (256, 256), (320, 256), (320, 256), (256, 320)]
    names = ["q", "k", "v", "o", "gate", "up", "down"]
    src = {"q": None, "k": None, "v": None, "o": "v", "gate": "o", "up": "o", "down": "gate"}
    lins, refs = [], []
    model = dp.Model(len(shapes))
    for i, (out, in_) in enumerate(shapes):
        lin = synth.make_linear(out, in_, 5, 3, seed=4100 + i)
        T = float("inf") if i % 2 == 0 else float("-inf")
        G = synth.make_G(lin, 3, 4, 16, seed=4200 + i)
        model.dpllm_load_linear(i, synth.planes_np(lin["planes"]),
                                {k: synth.lut_np(v) for k, v in lin["luts"].items()}, 3)
        model.dpllm_set_selector(i, 3, 4, dp.DPLLM_SEL_PROJ, G=G.cuda(), T=T)
        refs.append({"planes": synth.planes_np(lin["planes"]),
                     "luts": {k: synth.lut_np(v) for k, v in lin["luts"].items()},
                     "selector": {"l": 3, "h": 4, "kind": 1, "G": synth.lut_np(G), "T": T}})
    x0 = (synth.make_x(256, 1, seed=4300)[0].float() / 1024).half()   # keeps the chain inside fp16 range
    ybuf = {nm: torch.zeros(out, dtype=torch.float16, device="cuda") for nm, (out, _) in zip(names, shapes)}
    x0_dev = x0.cuda()
    xs = [x0_dev if src[nm] is None else ybuf[src[nm]] for nm in names]
    ys = [ybuf[nm] for nm in names]
    k_dev = torch.zeros(len(shapes), dtype=torch.int32, device="cuda")
    e_dev = torch.zeros(len(shapes), dtype=torch.float32, device="cuda")
    for _ in range(2):     # second call: cached plan
        for b in ybuf.values():
            b.zero_()
        model.dpllm_decode_step(xs, ys, k_dev, e_dev)
        torch.cuda.synchronize()
        ref_y = {}
        for i, nm in enumerate(names):
            x = synth.lut_np(x0) if src[nm] is None else ref_y[src[nm]].astype(np.float16).view(np.uint16)
            k_ref = 3 if i % 2 == 0 else 4
            ref_y[nm] = oracle.gemv(refs[i]["planes"], k_ref, refs[i]["luts"][k_ref], x)
            assert int(k_dev[i]) == k_ref
            assert rel_l2(ybuf[nm].float().cpu().numpy(), ref_y[nm]) <= REL_L2, nm
    model.close()


def test_decode_step_under_graph_capture_replays(dp):
    """A step with a cached plan only enqueues kernels, so it can be captured in a graph; every replay, with
    eager work and new inputs in between, must give what the eager call gives (bit for bit) and the oracle's
    decisions."""
    shapes = [(128, 256), (64, 256), (320, 256), (256, 320)]
    n_steps = 5
    model, refs, xs_by_in = _step_model(dp, shapes, 5, 3, 4, 64, n_steps, seed=5100, mode="mixed")
    n = len(shapes)
    xbuf = {in_: torch.zeros(in_, dtype=torch.float16, device="cuda") for in_ in xs_by_in}
    xs = [xbuf[in_] for _, in_ in shapes]
    ys = [torch.zeros(out, dtype=torch.float16, device="cuda") for out, _ in shapes]
    k_dev = torch.zeros(n, dtype=torch.int32, device="cuda")
    e_dev = torch.zeros(n, dtype=torch.float32, device="cuda")

    def set_inputs(t):
        for in_ in xbuf:
            xbuf[in_].copy_(xs_by_in[in_][t])

    set_inputs(0)
    model.dpllm_decode_step(xs, ys, k_dev, e_dev)      # builds the plan (not capturable: it copies tables)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        model.dpllm_decode_step(xs, ys, k_dev, e_dev)
    for t in range(n_steps):
        set_inputs(t)
        model.dpllm_decode_step(xs, ys, k_dev, e_dev)
        torch.cuda.synchronize()
        eager_y = [y.clone() for y in ys]
        eager_k, eager_e = k_dev.clone(), e_dev.clone()
        for y in ys:
            y.zero_()
        k_dev.zero_()
        e_dev.zero_()
        graph.replay()
        torch.cuda.synchronize()
        _, rk, _ = oracle.decode_step(refs, [synth.lut_np(xs_by_in[in_][t]) for _, in_ in shapes])
        assert k_dev.cpu().numpy().tolist() == rk.tolist()
        assert torch.equal(k_dev, eager_k) and torch.equal(e_dev, eager_e)
        for y, ey in zip(ys, eager_y):
            assert torch.equal(y, ey)
    model.close()


def _mixed_kind_model(dp, shapes, p, pairs, n_steps, seed):
    """Small model whose linears hold several candidate pairs and all three selector kinds: index % 3 == 0 the
    projection, 1 the linear regression, 2 none for the pair (l, l) (a layer pinned to one bitwidth)."""
    model = dp.Model(len(shapes))
    xs_by_in = {in_: synth.make_x(in_, n_steps, seed=seed + in_) for _, in_ in shapes}
    # activation norms that differ from step to step, so that the linear regression has something to decide on
    for in_ in xs_by_in:
        scale = torch.linspace(0.5, 2.0, n_steps)[torch.randperm(n_steps, generator=torch.Generator().manual_seed(seed))]
        xs_by_in[in_] = (xs_by_in[in_].float() * scale[:, None]).half()
    refs = []
    for i, (out, in_) in enumerate(shapes):
        lin = synth.make_linear(out, in_, p, 3, seed=seed + 13 * i)
        model.dpllm_load_linear(i, synth.planes_np(lin["planes"]),
                                {k: synth.lut_np(v) for k, v in lin["luts"].items()}, 3)
        sels = {}
        for l, h in reversed(pairs):
            xs = xs_by_in[in_]
            if i % 3 == 0:
                G = synth.make_G(lin, l, h, 64 if l == 3 else 40, seed=seed + 17 * i + l)
                est = synth.estimates_fp64(G, xs)
                sel = {"l": l, "h": h, "kind": 1, "G": synth.lut_np(G), "alpha": 0.0, "beta": 0.0}
                model.dpllm_set_selector(i, l, h, dp.DPLLM_SEL_PROJ, G=G.cuda(), T=0.0)
            elif i % 3 == 1:
                alpha, beta = 0.25 + 0.05 * i, -1.0
                est = synth.linreg_estimates_fp64(xs, alpha, beta)
                sel = {"l": l, "h": h, "kind": 2, "alpha": alpha, "beta": beta}
                model.dpllm_set_selector(i, l, h, dp.DPLLM_SEL_LINREG, alpha=alpha, beta=beta, T=0.0)
            else:
                est = None
                sel = {"l": l, "h": l, "kind": 0, "alpha": 0.0, "beta": 0.0}
                model.dpllm_set_selector(i, l, l, dp.DPLLM_SEL_NONE)
            sel["est"] = est
            sels[(l, h)] = sel
        refs.append({"planes": synth.planes_np(lin["planes"]),
                     "luts": {k: synth.lut_np(v) for k, v in lin["luts"].items()}, "sels": sels})
    return model, refs, xs_by_in


def _threshold(sel, rho):
    if sel["est"] is None:
        return 0.0
    return synth.nudge_threshold(synth.quantile_threshold(sel["est"], rho), sel["est"], band=1e-6)


def _oracle_step(refs, pair, Ts, x_np):
    lins = []
    for ref, T in zip(refs, Ts):
        s = dict(ref["sels"][pair])
        s["T"] = T
        lins.append({"planes": ref["planes"], "luts": ref["luts"], "selector": s})
    return oracle.decode_step(lins, x_np)


def test_decode_step_mixed_selector_kinds(dp):
    """One step launch with projection, linear-regression and no-estimator linears side by side; linears that
    read the same vector share one pass over x^2 (Sec. 5.1: about half the layers take the linear regression).
    Estimates, decisions and outputs against the oracle on every step."""
    shapes = [(128, 256), (128, 256), (64, 256), (128, 128), (320, 256), (320, 256), (256, 320), (96, 320), (64, 128)]
    n_steps = 10
    model, refs, xs_by_in = _mixed_kind_model(dp, shapes, 5, [(3, 4)], n_steps, seed=7300)
    n = len(shapes)
    Ts = [_threshold(r["sels"][(3, 4)], 0.5) for r in refs]
    for i, r in enumerate(refs):
        s = r["sels"][(3, 4)]
        if s["kind"]:
            model.dpllm_set_threshold(i, s["l"], s["h"], Ts[i])
    k_dev = torch.zeros(n, dtype=torch.int32, device="cuda")
    e_dev = torch.zeros(n, dtype=torch.float32, device="cuda")
    seen = {1: set(), 2: set()}
    for t in range(n_steps):
        xs = [xs_by_in[in_][t].cuda() for _, in_ in shapes]
        ys = [torch.empty(out, dtype=torch.float16, device="cuda") for out, _ in shapes]
        model.dpllm_decode_step(xs, ys, k_dev, e_dev)
        torch.cuda.synchronize()
        ry, rk, re = _oracle_step(refs, (3, 4), Ts, [synth.lut_np(xs_by_in[in_][t]) for _, in_ in shapes])
        for i in range(n):
            kind = refs[i]["sels"][(3, 4)]["kind"]
            if kind:
                assert abs(re[i] - Ts[i]) > DECISION_BAND * max(abs(Ts[i]), abs(re[i])), (i, t)
                seen[kind].add(int(rk[i]))
        assert k_dev.cpu().numpy().tolist() == rk.tolist(), t
        assert np.allclose(e_dev.cpu().numpy(), re, rtol=3e-7, atol=0), t
        for y, r in zip(ys, ry):
            assert rel_l2(y.float().cpu().numpy(), r) <= REL_L2
    assert seen[1] == {3, 4} and seen[2] == {3, 4}
    model.close()


def test_target_switch_between_graph_replays(dp):
    """Run-time adaptation (Sec. 2.1; Algorithm 1: one threshold list per target; Sec. 5.1: one G per pair): three
    targets resident -- (3,4) at the median threshold, (4,5) at the median, (3,4) at the 0.75 quantile -- and one
    captured step.  dpllm_set_target switches between replays with one device word; every replay must give the
    oracle's decisions, estimates and outputs for the target in force, and rebuild nothing."""
    shapes = [(128, 256), (128, 256), (64, 256), (128, 128), (320, 256), (320, 256), (256, 320)]
    n_steps = 8
    pairs = [(3, 4), (4, 5)]
    model, refs, xs_by_in = _mixed_kind_model(dp, shapes, 5, pairs, n_steps, seed=8400)
    n = len(shapes)
    targets = {0: ((3, 4), 0.5), 1: ((4, 5), 0.5), 2: ((3, 4), 0.75)}
    T_of = {}
    for t, (pair, rho) in targets.items():
        T_of[t] = [_threshold(r["sels"][pair], rho) for r in refs]
        for i, r in enumerate(refs):
            s = r["sels"][pair]
            if t == 0:
                if s["kind"]:
                    model.dpllm_set_threshold(i, s["l"], s["h"], T_of[t][i])
            else:
                model.dpllm_set_target_entry(t, i, s["l"], s["h"], T_of[t][i])
    xbuf = {in_: torch.zeros(in_, dtype=torch.float16, device="cuda") for in_ in xs_by_in}
    xs = [xbuf[in_] for _, in_ in shapes]
    ys = [torch.zeros(out, dtype=torch.float16, device="cuda") for out, _ in shapes]
    k_dev = torch.zeros(n, dtype=torch.int32, device="cuda")
    e_dev = torch.zeros(n, dtype=torch.float32, device="cuda")
    for in_ in xbuf:
        xbuf[in_].copy_(xs_by_in[in_][0])
    model.dpllm_decode_step(xs, ys, k_dev, e_dev)      # builds the plan and copies the tables (not capturable)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        model.dpllm_decode_step(xs, ys, k_dev, e_dev)
    seen = {t: set() for t in targets}
    for step, t in enumerate([0, 1, 2, 2, 0, 1, 0, 2]):
        model.dpllm_set_target(t)
        for in_ in xbuf:
            xbuf[in_].copy_(xs_by_in[in_][step])
        for y in ys:
            y.zero_()
        graph.replay()
        torch.cuda.synchronize()
        pair = targets[t][0]
        ry, rk, re = _oracle_step(refs, pair, T_of[t], [synth.lut_np(xs_by_in[in_][step]) for _, in_ in shapes])
        for i in range(n):
            if refs[i]["sels"][pair]["kind"]:
                assert abs(re[i] - T_of[t][i]) > DECISION_BAND * max(abs(T_of[t][i]), abs(re[i])), (i, step)
        assert k_dev.cpu().numpy().tolist() == rk.tolist(), (step, t)
        assert np.allclose(e_dev.cpu().numpy(), re, rtol=3e-7, atol=0), (step, t)
        for y, r in zip(ys, ry):
            assert rel_l2(y.float().cpu().numpy(), r) <= REL_L2, (step, t)
        seen[t].update(rk.tolist())
    assert seen[0] >= {3, 4} and seen[1] >= {4, 5} and seen[2] >= {3, 4}
    # the same switches with eager steps
    for step, t in enumerate([1, 0]):
        model.dpllm_set_target(t)
        model.dpllm_decode_step(xs, ys, k_dev, e_dev)
        torch.cuda.synchronize()
        _, rk, _ = _oracle_step(refs, targets[t][0], T_of[t], [synth.lut_np(xs_by_in[in_][7]) for _, in_ in shapes])
        assert k_dev.cpu().numpy().tolist() == rk.tolist(), (step, t)
    model.close()


def test_loaded_planes_sit_where_the_host_says(dp):
    """dpllm_debug_locate (host arithmetic, pinned without a GPU in test_abi_symbols.py) against what
    dpllm_load_linear really writes: planes with a few single bits set, loaded, and the arena read back: exactly
    the predicted bits of the plane regions are set, ragged rows and columns included."""
    import ctypes as C
    out, in_, p = 70, 288, 5
    rng = np.random.default_rng(5)
    planes = np.zeros((p, out, in_ // 32), dtype=np.uint32)
    picks = {(int(rng.integers(p)), int(rng.integers(out)), int(rng.integers(in_))) for _ in range(60)}
    picks |= {(0, 0, 0), (p - 1, out - 1, in_ - 1), (2, 63, 127), (3, 64, 128)}
    for b, o, c in picks:
        planes[b, o, c // 32] |= np.uint32(1) << np.uint32(c % 32)
    luts = {k: np.zeros((out, 1 << k), dtype=np.uint16) for k in range(3, p + 1)}
    model = dp.Model(1)
    model.dpllm_load_linear(0, planes, luts, 3)
    torch.cuda.synchronize()
    arena = model.arenas[0].cpu().numpy()
    nrq, ncc = (out + 63) // 64, (in_ // 32 + 3) // 4
    words = arena[:p * nrq * ncc * 1024].view(np.uint32)
    want = np.zeros_like(words)
    for b, o, c in picks:
        off, bit = C.c_size_t(0), C.c_int(0)
        assert dp.lib.dpllm_debug_locate(out, in_, p, 3, b, o, c, C.byref(off), C.byref(bit)) == dp.DPLLM_OK
        want[off.value // 4] |= np.uint32(1) << np.uint32(bit.value)
    assert int(np.unpackbits(want.view(np.uint8)).sum()) == len(picks)
    assert np.array_equal(words, want)
    model.close()


# ----------------------------------------------------------------------------- T7 error paths
def test_abi_error_paths(dp):
    lin = synth.make_linear(8, 64, 4, 3, seed=1)
    model = load(dp, [lin, lin])
    x = torch.zeros(64, dtype=torch.float16, device="cuda")
    with pytest.raises(dp.DpllmError) as ei:
        model.dpllm_gemv(0, 2, x)                      # below kmin
    assert ei.value.code == dp.DPLLM_ERANGE
    with pytest.raises(dp.DpllmError) as ei:
        model.dpllm_gemv(0, 5, x)                      # above p
    assert ei.value.code == dp.DPLLM_ERANGE
    with pytest.raises(dp.DpllmError) as ei:
        model.dpllm_gemv(5, 3, x)                      # bad id
    assert ei.value.code == dp.DPLLM_EINVAL
    with pytest.raises(dp.DpllmError) as ei:
        model.dpllm_gemv(0, 3, torch.zeros(9, 64, dtype=torch.float16, device="cuda"),
                         y=torch.zeros(9, 8, dtype=torch.float16, device="cuda"))
    assert ei.value.code == dp.DPLLM_ESHAPE
    with pytest.raises(dp.DpllmError) as ei:
        model.dpllm_estimate(0, 3, 4, x)               # selector not set
    assert ei.value.code == dp.DPLLM_ESTATE
    with pytest.raises(dp.DpllmError) as ei:
        model.dpllm_set_selector(0, 3, 4, dp.DPLLM_SEL_PROJ, G=torch.zeros(4, 64, dtype=torch.float16, device="cuda"),
                                 T=float("nan"))
    assert ei.value.code == dp.DPLLM_EINVAL
    with pytest.raises(dp.DpllmError) as ei:
        model.dpllm_gemv(0, -1, x)                     # dynamic k without k_dev
    assert ei.value.code == dp.DPLLM_EINVAL
    k_dev = torch.zeros(2, dtype=torch.int32, device="cuda")
    e_dev = torch.zeros(2, dtype=torch.float32, device="cuda")
    with pytest.raises(dp.DpllmError) as ei:           # decode step without selectors
        model.dpllm_decode_step([x, x], [torch.zeros(8, dtype=torch.float16, device="cuda")] * 2, k_dev, e_dev)
    assert ei.value.code == dp.DPLLM_ESTATE
    empty = dp.Model(1)
    with pytest.raises(dp.DpllmError) as ei:
        empty.dpllm_gemv(0, 3, x)                      # not loaded
    assert ei.value.code == dp.DPLLM_ESTATE
    import ctypes as C
    n = C.c_size_t(0)
    assert dp.lib.dpllm_linear_device_bytes(8, 48, 4, 3, C.byref(n)) == dp.DPLLM_ESHAPE
    # x and y of one GEMV must not overlap
    buf = torch.zeros(128, dtype=torch.float16, device="cuda")
    with pytest.raises(dp.DpllmError) as ei:
        model.dpllm_gemv(0, 3, buf[:64], y=buf[56:64])
    assert ei.value.code == dp.DPLLM_EINVAL
    # targets: 1 .. DPLLM_MAX_TARGETS - 1 hold entries, the pair of an entry must have been attached
    model.dpllm_set_selector(0, 3, 4, dp.DPLLM_SEL_LINREG, alpha=1.0, beta=0.0, T=1.0)
    for bad in (0, dp.DPLLM_MAX_TARGETS, -1):
        with pytest.raises(dp.DpllmError) as ei:
            model.dpllm_set_target_entry(bad, 0, 3, 4, 1.0)
        assert ei.value.code == dp.DPLLM_EINVAL
    with pytest.raises(dp.DpllmError) as ei:
        model.dpllm_set_target_entry(1, 0, 3, 3, 1.0)          # pair (3,3) was never attached
    assert ei.value.code == dp.DPLLM_ESTATE
    with pytest.raises(dp.DpllmError) as ei:
        model.dpllm_set_target_entry(1, 0, 3, 4, float("nan"))
    assert ei.value.code == dp.DPLLM_EINVAL
    for bad in (-1, dp.DPLLM_MAX_TARGETS):
        with pytest.raises(dp.DpllmError) as ei:
            model.dpllm_set_target(bad)
        assert ei.value.code == dp.DPLLM_EINVAL
    # the workspace: too small, misaligned; a step, an estimate and a target switch without one
    need = model.dpllm_workspace_bytes()
    small = torch.empty(need, dtype=torch.uint8, device="cuda")
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    assert dp.lib.dpllm_set_workspace(model.h, C.c_void_p(small.data_ptr()), C.c_size_t(need - 256), stream) == dp.DPLLM_ESTATE
    assert dp.lib.dpllm_set_workspace(model.h, C.c_void_p(small.data_ptr() + 16), C.c_size_t(need), stream) == dp.DPLLM_EINVAL
    bare = dp.Model(1)
    bare.dpllm_load_linear(0, synth.planes_np(lin["planes"]), {k: synth.lut_np(v) for k, v in lin["luts"].items()}, 3)
    bare.dpllm_set_selector(0, 3, 4, dp.DPLLM_SEL_LINREG, alpha=1.0, beta=0.0, T=1.0)
    assert bare.workspace is None
    assert dp.lib.dpllm_set_target(bare.h, 1, stream) == dp.DPLLM_ESTATE
    e1 = torch.zeros(1, dtype=torch.float32, device="cuda")
    k1 = torch.zeros(1, dtype=torch.int32, device="cuda")
    assert dp.lib.dpllm_estimate(bare.h, 0, 3, 4, C.c_void_p(x.data_ptr()), C.c_void_p(e1.data_ptr()), C.c_void_p(k1.data_ptr()),
                                 stream) == dp.DPLLM_ESTATE
    y8 = torch.zeros(8, dtype=torch.float16, device="cuda")
    xs1, ys1 = (C.c_void_p * 1)(x.data_ptr()), (C.c_void_p * 1)(y8.data_ptr())
    assert dp.lib.dpllm_decode_step(bare.h, xs1, ys1, C.c_void_p(k1.data_ptr()), C.c_void_p(e1.data_ptr()), stream) == dp.DPLLM_ESTATE
    # ... while a GEMV needs none, and the entry point that allocates nothing neither
    assert dp.lib.dpllm_gemv(bare.h, 0, 3, None, C.c_void_p(x.data_ptr()), C.c_void_p(y8.data_ptr()), 1, stream) == dp.DPLLM_OK
    assert dp.lib.dpllm_estimate_noalloc(bare.h, 0, 3, 4, C.c_void_p(x.data_ptr()), C.c_void_p(e1.data_ptr()),
                                         C.c_void_p(k1.data_ptr()), stream) == dp.DPLLM_OK
    torch.cuda.synchronize()
    assert bare.workspace is None and int(k1.item()) == 3      # x = 0: estimate 0 <= T
    model.close()
    empty.close()
    bare.close()


# ----------------------------------------------------------------------------- T8 random shapes, long runs
@pytest.mark.parametrize("seed", range(6))
def test_gemv_random_shapes(dp, seed):
    """Random odd shapes, every bitwidth the linear serves, random batch: ragged rows, ragged strips, short
    and empty tails."""
    rng = np.random.default_rng(1000 + seed)
    for _ in range(4):
        out = int(rng.integers(1, 600))
        in_ = 32 * int(rng.integers(1, 300))
        p = int(rng.integers(3, 9))
        B = int(rng.integers(1, 6))
        lin = synth.make_linear(out, in_, p, 3, seed=int(rng.integers(1 << 30)))
        model = load(dp, [lin])
        X = synth.make_x(in_, B, seed=int(rng.integers(1 << 30)))
        planes = synth.planes_np(lin["planes"])
        for k in range(3, p + 1):
            ref = oracle.gemv(planes, k, synth.lut_np(lin["luts"][k]), synth.lut_np(X))
            got = model.dpllm_gemv(0, k, (X if B > 1 else X[0]).cuda()).float().cpu().numpy().reshape(B, out)
            for b in range(B):
                assert rel_l2(got[b], ref[b]) <= REL_L2, (out, in_, p, k, B, b)
        model.close()


@pytest.mark.parametrize("out,in_", [(65600, 160), (65604, 4096)])
def test_gemv_many_rows_several_row_quads_per_wavefront(dp, out, in_):
    """More than 16384 row quads in one launch: every wavefront streams two or more row quads (table hand-over,
    resident activations, ring across row-quad boundaries), batch 1 and 2."""
    lin = synth.make_linear(out, in_, 5, 3, seed=out + in_, device="cuda", keep_codes=False)
    model = dp.Model(1)
    model.dpllm_load_linear(0, lin["planes"], lin["luts"], 3)
    X = synth.make_x(in_, 2, seed=77)
    planes = synth.planes_np(lin["planes"])
    for k in (3, 4, 5):
        lut = synth.lut_np(lin["luts"][k])
        ref = oracle.gemv(planes, k, lut, synth.lut_np(X))
        got1 = model.dpllm_gemv(0, k, X[0].cuda()).float().cpu().numpy()
        got2 = model.dpllm_gemv(0, k, X.cuda()).float().cpu().numpy()
        assert rel_l2(got1, ref[0]) <= REL_L2, k
        assert rel_l2(got2[0], ref[0]) <= REL_L2 and rel_l2(got2[1], ref[1]) <= REL_L2, k
    model.close()


@pytest.mark.parametrize("out,in_", [(200, 3072), (64, 8192 + 32), (130, 2080), (1, 16384)])
def test_gemv_few_rows_long_columns(dp, out, in_):
    """Launches with far fewer blocks of rows than compute units: in the row-per-lane arrangement several
    workgroups share a block of rows and the last one to finish adds up their partial sums.  Single calls with
    one to three samples and a decode step; every call twice, which must give the same bits (the arrival counters
    are back at zero, the order of the additions is fixed)."""
    lin = synth.make_linear(out, in_, 8, 3, seed=out + in_)
    other = synth.make_linear(96, in_, 8, 3, seed=out + in_ + 1)
    model = load(dp, [lin, other])
    X = synth.make_x(in_, 3, seed=31)
    planes = synth.planes_np(lin["planes"])
    for k in range(3, 9):
        ref = oracle.gemv(planes, k, synth.lut_np(lin["luts"][k]), synth.lut_np(X))
        for B in (1, 2, 3):
            xb = (X[:B] if B > 1 else X[0]).cuda()
            got = model.dpllm_gemv(0, k, xb)
            again = model.dpllm_gemv(0, k, xb)
            assert torch.equal(got, again), (k, B)
            got = got.float().cpu().numpy().reshape(B, out)
            for b in range(B):
                assert rel_l2(got[b], ref[b]) <= REL_L2, (k, B, b)
    # both linears in one launch of the decode step
    xs = [X[0].cuda(), X[1].cuda()]
    ys = [torch.empty(out, dtype=torch.float16, device="cuda"), torch.empty(96, dtype=torch.float16, device="cuda")]
    k_dev = torch.zeros(2, dtype=torch.int32, device="cuda")
    e_dev = torch.zeros(2, dtype=torch.float32, device="cuda")
    for k in (3, 6):
        for i in range(2):
            model.dpllm_set_selector(i, k, k, dp.DPLLM_SEL_NONE)
        first = None
        for _ in range(2):
            model.dpllm_decode_step(xs, ys, k_dev, e_dev)
            torch.cuda.synchronize()
            if first is None:
                first = [y.clone() for y in ys]
        assert all(torch.equal(a, b) for a, b in zip(first, ys))
        for i, l in enumerate((lin, other)):
            ref = oracle.gemv(synth.planes_np(l["planes"]), k, synth.lut_np(l["luts"][k]), synth.lut_np(X[i]))
            assert rel_l2(ys[i].float().cpu().numpy(), ref) <= REL_L2, (k, i)
    model.close()


def test_decode_step_async_selectors_in_chained_blocks(dp):
    """Two chained blocks (q, k, v, o, gate, up, down) with asynchronous estimation (Sec. 5.2): q, k, v of the
    second block estimate from the first block's attention output, gate and up from their block's input.  The
    library runs those selectors in an earlier selector launch than their own group's; every estimate must
    still come from the buffer named, as it stands when the linear runs, every decision from that estimate,
    every GEMV from its immediate input at the decided bitwidth.  Checked on the buffers read back."""
    d, f = 256, 320
    names = ["q", "k", "v", "o", "gate", "up", "down"]
    shapes = [(d, d), (d, d), (d, d), (d, d), (f, d), (f, d), (d, f)]
    nb = 2
    n = nb * 7
    model = dp.Model(n)
    refs = []
    for i in range(n):
        out, in_ = shapes[i % 7]
        lin = synth.make_linear(out, in_, 5, 3, seed=5100 + i)
        lin["luts"] = {k: (v.float() / 16).half() for k, v in lin["luts"].items()}   # keeps the chain inside fp16 range
        G = synth.make_G(lin, 3, 4, 32, seed=5200 + i)
        model.dpllm_load_linear(i, synth.planes_np(lin["planes"]),
                                {k: synth.lut_np(v) for k, v in lin["luts"].items()}, 3)
        model.dpllm_set_selector(i, 3, 4, dp.DPLLM_SEL_PROJ, G=G.cuda(), T=float("inf"))
        refs.append({"planes": synth.planes_np(lin["planes"]), "luts": {k: synth.lut_np(v) for k, v in lin["luts"].items()},
                     "G": G})
    res = [torch.zeros(d, dtype=torch.float16, device="cuda") for _ in range(nb + 1)]
    res[0].copy_(synth.make_x(d, 1, seed=5300)[0])
    xs, ys, sel_in = [], [], [None] * n
    for b in range(nb):
        q, k_, v, o = (torch.zeros(d, dtype=torch.float16, device="cuda") for _ in range(4))
        g, u = (torch.zeros(f, dtype=torch.float16, device="cuda") for _ in range(2))
        xs += [res[b], res[b], res[b], v, o, o, g]
        ys += [q, k_, v, o, g, u, res[b + 1]]
    for b in range(nb):
        if b > 0:
            for j in (0, 1, 2):
                sel_in[7 * b + j] = ys[7 * (b - 1) + 3]
        for j in (4, 5):
            sel_in[7 * b + j] = res[b]
    k_dev = torch.zeros(n, dtype=torch.int32, device="cuda")
    e_dev = torch.zeros(n, dtype=torch.float32, device="cuda")

    def check(T, use_sel):
        for _ in range(2):   # twice with the same inputs: every buffer holds the value its readers saw
            model.dpllm_decode_step(xs, ys, k_dev, e_dev)
        torch.cuda.synchronize()
        ks, es = k_dev.cpu().numpy(), e_dev.cpu().numpy()
        for i in range(n):
            src = sel_in[i] if use_sel and sel_in[i] is not None else xs[i]
            e_ref = oracle.estimate(synth.lut_np(refs[i]["G"]), synth.lut_np(src))
            assert math.isclose(float(es[i]), e_ref, rel_tol=3e-7), i
            assert math.isinf(T[i]) or abs(e_ref - T[i]) > DECISION_BAND * max(abs(T[i]), e_ref)
            assert int(ks[i]) == oracle.decide(e_ref, T[i], 3, 4), i
            y_ref = oracle.gemv(refs[i]["planes"], int(ks[i]), refs[i]["luts"][int(ks[i])], synth.lut_np(xs[i]))
            assert rel_l2(ys[i].float().cpu().numpy(), y_ref) <= REL_L2, i
        return ks, es

    _, es = check([float("inf")] * n, False)             # immediate inputs, everything at l: the scale of the estimates
    for i in range(n):
        model.dpllm_set_selector_input(i, sel_in[i])
    T = [float(es[i]) * (0.5 if i % 2 else 2.0) for i in range(n)]
    for i in range(n):
        model.dpllm_set_selector(i, 3, 4, dp.DPLLM_SEL_PROJ, G=refs[i]["G"].cuda(), T=T[i])
    ks, _ = check(T, True)
    assert set(ks.tolist()) == {3, 4}
    model.close()


@pytest.mark.parametrize("in_,r", [(1056, 17), (11008, 64), (11008, 1024), (32, 3), (16416, 40)])
def test_estimate_ranks_and_row_lengths(dp, in_, r):
    """The selector alone over row lengths that are not multiples of a column chunk (512) and ranks that are not
    multiples of a row group (16), up to the largest rank: a lone selector is cut into row groups x column chunks
    and the part that finishes last adds up the partial products."""
    lin = synth.make_linear(4, in_, 4, 3, seed=in_ + r)
    model = load(dp, [lin])
    g = torch.Generator().manual_seed(in_ * 7 + r)
    G = (torch.randn(r, in_, generator=g) / math.sqrt(r)).half()
    xs = synth.make_x(in_, 3, seed=r)
    est = [oracle.estimate(synth.lut_np(G), synth.lut_np(x)) for x in xs]
    T = synth.nudge_threshold(float(np.median(est)), torch.tensor(est))
    model.dpllm_set_selector(0, 3, 4, dp.DPLLM_SEL_PROJ, G=G.cuda(), T=T)
    for x, e_ref in zip(xs, est):
        for _ in range(2):      # the arrival counter is back at zero after a call
            e, k = model.dpllm_estimate(0, 3, 4, x.cuda())
            assert math.isclose(float(e), e_ref, rel_tol=3e-7)
            assert abs(e_ref - T) > DECISION_BAND * max(abs(T), e_ref)
            assert int(k) == oracle.decide(e_ref, T, 3, 4)
    model.close()
