"""GPU parity at the full sizes of the benchmark configurations, in the launch configuration bench.py
times (one selector launch + one GEMV launch per candidate pair for the whole step).  Decisions are checked
for every linear against the oracle; GEMV outputs are checked against the oracle on the linears whose
canonical planes are kept on the host, and on every other linear through a property that holds at any
size: the multi-job step launch must reproduce, bit for bit, the single-linear call at the same bitwidth."""
import numpy as np
import pytest
import torch

import oracle
import synth

pytestmark = pytest.mark.gpu

REL_L2 = 2e-3
DECISION_BAND = 1e-9


@pytest.fixture(scope="module", params=["rowquad", "rowlane"])
def dp(request):
    """The binding, with every model of the test created in one of the two plane arrangements."""
    import os
    import paper_2508_06041_amd as dp
    assert torch.cuda.is_available()
    old = os.environ.get("DPLLM_LAYOUT")
    os.environ["DPLLM_LAYOUT"] = request.param
    yield dp
    if old is None:
        del os.environ["DPLLM_LAYOUT"]
    else:
        os.environ["DPLLM_LAYOUT"] = old


def rel_l2(got, ref):
    ref = np.asarray(ref, dtype=np.float64)
    return np.linalg.norm(np.asarray(got, dtype=np.float64) - ref) / max(np.linalg.norm(ref), 1e-300)


def same_up_to_sum_order(a, b):
    return torch.equal(a, b) or rel_l2(a.float().cpu().numpy(), b.double().cpu().numpy()) <= 2e-4


def run_step_checks(dp, model, meta, l, h, steps, check_all_single=True):
    import bench  # noqa: F401  (build_model lives there)
    shapes = meta["shapes"]
    n = len(shapes)
    ins = sorted(meta["xs_by_in"])
    xbuf = {in_: torch.empty(in_, dtype=torch.float16, device="cuda") for in_ in ins}
    xs = [xbuf[in_] for _, in_ in shapes]
    ys = [torch.empty(out, dtype=torch.float16, device="cuda") for out, _ in shapes]
    k_dev = torch.zeros(n, dtype=torch.int32, device="cuda")
    e_dev = torch.zeros(n, dtype=torch.float32, device="cuda")
    G_np = [synth.lut_np(G) for G in meta["G"]]
    seen = set()
    for t in steps:
        for in_ in ins:
            xbuf[in_].copy_(meta["xs_by_in"][in_][t])
        model.dpllm_decode_step(xs, ys, k_dev, e_dev)
        torch.cuda.synchronize()
        ks = k_dev.cpu().numpy()
        es = e_dev.cpu().numpy()
        x_np = {in_: synth.lut_np(meta["xs_by_in"][in_][t]) for in_ in ins}
        for i, (out, in_) in enumerate(shapes):      # every decision, every estimate
            e_ref = oracle.estimate(G_np[i], x_np[in_])
            T = meta["T"][i]
            assert abs(e_ref - T) > DECISION_BAND * max(abs(T), e_ref), (i, t)
            assert int(ks[i]) == oracle.decide(e_ref, T, l, h), (i, t, e_ref, T)
            assert abs(float(es[i]) - e_ref) <= 3e-7 * e_ref
        seen.update(int(k) for k in ks)
        for i, ref in meta["host"].items():           # oracle GEMV where canonical planes are on the host
            k = int(ks[i])
            y_ref = oracle.gemv(ref["planes"], k, ref["luts"][k], x_np[shapes[i][1]])
            assert rel_l2(ys[i].float().cpu().numpy(), y_ref) <= REL_L2, (i, t, k)
        if check_all_single:
            # multi-job launch == single-linear launch: bitwise, unless the small launch split the columns of a
            # row over several workgroups (row-per-lane arrangement), which changes the order of the fp32 sums
            for i in range(n):
                y1 = model.dpllm_gemv(i, int(ks[i]), xs[i])
                assert same_up_to_sum_order(y1, ys[i]), (i, t)
    return seen


def test_decode_step_llama7b_full(dp):
    """32 blocks x 7 linears, p = 8, (l,h) = (3,4), rank-64 selectors: every decision of 3 steps exact, GEMV
    outputs of block 0 against the oracle, all 224 outputs against the single-linear launches."""
    import bench
    model, meta = bench.build_model(dp, synth, torch, synth.LLAMA_7B, 32, 8, 3, 4, 8, seed=4321, keep_blocks=(0,))
    seen = run_step_checks(dp, model, meta, 3, 4, steps=[0, 3, 7])
    assert seen == {3, 4}
    # The parts of a selector hand their partial sums over inside one launch; the same step repeated must give
    # the same bits every time, also while other launches keep the memory system busy (a hand-over that is not
    # ordered shows up as a stale partial sum once in a few hundred estimates).
    n_all = len(meta["shapes"])
    xs_r = [meta["xs_by_in"][in_][5].contiguous() for _, in_ in meta["shapes"]]
    ys_r = [torch.empty(out, dtype=torch.float16, device="cuda") for out, _ in meta["shapes"]]
    k_r = torch.zeros(n_all, dtype=torch.int32, device="cuda")
    e_r = torch.zeros(n_all, dtype=torch.float32, device="cuda")
    other = torch.cuda.Stream()
    big = torch.ones(1 << 27, dtype=torch.int32, device="cuda")
    first = None
    for rep in range(40):
        with torch.cuda.stream(other):     # unrelated traffic next to the step
            big.add_(1)
        model.dpllm_decode_step(xs_r, ys_r, k_r, e_r)
        torch.cuda.synchronize()
        now = (k_r.clone(), e_r.clone(), ys_r[6].clone(), ys_r[-1].clone())
        if first is None:
            first = now
        assert all(torch.equal(a, b) for a, b in zip(first, now)), rep
    del big
    # every bitwidth pinned for all layers (the +/-inf protocol of the latency runs): the streaming launch
    # (several row quads per wavefront) against the oracle on block 0 and against single launches elsewhere
    shapes = meta["shapes"]
    n = len(shapes)
    ins = sorted(meta["xs_by_in"])
    xs = [meta["xs_by_in"][in_][1].contiguous() for _, in_ in shapes]
    ys = [torch.empty(out, dtype=torch.float16, device="cuda") for out, _ in shapes]
    k_dev = torch.zeros(n, dtype=torch.int32, device="cuda")
    e_dev = torch.zeros(n, dtype=torch.float32, device="cuda")
    for k in range(3, 9):
        for i in range(n):
            model.dpllm_set_selector(i, k, k, dp.DPLLM_SEL_NONE)
        model.dpllm_decode_step(xs, ys, k_dev, e_dev)
        torch.cuda.synchronize()
        assert (k_dev.cpu().numpy() == k).all()
        for i, ref in meta["host"].items():
            y_ref = oracle.gemv(ref["planes"], k, ref["luts"][k], synth.lut_np(xs[i]))
            assert rel_l2(ys[i].float().cpu().numpy(), y_ref) <= REL_L2, (i, k)
        for i in range(0, n, 5):
            assert same_up_to_sum_order(model.dpllm_gemv(i, k, xs[i]), ys[i]), (i, k)
    model.close()


def test_decode_step_llama70b_shapes_quantile_thresholds(dp):
    """Two blocks of the 70B shape (q/o 8192^2, k/v 1024x8192, gate/up 28672x8192, down 8192x28672), p = 6,
    thresholds = 0.75-quantile of the calibration estimates (3.25-bit target)."""
    import bench
    n_x = 16
    model, meta = bench.build_model(dp, synth, torch, synth.LLAMA_70B, 2, 6, 3, 4, n_x, seed=99, keep_blocks=(0,),
                                    quantile=0.75)
    seen = run_step_checks(dp, model, meta, 3, 4, steps=[0, n_x - 1])
    assert seen == {3, 4}
    # realised share of low-precision decisions over the calibration set: 0.75 +- 1/n per layer
    shapes = meta["shapes"]
    for i, est in enumerate(meta["est"]):
        frac_l = float((est.cpu().numpy() <= meta["T"][i]).mean())
        assert abs(frac_l - 0.75) <= 1.0 / n_x + 1e-9, (i, frac_l)
    model.close()


@pytest.mark.parametrize("name,out,in_", [(n, o, i) for n, o, i in synth.LLAMA3_8B if n in ("q", "k", "gate", "down")])
def test_llama3_8b_shapes_small_batch(dp, name, out, in_):
    """8B shapes, p = 8, the bitwidths of the pairs (3,4) (4,5) (5,6), batch 1, 2, 4, 8."""
    lin = synth.make_linear(out, in_, 8, 3, seed=out + 3 * in_, device="cuda", keep_codes=False)
    model = dp.Model(1)
    model.dpllm_load_linear(0, lin["planes"], lin["luts"], 3)
    planes = synth.planes_np(lin["planes"])
    X = synth.make_x(in_, 8, seed=5)
    for k in (3, 4, 5, 6):
        lut = synth.lut_np(lin["luts"][k])
        ref = oracle.gemv(planes, k, lut, synth.lut_np(X))
        for B in (1, 2, 4, 8):
            xb = X[0].cuda() if B == 1 else X[:B].cuda()
            got = model.dpllm_gemv(0, k, xb).float().cpu().numpy()
            r = ref[0] if B == 1 else ref[:B]
            assert rel_l2(got, r) <= REL_L2, (k, B, rel_l2(got, r))
    model.close()
