"""GPU parity at the full sizes of the benchmark configurations, in the launch configuration bench.py
times (one selector launch + one GEMV launch for the whole step).  Every decision and estimate of every
(step, linear) is checked against the oracle; GEMV outputs are checked against the oracle, by norm and row
by row, on the first, middle and last Transformer block, whose canonical planes are kept on the host."""
import numpy as np
import pytest
import torch

import oracle
import synth

pytestmark = pytest.mark.gpu

REL_L2 = 2e-3
DECISION_BAND = 1e-9


@pytest.fixture(scope="module")
def dp():
    """The binding (importing it loads the HIP library; there is no other path)."""
    import paper_2508_06041_amd as dp
    assert torch.cuda.is_available()
    return dp


def rel_l2(got, ref):
    ref = np.asarray(ref, dtype=np.float64)
    return np.linalg.norm(np.asarray(got, dtype=np.float64) - ref) / max(np.linalg.norm(ref), 1e-300)


def row_bound(y_ref, lut_k, x_bits, in_):
    """Per-row error allowed to a GEMV that accumulates in fp32 and stores fp16: half an fp16 ulp of the result
    twice over, plus the rounding of ~in fp32 additions of terms no larger than max|W_row| max|x| (random-walk
    growth, factor 2), plus the smallest fp16 step."""
    wmax = np.abs(lut_k.view(np.float16).astype(np.float64)).max(axis=1)
    xmax = float(np.abs(x_bits.view(np.float16).astype(np.float64)).max())
    return 2.0 ** -10 * np.abs(y_ref) + 2.0 * np.sqrt(in_) * 2.0 ** -24 * wmax * xmax + 2.0 ** -24


def check_gemv(y_gpu, ref, k, x_bits, where):
    """Norm-wise (the stated 2e-3) and row by row: a row that drops or doubles a tile fails the second."""
    y_ref = oracle.gemv(ref["planes"], k, ref["luts"][k], x_bits)
    got = y_gpu.float().cpu().numpy().astype(np.float64)
    assert rel_l2(got, y_ref) <= REL_L2, where
    bad = np.abs(got - y_ref) > row_bound(y_ref, ref["luts"][k], x_bits, x_bits.size)
    assert not bad.any(), (where, int(bad.sum()), int(np.argmax(bad)))


def step_buffers(meta):
    shapes = meta["shapes"]
    ins = sorted(meta["xs_by_in"])
    xbuf = {in_: torch.empty(in_, dtype=torch.float16, device="cuda") for in_ in ins}
    xs = [xbuf[in_] for _, in_ in shapes]
    ys = [torch.empty(out, dtype=torch.float16, device="cuda") for out, _ in shapes]
    k_dev = torch.zeros(len(shapes), dtype=torch.int32, device="cuda")
    e_dev = torch.zeros(len(shapes), dtype=torch.float32, device="cuda")
    return xbuf, xs, ys, k_dev, e_dev


def check_all_decisions(model, meta, pair, steps, gemv_steps):
    """Every (step, linear): estimate and decision against the oracle.  On `gemv_steps`: the GEMV outputs of the
    linears whose planes are on the host.  The oracle's estimates (one plain C call each) are spread over a pool
    of host threads."""
    from concurrent.futures import ThreadPoolExecutor
    shapes = meta["shapes"]
    ins = sorted(meta["xs_by_in"])
    xbuf, xs, ys, k_dev, e_dev = step_buffers(meta)
    sel = meta["sel"][pair]
    G_np = [synth.lut_np(s["G"]) for s in sel]
    x_np = {in_: synth.lut_np(meta["xs_by_in"][in_]) for in_ in ins}
    steps = list(steps)
    ks_all, es_all = [], []
    for t in steps:
        for in_ in ins:
            xbuf[in_].copy_(meta["xs_by_in"][in_][t])
        model.dpllm_decode_step(xs, ys, k_dev, e_dev)
        torch.cuda.synchronize()
        ks_all.append(k_dev.cpu().numpy())
        es_all.append(e_dev.cpu().numpy())
        if t in gemv_steps:
            for i, ref in meta["host"].items():
                check_gemv(ys[i], ref, int(ks_all[-1][i]), x_np[shapes[i][1]][t], (i, t))

    def one_linear(i):
        in_ = shapes[i][1]
        return [oracle.estimate(G_np[i], x_np[in_][t]) for t in steps]

    with ThreadPoolExecutor(max_workers=16) as pool:
        e_ref_all = list(pool.map(one_linear, range(len(shapes))))
    for i in range(len(shapes)):
        T = sel[i]["T"]
        for j, t in enumerate(steps):
            e_ref = e_ref_all[i][j]
            assert abs(e_ref - T) > DECISION_BAND * max(abs(T), e_ref), (i, t)
            assert int(ks_all[j][i]) == oracle.decide(e_ref, T, *pair), (i, t, e_ref, T)
            assert abs(float(es_all[j][i]) - e_ref) <= 3e-7 * e_ref, (i, t)
    params = np.array([o * i for o, i in shapes], dtype=np.int64)
    seen = set(int(k) for ks in ks_all for k in ks)
    bits = [oracle.effective_bits(ks, params) for ks in ks_all]
    return seen, bits


def test_decode_step_llama7b_every_step_every_linear(dp):
    """32 blocks x 7 linears, p = 8, (l,h) = (3,4), rank-64 selectors, 256 activation vectors: every decision and
    estimate of the 256 x 224 (step, linear) pairs exact against the oracle; GEMV outputs of blocks 0, 15 and 31
    against the oracle, norm-wise and row by row."""
    model, meta = synth.build_model(dp, synth.LLAMA_7B, 32, 8, [(3, 4)], 256, seed=4321, keep_blocks=(0, 15, 31))
    seen, bits = check_all_decisions(model, meta, (3, 4), steps=range(256), gemv_steps={0, 255})
    assert seen == {3, 4}
    assert 3.2 < float(np.mean(bits)) < 3.8
    # every bitwidth pinned for all layers (the +/-inf protocol of the latency runs)
    shapes = meta["shapes"]
    n = len(shapes)
    xbuf, xs, ys, k_dev, e_dev = step_buffers(meta)
    ins = sorted(meta["xs_by_in"])
    for in_ in ins:
        xbuf[in_].copy_(meta["xs_by_in"][in_][1])
    x_np = {in_: synth.lut_np(meta["xs_by_in"][in_][1]) for in_ in ins}
    for k in range(3, 9):
        for i in range(n):
            model.dpllm_set_selector(i, k, k, dp.DPLLM_SEL_NONE)
        model.dpllm_decode_step(xs, ys, k_dev, e_dev)
        torch.cuda.synchronize()
        assert (k_dev.cpu().numpy() == k).all()
        for i, ref in meta["host"].items():
            check_gemv(ys[i], ref, k, x_np[shapes[i][1]], (i, k))
    model.close()


def test_decode_step_llama70b_all_blocks_quantile_thresholds(dp):
    """All 80 blocks of the 70B shape resident (q/o 8192^2, k/v 1024x8192, gate/up 28672x8192, down 8192x28672,
    p = 6: 51 GB of planes), thresholds = 0.75-quantile of the calibration estimates, the 3.25-bit target: every
    decision of every calibration step exact, realised average 3.25 bits, GEMV outputs of blocks 0, 39 and 79
    against the oracle on the first and last step."""
    n_x = 32
    model, meta = synth.build_model(dp, synth.LLAMA_70B, 80, 6, [(3, 4)], n_x, seed=99, keep_blocks=(0, 39, 79),
                                    quantile=0.75)
    seen, bits = check_all_decisions(model, meta, (3, 4), steps=range(n_x), gemv_steps={0, n_x - 1})
    assert seen == {3, 4}
    # realised share of low-precision decisions over the calibration set: 0.75 +- 1/n per layer, hence 3.25 bits
    for i, s in enumerate(meta["sel"][(3, 4)]):
        frac_l = float((s["est"].cpu().numpy() <= s["T"]).mean())
        assert abs(frac_l - 0.75) <= 1.0 / n_x + 1e-9, (i, frac_l)
    assert abs(float(np.mean(bits)) - 3.25) <= 0.01, float(np.mean(bits))
    model.close()


@pytest.mark.parametrize("name,out,in_", [(n, o, i) for n, o, i in synth.LLAMA3_8B if n in ("q", "k", "gate", "down")])
def test_llama3_8b_shapes_small_batch(dp, name, out, in_):
    """8B shapes, p = 8, the bitwidths of the pairs (3,4) (4,5) (5,6), batch 1, 2, 4, 8."""
    lin = synth.make_linear(out, in_, 8, 3, seed=out + 3 * in_, device="cuda", keep_codes=False)
    model = dp.Model(1)
    model.dpllm_load_linear(0, lin["planes"], lin["luts"], 3)
    ref = {"planes": synth.planes_np(lin["planes"]), "luts": {k: synth.lut_np(v) for k, v in lin["luts"].items()}}
    X = synth.make_x(in_, 8, seed=5)
    for k in (3, 4, 5, 6):
        for B in (1, 2, 4, 8):
            xb = X[0].cuda() if B == 1 else X[:B].cuda()
            got = model.dpllm_gemv(0, k, xb).reshape(B, out)
            for b in range(B):
                check_gemv(got[b], ref, k, synth.lut_np(X[b]), (k, B, b))
    model.close()
