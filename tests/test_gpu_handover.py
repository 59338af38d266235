"""GPU tests of the two places where workgroups hand partial results to one another inside a launch: the parts
of a projection selector (partial dot products of G x) and the column-split GEMV (partial row sums).  Both
leave their partial results in workspace slots that the launch plan fixes, so a slot that the last-arriving
workgroup reads before the writer's value is visible still holds what the PREVIOUS launch left there.  The tests
therefore alternate two different input sets on successive launches: a stale slot then holds the other input's
partial result, which changes the estimate (or the output row) by a large factor and fails the bitwise comparison
with a clean run of the same input and the comparison with the oracle.  (Repeating one input would hide exactly
this failure: a stale slot would hold the right value.)"""
import numpy as np
import pytest
import torch

import oracle
import synth

pytestmark = pytest.mark.gpu

REL_L2 = 2e-3


@pytest.fixture(scope="module")
def dp():
    import paper_2508_06041_amd as dp
    assert torch.cuda.is_available()
    return dp


def rel_l2(got, ref):
    ref = np.asarray(ref, dtype=np.float64)
    return np.linalg.norm(np.asarray(got, dtype=np.float64) - ref) / max(np.linalg.norm(ref), 1e-300)


def test_selector_handover_alternating_inputs_full_step(dp):
    """The 224 selectors of a 7B-shaped step (one launch, every selector cut into parts).  Inputs A and B
    alternate on successive launches, eager and as replays of one captured graph, while a second stream keeps the
    memory system busy.  After every launch all 224 estimates and bitwidths must equal, bit for bit, those of a
    clean run of the same input, and the clean runs must match the oracle."""
    from concurrent.futures import ThreadPoolExecutor
    model, meta = synth.build_model(dp, synth.LLAMA_7B, 32, 8, [(3, 4)], 8, seed=777, keep_blocks=())
    shapes = meta["shapes"]
    n = len(shapes)
    ins = sorted(meta["xs_by_in"])
    xbuf = {in_: torch.zeros(in_, dtype=torch.float16, device="cuda") for in_ in ins}
    xs = [xbuf[in_] for _, in_ in shapes]
    ys = [torch.empty(out, dtype=torch.float16, device="cuda") for out, _ in shapes]
    k_dev = torch.zeros(n, dtype=torch.int32, device="cuda")
    e_dev = torch.zeros(n, dtype=torch.float32, device="cuda")
    sets = {"A": 2, "B": 5}

    def put(name):
        for in_ in ins:
            xbuf[in_].copy_(meta["xs_by_in"][in_][sets[name]])

    # clean runs: the same input twice in a row, nothing else on the GPU; checked against the oracle
    clean = {}
    sel = meta["sel"][(3, 4)]
    for name in sets:
        put(name)
        for _ in range(2):
            model.dpllm_decode_step_parts(xs, ys, k_dev, e_dev, dp.DPLLM_STEP_SELECT)
        torch.cuda.synchronize()
        clean[name] = (k_dev.clone(), e_dev.clone())
        x_np = {in_: synth.lut_np(meta["xs_by_in"][in_][sets[name]]) for in_ in ins}
        with ThreadPoolExecutor(max_workers=16) as pool:
            e_ref = list(pool.map(lambda i: oracle.estimate(synth.lut_np(sel[i]["G"]), x_np[shapes[i][1]]), range(n)))
        ks, es = k_dev.cpu().numpy(), e_dev.cpu().numpy()
        for i in range(n):
            assert abs(float(es[i]) - e_ref[i]) <= 3e-7 * e_ref[i], (name, i)
            assert int(ks[i]) == oracle.decide(e_ref[i], sel[i]["T"], 3, 4), (name, i)
    assert not torch.equal(clean["A"][1], clean["B"][1])
    # how far apart the two inputs' estimates are: a stale partial sum moves an estimate by about this much
    gap = ((clean["A"][1] - clean["B"][1]).abs() / clean["A"][1]).median().item()
    assert gap > 1e-3, gap

    other = torch.cuda.Stream()
    big = torch.ones(1 << 27, dtype=torch.int32, device="cuda")
    order = ["A", "B"] * 20
    for rep, name in enumerate(order):                       # eager launches, selectors and GEMVs
        with torch.cuda.stream(other):                       # unrelated traffic next to the step
            big.add_(1)
        put(name)
        model.dpllm_decode_step(xs, ys, k_dev, e_dev)
        torch.cuda.synchronize()
        assert torch.equal(k_dev, clean[name][0]), ("eager", rep, name)
        assert torch.equal(e_dev, clean[name][1]), ("eager", rep, name)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        model.dpllm_decode_step(xs, ys, k_dev, e_dev)
    for rep, name in enumerate(order):                       # replays of one graph, eager copies in between
        with torch.cuda.stream(other):
            big.add_(1)
        put(name)
        k_dev.zero_()
        e_dev.zero_()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(k_dev, clean[name][0]), ("graph", rep, name)
        assert torch.equal(e_dev, clean[name][1]), ("graph", rep, name)
    del big
    model.close()


@pytest.mark.parametrize("in_,r", [(4096, 64), (11008, 256), (1056, 17)])
def test_lone_selector_handover_alternating_inputs(dp, in_, r):
    """dpllm_estimate on one linear: few row groups, so the columns are cut into many chunks and every estimate is
    the sum of many parts' partial products.  Alternating inputs, every call against the oracle."""
    lin = synth.make_linear(4, in_, 4, 3, seed=in_ + r)
    model = dp.Model(1)
    model.dpllm_load_linear(0, synth.planes_np(lin["planes"]), {k: synth.lut_np(v) for k, v in lin["luts"].items()}, 3)
    g = torch.Generator().manual_seed(in_ * 7 + r)
    G = (torch.randn(r, in_, generator=g) / np.sqrt(r)).half()
    X = synth.make_x(in_, 2, seed=r)
    X[1] *= 3.0                                               # the two estimates differ by a factor of three
    e_ref = [oracle.estimate(synth.lut_np(G), synth.lut_np(x)) for x in X]
    T = 0.5 * (e_ref[0] + e_ref[1])
    model.dpllm_set_selector(0, 3, 4, dp.DPLLM_SEL_PROJ, G=G.cuda(), T=T)
    xd = [x.cuda() for x in X]
    for rep in range(30):
        which = rep & 1
        e, k = model.dpllm_estimate(0, 3, 4, xd[which])
        assert abs(float(e) - e_ref[which]) <= 3e-7 * e_ref[which], (rep, which)
        assert int(k) == oracle.decide(e_ref[which], T, 3, 4) == (3, 4)[which], (rep, which)
    model.close()


@pytest.mark.parametrize("out,in_", [(200, 3072), (64, 8192 + 32), (130, 2080), (1, 16384), (4096, 14336)])
def test_split_gemv_handover_alternating_inputs(dp, out, in_):
    """Launches with far fewer blocks of rows than compute units: several workgroups share a block of rows and the
    last one to finish adds up their partial sums.  Two different right-hand sides alternate on successive calls
    (single calls with one to three samples, and a decode-step launch of two linears); every call is compared
    with the oracle (norm-wise and row by row) and, bit for bit, with the first call on the same input."""
    lin = synth.make_linear(out, in_, 8, 3, seed=out + in_, device="cuda")
    other = synth.make_linear(96, in_, 8, 3, seed=out + in_ + 1, device="cuda")
    model = dp.Model(2)
    model.dpllm_load_linear(0, lin["planes"], lin["luts"], 3)
    model.dpllm_load_linear(1, other["planes"], other["luts"], 3)
    refs = [{"planes": synth.planes_np(l["planes"]), "luts": {k: synth.lut_np(v) for k, v in l["luts"].items()}}
            for l in (lin, other)]
    XA = synth.make_x(in_, 3, seed=31)
    XB = -2.0 * synth.make_x(in_, 3, seed=32)
    X = {"A": XA, "B": XB}

    def row_ok(got, y_ref, lut, x_bits):
        wmax = np.abs(lut.view(np.float16).astype(np.float64)).max(axis=1)
        xmax = float(np.abs(x_bits.view(np.float16).astype(np.float64)).max())
        tol = 2.0 ** -10 * np.abs(y_ref) + 2.0 * np.sqrt(in_) * 2.0 ** -24 * wmax * xmax + 2.0 ** -24
        return bool((np.abs(got - y_ref) <= tol).all())

    ks = (3, 4, 6, 8) if out * in_ < 1 << 24 else (3, 5)
    for k in ks:
        for B in (1, 2, 3):
            ref = {nm: oracle.gemv(refs[0]["planes"], k, refs[0]["luts"][k], synth.lut_np(X[nm][:B])) for nm in X}
            first = {}
            for rep in range(6):
                nm = "AB"[rep & 1]
                xb = (X[nm][:B] if B > 1 else X[nm][0]).cuda()
                got = model.dpllm_gemv(0, k, xb)
                torch.cuda.synchronize()
                if nm not in first:
                    first[nm] = got.clone()
                assert torch.equal(got, first[nm]), (k, B, rep)
                g = got.float().cpu().numpy().astype(np.float64).reshape(B, out)
                for b in range(B):
                    assert rel_l2(g[b], ref[nm][b]) <= REL_L2, (k, B, rep, b)
                    assert row_ok(g[b], ref[nm][b], refs[0]["luts"][k], synth.lut_np(X[nm][b])), (k, B, rep, b)
    # both linears in one launch of the decode step, inputs alternating
    xbuf = [torch.zeros(in_, dtype=torch.float16, device="cuda") for _ in range(2)]
    ys = [torch.empty(out, dtype=torch.float16, device="cuda"), torch.empty(96, dtype=torch.float16, device="cuda")]
    k_dev = torch.zeros(2, dtype=torch.int32, device="cuda")
    e_dev = torch.zeros(2, dtype=torch.float32, device="cuda")
    for k in (3, 6):
        for i in range(2):
            model.dpllm_set_selector(i, k, k, dp.DPLLM_SEL_NONE)
        for rep in range(6):
            nm = "AB"[rep & 1]
            for i in range(2):
                xbuf[i].copy_(X[nm][i])
            model.dpllm_decode_step(xbuf, ys, k_dev, e_dev)
            torch.cuda.synchronize()
            for i in range(2):
                y_ref = oracle.gemv(refs[i]["planes"], k, refs[i]["luts"][k], synth.lut_np(X[nm][i]))
                g = ys[i].float().cpu().numpy().astype(np.float64)
                assert rel_l2(g, y_ref) <= REL_L2, (k, rep, i)
                assert row_ok(g, y_ref, refs[i]["luts"][k], synth.lut_np(X[nm][i])), (k, rep, i)
    model.close()
