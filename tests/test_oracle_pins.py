"""Pins for the CPU oracle: every oracle function is checked here against something
other than itself — a library routine, a closed form, brute force written out in the
test, a hand-worked fixture, or a figure the paper prints.  No GPU, no GPU library."""
import math
import os

import numpy as np
import pytest
import torch

import oracle
import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def read_kv(name):
    d = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                key, val = line.split()
                d[key] = val
    return d


# ----------------------------------------------------------------------------- helpers
def brute_pack(codes, p):
    """Definition of the canonical layout, one bit at a time (test-local, pure Python)."""
    out, in_ = codes.shape
    planes = np.zeros((p, out, in_ // 32), dtype=np.uint32)
    for o in range(out):
        for c in range(in_):
            for b in range(p):
                bit = (int(codes[o, c]) >> (p - 1 - b)) & 1
                if bit:
                    planes[b, o, c // 32] |= np.uint32(1 << (c % 32))
    return planes


def brute_dense(planes, p, k, lut_k):
    """W_k built weight by weight from the planes, as numpy float64."""
    _, out, nw = planes.shape
    W = np.zeros((out, nw * 32))
    for o in range(out):
        for c in range(nw * 32):
            code = 0
            for b in range(p):
                code = (code << 1) | ((int(planes[b, o, c // 32]) >> (c % 32)) & 1)
            W[o, c] = float(lut_k[o, code >> (p - k)])
    return W


def random_lut(rng, out, k):
    return (rng.standard_normal((out, 1 << k)) * 0.7).astype(np.float16)


# ----------------------------------------------------------------------------- P0 fp16
def test_half_to_double_all_patterns():
    bits = np.arange(65536, dtype=np.uint16)
    ref = bits.view(np.float16).astype(np.float64)
    got = np.array([oracle.half_to_double(int(b)) for b in bits])
    nan = np.isnan(ref)
    assert (np.isnan(got) == nan).all()
    assert (got[~nan] == ref[~nan]).all()
    assert math.copysign(1.0, oracle.half_to_double(0x8000)) == -1.0


# ----------------------------------------------------------------------------- P1 unpack
def test_unpack_hand_worked_fixture():
    g = read_kv("bitplane_example.txt")
    p, out, in_ = int(g["p"]), int(g["out"]), int(g["in"])
    planes = np.array([[[int(g["plane%d" % b], 16)]] for b in range(p)], dtype=np.uint32)
    assert planes.shape == (p, out, in_ // 32)
    codes = oracle.unpack(planes)
    assert codes.tolist() == [[c % 8 for c in range(32)]]
    assert oracle.index_k(codes, 3, 2).tolist() == [[(c % 8) >> 1 for c in range(32)]]


@pytest.mark.parametrize("p", range(1, 9))
def test_unpack_round_trip(p):
    rng = np.random.default_rng(100 + p)
    for out, in_ in [(1, 32), (3, 64), (5, 96), (2, 160)]:
        codes = rng.integers(0, 1 << p, size=(out, in_), dtype=np.uint8)
        planes = brute_pack(codes, p)
        assert (oracle.unpack(planes) == codes).all()


def test_unpack_single_bit_probe():
    """One set bit at (plane b, row o, column c) must give code 1 << (p-1-b) at (o, c) only."""
    p, out, in_ = 5, 3, 96
    for b, o, c in [(0, 0, 0), (4, 2, 95), (2, 1, 31), (1, 2, 32), (3, 0, 63)]:
        planes = np.zeros((p, out, in_ // 32), dtype=np.uint32)
        planes[b, o, c // 32] = np.uint32(1 << (c % 32))
        codes = oracle.unpack(planes)
        expect = np.zeros((out, in_), dtype=np.uint8)
        expect[o, c] = 1 << (p - 1 - b)
        assert (codes == expect).all()


def test_generator_pack_matches_brute_pack():
    lin = synth.make_linear(7, 96, 5, 3, seed=3)
    codes = synth.to_np(lin["codes"])
    assert (synth.planes_np(lin["planes"]) == brute_pack(codes, 5)).all()


# ----------------------------------------------------------------------------- P2 prefix
def test_prefix_property():
    rng = np.random.default_rng(7)
    for p in range(1, 9):
        codes = rng.integers(0, 1 << p, size=(4, 64), dtype=np.uint8)
        prev = codes
        assert (oracle.index_k(codes, p, p) == codes).all()
        for k in range(p - 1, 0, -1):
            ik = oracle.index_k(codes, p, k)
            assert (ik == codes >> (p - k)).all()
            assert (ik == prev >> 1).all()
            prev = ik


# ----------------------------------------------------------------------------- P3 generator + dequant
def test_generator_lut_consistency_and_nearest_centroid():
    p, kmin = 6, 3
    lin = synth.make_linear(16, 128, p, kmin, seed=11)
    luts = {k: synth.to_np(v).astype(np.float64) for k, v in lin["luts"].items()}
    for k in range(kmin, p):
        child_mean = 0.5 * (luts[k + 1][:, 0::2] + luts[k + 1][:, 1::2])
        ulp = np.spacing(np.abs(luts[k]).astype(np.float16)).astype(np.float64)
        assert (np.abs(luts[k] - child_mean) <= ulp).all()
    w = synth.to_np(lin["w16"]).astype(np.float64)
    codes = synth.to_np(lin["codes"])
    cent = luts[p]
    for o in range(16):
        d = np.abs(w[o][:, None] - cent[o][None, :])
        assert (np.argmin(d, axis=1) == codes[o]).all()      # argmin returns the lowest index on ties
    planes = synth.planes_np(lin["planes"])
    idx_p = oracle.unpack(planes)
    errs = []
    for k in range(kmin, p + 1):
        Wk = oracle.dequant(oracle.index_k(idx_p, p, k), synth.lut_np(lin["luts"][k]), k)
        errs.append(np.linalg.norm(w - Wk))
    assert all(errs[i + 1] <= errs[i] * (1 + 1e-12) for i in range(len(errs) - 1)), errs


def test_dequant_is_table_lookup():
    rng = np.random.default_rng(5)
    k, out, in_ = 3, 4, 64
    idx = rng.integers(0, 1 << k, size=(out, in_), dtype=np.uint8)
    lut = random_lut(rng, out, k)
    W = oracle.dequant(idx, lut.view(np.uint16), k)
    for o in range(out):
        for c in range(in_):
            assert W[o, c] == float(lut[o, idx[o, c]])


# ----------------------------------------------------------------------------- P4 brute-force GEMV
@pytest.mark.parametrize("out,in_,p", [(2, 32, 4), (7, 64, 8), (33, 96, 5), (5, 160, 3)])
def test_gemv_brute_force_tiny(out, in_, p):
    rng = np.random.default_rng(out * 1000 + in_)
    codes = rng.integers(0, 1 << p, size=(out, in_), dtype=np.uint8)
    planes = brute_pack(codes, p)
    x = rng.standard_normal(in_).astype(np.float16)
    for k in range(max(1, p - 3), p + 1):
        lut = random_lut(rng, out, k)
        W = brute_dense(planes, p, k, lut)
        ref = W @ x.astype(np.float64)
        got = oracle.gemv(planes, k, lut.view(np.uint16), x.view(np.uint16))
        assert np.allclose(got, ref, rtol=1e-12, atol=1e-12)


def test_gemv_batch_is_per_sample():
    rng = np.random.default_rng(9)
    p, k, out, in_ = 5, 4, 6, 64
    codes = rng.integers(0, 1 << p, size=(out, in_), dtype=np.uint8)
    planes = brute_pack(codes, p)
    lut = random_lut(rng, out, k)
    X = rng.standard_normal((3, in_)).astype(np.float16)
    Y = oracle.gemv(planes, k, lut.view(np.uint16), X.view(np.uint16))
    assert Y.shape == (3, out)
    for b in range(3):
        assert (Y[b] == oracle.gemv(planes, k, lut.view(np.uint16), X[b].view(np.uint16))).all()
    W = brute_dense(planes, p, k, lut)
    assert np.allclose(Y, X.astype(np.float64) @ W.T, rtol=1e-12, atol=1e-12)


def test_gemv_config0_against_generator_dense():
    """1024 x 1024, p = 4, k in {3, 4}: the dense W_k comes from the generator's own codes
    (never unpacked from planes) and numpy's fp64 matmul."""
    lin = synth.make_linear(1024, 1024, 4, 3, seed=0)
    x = synth.make_x(1024, 1, seed=0, outliers=False)[0]
    planes = synth.planes_np(lin["planes"])
    for k in (3, 4):
        W = synth.to_np(synth.dense_weight(lin, k, torch.float64))
        ref = W @ synth.to_np(x).astype(np.float64)
        got = oracle.gemv(planes, k, synth.lut_np(lin["luts"][k]), synth.lut_np(x))
        assert np.linalg.norm(got - ref) <= 1e-12 * np.linalg.norm(ref)


# ----------------------------------------------------------------------------- P5 special cases
def test_gemv_special_cases():
    rng = np.random.default_rng(21)
    p, out, in_ = 6, 5, 96
    x = rng.standard_normal(in_).astype(np.float16)
    xs = x.astype(np.float64).sum()
    # all codes zero: y[o] = LUT[o][0] * sum(x)
    planes = np.zeros((p, out, in_ // 32), dtype=np.uint32)
    for k in (3, 6):
        lut = random_lut(rng, out, k)
        y = oracle.gemv(planes, k, lut.view(np.uint16), x.view(np.uint16))
        assert np.allclose(y, lut[:, 0].astype(np.float64) * xs, rtol=1e-12)
    # x = e_c picks column c of W_k
    codes = rng.integers(0, 1 << p, size=(out, in_), dtype=np.uint8)
    planes = brute_pack(codes, p)
    k = 4
    lut = random_lut(rng, out, k)
    for c in (0, 31, 32, 95):
        e = np.zeros(in_, dtype=np.float16)
        e[c] = 1.0
        y = oracle.gemv(planes, k, lut.view(np.uint16), e.view(np.uint16))
        assert (y == lut[np.arange(out), codes[:, c] >> (p - k)].astype(np.float64)).all()
    # k = p with a linear-ramp table reduces to a uniform-quantised GEMV: a * (codes @ x) + b * sum(x)
    a, b = 0.125, -2.0
    ramp = (a * np.arange(1 << p) + b).astype(np.float16)
    assert (ramp.astype(np.float64) == a * np.arange(1 << p) + b).all()
    lut = np.tile(ramp, (out, 1))
    y = oracle.gemv(planes, p, lut.view(np.uint16), x.view(np.uint16))
    ref = a * (codes.astype(np.float64) @ x.astype(np.float64)) + b * xs
    assert np.allclose(y, ref, rtol=1e-12, atol=1e-12)


def test_gemv_row_and_column_orientation():
    """A transposed operand or swapped row/column stride must fail here: out != in and
    each row has its own table."""
    p = k = 2
    out, in_ = 3, 64
    codes = np.zeros((out, in_), dtype=np.uint8)
    codes[1, 5] = 3
    codes[2, 40] = 2
    planes = brute_pack(codes, p)
    lut = np.zeros((out, 4), dtype=np.float16)
    lut[1, 3] = 2.0
    lut[2, 2] = -4.0
    lut[0, 3] = 100.0          # never selected: row 0 holds code 0 only
    x = np.zeros(in_, dtype=np.float16)
    x[5] = 3.0
    x[40] = 0.5
    y = oracle.gemv(planes, k, lut.view(np.uint16), x.view(np.uint16))
    assert y.tolist() == [0.0, 6.0, -2.0]


# ----------------------------------------------------------------------------- P6 closed forms
def test_g_memory_closed_form_matches_paper():
    g = read_kv("paper_constants.txt")
    r = int(g["projection_rank"])
    # Phi-3-Medium: 40 blocks, fused qkv / o / fused gate-up read 5120 channels, down reads 17920
    ins = [5120, 5120, 5120, 17920]
    assert 40 * len(ins) == int(g["phi3_medium_selectors"])
    total = sum(r * in_ * 2 for in_ in ins) * 40          # fp16 G of shape [r][in] per linear
    assert round(total / 1e9, 2) == float(g["g_bytes_per_pair_gb"])
    assert round(3 * total / 1e9, 2) == float(g["g_bytes_three_pairs_gb"])
    assert 32 * len(synth.LLAMA3_8B) == int(g["llama3_8b_selectors"])
    G = synth.make_G(synth.make_linear(8, 64, 4, 3, seed=1), 3, 4, r, seed=2)
    assert tuple(G.shape) == (r, 64) and G.element_size() == 2


# ----------------------------------------------------------------------------- O5 exact error
def test_exact_err_against_dense_difference():
    lin = synth.make_linear(24, 96, 6, 3, seed=31)
    planes = synth.planes_np(lin["planes"])
    x = synth.make_x(96, 1, seed=32)[0]
    xd = synth.to_np(x).astype(np.float64)
    for l, h in [(3, 4), (4, 5), (3, 6)]:
        Wl = brute_dense(planes, 6, l, synth.to_np(lin["luts"][l]))
        Wh = brute_dense(planes, 6, h, synth.to_np(lin["luts"][h]))
        e, nh = oracle.exact_err(planes, l, h, synth.lut_np(lin["luts"][l]), synth.lut_np(lin["luts"][h]),
                                 synth.lut_np(x))
        assert math.isclose(e, np.linalg.norm((Wh - Wl) @ xd), rel_tol=1e-12)
        assert math.isclose(nh, np.linalg.norm(Wh @ xd), rel_tol=1e-12)
    e, _ = oracle.exact_err(planes, 4, 4, synth.lut_np(lin["luts"][4]), synth.lut_np(lin["luts"][4]),
                            synth.lut_np(x))
    assert e == 0.0                                         # l == h: the difference vanishes


# ----------------------------------------------------------------------------- P7 estimator
def test_estimate_is_norm_of_matvec():
    rng = np.random.default_rng(41)
    G = rng.standard_normal((64, 96)).astype(np.float16)
    x = rng.standard_normal(96).astype(np.float16)
    e, g = oracle.estimate(G.view(np.uint16), x.view(np.uint16), return_g=True)
    ref = G.astype(np.float64) @ x.astype(np.float64)
    assert np.allclose(g, ref, rtol=1e-13, atol=1e-13)
    assert math.isclose(e, np.linalg.norm(ref), rel_tol=1e-13)
    # a non-square G with one non-zero entry fixes the orientation
    G = np.zeros((3, 64), dtype=np.float16)
    G[2, 7] = 2.0
    x = np.zeros(64, dtype=np.float16)
    x[7] = -3.0
    e, g = oracle.estimate(G.view(np.uint16), x.view(np.uint16), return_g=True)
    assert g.tolist() == [0.0, 0.0, -6.0] and e == 6.0


def _ratio_samples(lin, l, h, r, n_draws, seed):
    """e^/e* over fresh Gaussian projections A and fresh activations."""
    planes = synth.planes_np(lin["planes"])
    ll, lh = synth.lut_np(lin["luts"][l]), synth.lut_np(lin["luts"][h])
    dW = (synth.dense_weight(lin, h) - synth.dense_weight(lin, l)) * 64.0   # keep fp16(G) well scaled
    xs = synth.make_x(lin["in"], n_draws, seed=seed)
    gA = torch.Generator().manual_seed(seed + 1)
    ratios = np.empty(n_draws)
    for t in range(n_draws):
        A = torch.randn(r, lin["out"], generator=gA) / math.sqrt(r)
        G = (A @ dW).half()
        e_hat = oracle.estimate(synth.lut_np(G), synth.lut_np(xs[t])) / 64.0
        e_star, _ = oracle.exact_err(planes, l, h, ll, lh, synth.lut_np(xs[t]))
        ratios[t] = e_hat / e_star
    return ratios


def test_jl_statistics_rank64_match_paper():
    g = read_kv("paper_constants.txt")
    r = int(g["projection_rank"])
    lin = synth.make_linear(96, 64, 4, 3, seed=51)
    ratios = _ratio_samples(lin, 3, 4, r, 12000, seed=52)
    assert abs(np.mean(ratios ** 2) - 1.0) < 0.01                      # E||Az||^2 = ||z||^2
    assert abs(np.std(ratios) - 1.0 / math.sqrt(2 * r)) < 0.004        # chi_r / sqrt(r)
    inside = np.mean(np.abs(ratios - 1.0) < float(g["jl_tolerance"]))
    assert abs(inside - float(g["jl_confidence"])) <= 0.01, inside


def test_estimator_converges_as_rank_grows():
    lin = synth.make_linear(96, 64, 4, 3, seed=61)
    spreads = []
    for r in (16, 64, 256, 1024):
        ratios = _ratio_samples(lin, 3, 4, r, 1500, seed=62 + r)
        spreads.append(np.std(ratios))
        assert abs(spreads[-1] * math.sqrt(2 * r) - 1.0) < 0.12, (r, spreads[-1])
    assert spreads == sorted(spreads, reverse=True)


def test_orthonormal_full_rank_projection_is_exact():
    lin = synth.make_linear(64, 96, 5, 3, seed=71)
    out = lin["out"]
    Q, _ = torch.linalg.qr(torch.randn(out, out, dtype=torch.float64, generator=torch.Generator().manual_seed(72)))
    dW = (synth.dense_weight(lin, 5, torch.float64) - synth.dense_weight(lin, 4, torch.float64)) * 64.0
    G = (Q @ dW).half()
    x = synth.make_x(96, 1, seed=73)[0]
    e_hat = oracle.estimate(synth.lut_np(G), synth.lut_np(x)) / 64.0
    e_star, _ = oracle.exact_err(synth.planes_np(lin["planes"]), 4, 5, synth.lut_np(lin["luts"][4]),
                                 synth.lut_np(lin["luts"][5]), synth.lut_np(x))
    assert abs(e_hat / e_star - 1.0) < 2e-3                             # only fp16 rounding of G remains


def test_linreg_estimate():
    x = np.array([3.0, -4.0] + [0.0] * 30, dtype=np.float16)
    assert oracle.linreg_estimate(x.view(np.uint16), 0.5, 0.25) == 0.5 * 5.0 + 0.25


# ----------------------------------------------------------------------------- P8 decisions
def test_decide_rule_and_degenerate_thresholds():
    assert oracle.decide(1.0, 0.5, 3, 4) == 4            # exceeds -> h
    assert oracle.decide(0.25, 0.5, 3, 4) == 3           # below -> l
    assert oracle.decide(0.5, 0.5, 3, 4) == 3            # equality does not exceed
    assert oracle.decide(1e30, float("inf"), 3, 4) == 3  # +inf pins l
    assert oracle.decide(0.0, float("-inf"), 3, 4) == 4  # -inf pins h
    assert oracle.decide(0.0, -1.0, 5, 6) == 6           # negative T: a norm always exceeds it
    t32 = float(np.float32(0.1))
    assert oracle.decide(np.nextafter(t32, 1.0), 0.1, 3, 4) == 4       # compared at double precision
    assert oracle.decide(t32, 0.1, 3, 4) == 3


def _tiny_model(T_of):
    lins, xs = [], []
    for i, (out, in_) in enumerate([(8, 64), (12, 64), (8, 96)]):
        lin = synth.make_linear(out, in_, 5, 3, seed=80 + i)
        G = synth.make_G(lin, 3, 4, 16, seed=90 + i)
        x = synth.make_x(in_, 1, seed=95 + i)[0]
        e = oracle.estimate(synth.lut_np(G), synth.lut_np(x))
        lins.append({"planes": synth.planes_np(lin["planes"]),
                     "luts": {k: synth.lut_np(v) for k, v in lin["luts"].items()},
                     "selector": {"l": 3, "h": 4, "kind": 1, "G": synth.lut_np(G), "T": T_of(i, e)}})
        xs.append(synth.lut_np(x))
    return lins, xs


def test_decode_step_degenerate_and_mixed():
    for T, kk in [(float("inf"), 3), (float("-inf"), 4)]:
        lins, xs = _tiny_model(lambda i, e: T)
        ys, ks, es = oracle.decode_step(lins, xs)
        assert ks.tolist() == [kk] * 3
        for lin, x, y in zip(lins, xs, ys):
            assert (y == oracle.gemv(lin["planes"], kk, lin["luts"][kk], x)).all()
    lins, xs = _tiny_model(lambda i, e: e * (0.9 if i == 1 else 1.1))
    ys, ks, es = oracle.decode_step(lins, xs)
    assert ks.tolist() == [3, 4, 3]
    sizes = [8 * 64, 12 * 64, 8 * 96]
    assert math.isclose(oracle.effective_bits(ks, sizes), (3 * 512 + 4 * 768 + 3 * 768) / 2048.0)


def test_decode_step_selector_input_moves_the_decision_not_the_product():
    """Sec. 5.2: with a selector input the estimate is ||G x_sel|| (numpy matvec), the output is still W_k x."""
    lins, xs = _tiny_model(lambda i, e: e)          # T = the estimate on the immediate input: selects l (not >)
    assert oracle.decode_step(lins, xs)[1].tolist() == [3, 3, 3]
    x_big = [(np.asarray(x).view(np.float16).astype(np.float32) * 2).astype(np.float16).view(np.uint16) for x in xs]
    xs_sel = [None, x_big[1], None]
    ys, ks, es = oracle.decode_step(lins, xs, xs_sel)
    assert ks.tolist() == [3, 4, 3]                 # doubling the selector input doubles the estimate
    G = lins[1]["selector"]["G"].view(np.float16).astype(np.float64)
    want = np.linalg.norm(G @ x_big[1].view(np.float16).astype(np.float64))
    assert math.isclose(es[1], want, rel_tol=1e-12)
    assert (ys[1] == oracle.gemv(lins[1]["planes"], 4, lins[1]["luts"][4], xs[1])).all()
    same = oracle.decode_step(lins, xs, [None, None, None])
    assert same[1].tolist() == [3, 3, 3]


# ----------------------------------------------------------------------------- P9 quantile calibration
def test_quantile_threshold_realises_target_bits():
    lin = synth.make_linear(64, 128, 5, 3, seed=101)
    G = synth.make_G(lin, 3, 4, 64, seed=102)
    xs = synth.make_x(128, 256, seed=103)
    est = synth.estimates_fp64(G, xs)
    for target in (3.25, 3.5, 3.75):
        rho = 1.0 - (target - 3)                         # fraction of inputs that should take l
        T = synth.nudge_threshold(synth.quantile_threshold(est, rho), est)
        ks = [oracle.decide(oracle.estimate(synth.lut_np(G), synth.lut_np(x)), T, 3, 4) for x in xs]
        frac_l = ks.count(3) / len(ks)
        assert abs(frac_l - rho) <= 1.0 / 256 + 1e-12
        assert abs(np.mean(ks) - target) <= 0.01
