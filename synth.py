"""Seeded synthetic inputs shared by the tests, the smoke check and the bench.

This module only *makes inputs*: quantised linears in the canonical host layout,
activation vectors, projection matrices G and thresholds.  It implements none
of the hot path (no bitplane unpack, no GEMV, no selector) and is imported by
neither the oracle nor the GPU library; both consume the arrays it returns.
(build_model hands the generated arrays to a binding module it is given; it calls
only that module's load and set_selector.)

Recipe (shapes of Llama-class linears; stands in for trained weights and real
activations, which are not available here):
  * weights   w = fp16(z * s_row), z ~ N(0,1), s_row ~ lognormal(0, 0.5)
  * centroids c_j = fp16(Phi^-1((j + 1/2) / 2^p) * s_row), j < 2^p  (Gaussian quantiles)
  * parent code of a weight = index of its nearest centroid (ties -> lower index)
  * child table LUT_k[j] = fp16(mean of the 2^(p-k) parent centroids with prefix j)
  * planes: uint32 [p][out][in/32], plane 0 = most significant code bit,
    column c = bit (c % 32) of word c // 32
  * activations x = fp16 N(0,1) with a fixed 1 % of channels scaled by 20
  * G = fp16(A (W_h - W_l)), A ~ N(0,1)/sqrt(r)  (projection of Sec. 5.1 of the paper)
  * thresholds: tau ~ U[0.05, 0.3] times the median of ||W_h x_t|| over the
    synthetic activations, moved out of the tie guard band of every estimate
Everything runs in torch on the device asked for ("cpu" here, "cuda" for the
full-model configurations whose generation would take too long on the host).
"""
import math

import numpy as np
import torch


def _gen(seed, device):
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def pack_planes(idx_p: torch.Tensor, p: int) -> torch.Tensor:
    """codes uint8 [out][in] -> planes int32 (bit pattern of uint32) [p][out][in/32]."""
    out, in_ = idx_p.shape
    assert in_ % 32 == 0
    weights = (torch.ones(32, dtype=torch.int64, device=idx_p.device) << torch.arange(32, device=idx_p.device))
    planes = torch.empty((p, out, in_ // 32), dtype=torch.int32, device=idx_p.device)
    for b in range(p):
        bits = ((idx_p >> (p - 1 - b)) & 1).to(torch.int64).reshape(out, in_ // 32, 32)
        words = (bits * weights).sum(dim=-1)
        planes[b] = torch.where(words >= 2 ** 31, words - 2 ** 32, words).to(torch.int32)
    return planes


def make_linear(out: int, in_: int, p: int, kmin: int, seed: int, device="cpu", keep_codes=True):
    """One quantised linear.  Returns a dict of torch tensors on `device`:
    planes int32 [p][out][in/32], luts {k: fp16 [out][2^k]}, codes uint8 [out][in] (optional)."""
    g = _gen(seed, device)
    s = torch.exp(0.5 * torch.randn(out, generator=g, device=device, dtype=torch.float64))
    z = torch.randn(out, in_, generator=g, device=device, dtype=torch.float32)
    w16 = (z * s[:, None].float()).half()
    del z
    n = 1 << p
    q = torch.special.ndtri((torch.arange(n, device=device, dtype=torch.float64) + 0.5) / n)
    cent = (q[None, :] * s[:, None]).half()                      # [out][2^p], non-decreasing
    mid = (cent[:, :-1].double() + cent[:, 1:].double()) * 0.5   # exact midpoints
    codes = torch.empty((out, in_), dtype=torch.uint8, device=device)
    step = max(1, (1 << 24) // in_)
    for r0 in range(0, out, step):
        r1 = min(out, r0 + step)
        # number of midpoints strictly below w  == nearest centroid, ties to the lower index
        codes[r0:r1] = torch.searchsorted(mid[r0:r1].contiguous(), w16[r0:r1].double().contiguous(),
                                          right=False).to(torch.uint8)
    luts = {p: cent}
    for k in range(kmin, p):
        luts[k] = cent.double().reshape(out, 1 << k, 1 << (p - k)).mean(dim=-1).half()
    lin = {"out": out, "in": in_, "p": p, "kmin": kmin, "planes": pack_planes(codes, p), "luts": luts}
    if keep_codes:
        lin["codes"] = codes
        lin["w16"] = w16
    return lin


def dense_weight(lin, k: int, dtype=torch.float32) -> torch.Tensor:
    """Harness-side dense W_k from the generator's own codes (used to build G and thresholds)."""
    codes = lin["codes"]
    idx = (codes >> (lin["p"] - k)).long()
    return torch.gather(lin["luts"][k].to(dtype), 1, idx)


def outlier_channels(in_: int, seed: int, frac=0.01) -> torch.Tensor:
    g = _gen(seed, "cpu")
    n = max(1, int(round(in_ * frac)))
    return torch.randperm(in_, generator=g)[:n].sort().values


def make_x(in_: int, n: int, seed: int, device="cpu", outliers=True, channel_seed=None) -> torch.Tensor:
    """n activation vectors fp16 [n][in]; the outlier channel set depends only on (in, channel_seed)."""
    g = _gen(seed, device)
    x = torch.randn(n, in_, generator=g, device=device, dtype=torch.float32)
    if outliers:
        ch = outlier_channels(in_, 1000003 * in_ + 17 if channel_seed is None else channel_seed).to(device)
        x[:, ch] *= 20.0
    return x.half()


def make_A(r: int, out: int, seed: int, device="cpu") -> torch.Tensor:
    g = _gen(seed, device)
    return torch.randn(r, out, generator=g, device=device, dtype=torch.float32) / math.sqrt(r)


def make_G(lin, l: int, h: int, r: int, seed: int, A=None) -> torch.Tensor:
    """G = fp16(A (W_h - W_l)), fp16 [r][in]."""
    dev = lin["planes"].device
    if A is None:
        A = make_A(r, lin["out"], seed, dev)
    dW = dense_weight(lin, h) - dense_weight(lin, l)
    return (A.to(dev) @ dW).half()


def thresholds_from_tau(lin, h: int, xs: torch.Tensor, tau: float) -> float:
    """T = tau * median_t ||W_h x_t||_2 over the synthetic activations."""
    Wh = dense_weight(lin, h)
    norms = (xs.float() @ Wh.T).double().norm(dim=1)
    return float(tau * norms.median())


def estimates_fp64(G: torch.Tensor, xs: torch.Tensor) -> torch.Tensor:
    """Calibration-side ||G x_t|| for every activation (used only to place thresholds)."""
    return (xs.double() @ G.double().T).norm(dim=1)


def nudge_threshold(T: float, est: torch.Tensor, band=1e-6) -> float:
    """Move T out of the relative band around every calibration estimate, to the middle of the
    neighbouring gap, so that no decision rests on the last bits of a sum."""
    e = np.sort(est.detach().cpu().numpy().astype(np.float64))
    if not np.isfinite(T):
        return T
    T32 = float(np.float32(T))
    close = np.abs(e - T32) <= band * np.maximum(np.abs(T32), e)
    if not close.any():
        return T32
    i = int(np.searchsorted(e, T32))
    lo = e[i - 1] if i > 0 else e[0] * 0.5
    hi = e[i] if i < len(e) else e[-1] * 1.5
    for cand in (0.5 * (lo + hi), 0.5 * (e[max(i - 2, 0)] + lo), 0.5 * (hi + e[min(i + 1, len(e) - 1)])):
        c32 = float(np.float32(cand))
        if not (np.abs(e - c32) <= band * np.maximum(np.abs(c32), e)).any():
            return c32
    raise RuntimeError("no threshold outside the guard band near %g" % T)


def quantile_threshold(est: torch.Tensor, rho: float) -> float:
    """rho-quantile of the calibration estimates (Phase 3 of Algorithm 1 of the paper)."""
    return float(np.quantile(est.detach().cpu().numpy().astype(np.float64), rho))


LLAMA_7B = [("q", 4096, 4096), ("k", 4096, 4096), ("v", 4096, 4096), ("o", 4096, 4096),
            ("gate", 11008, 4096), ("up", 11008, 4096), ("down", 4096, 11008)]
LLAMA3_8B = [("q", 4096, 4096), ("k", 1024, 4096), ("v", 1024, 4096), ("o", 4096, 4096),
             ("gate", 14336, 4096), ("up", 14336, 4096), ("down", 4096, 14336)]
LLAMA_70B = [("q", 8192, 8192), ("k", 1024, 8192), ("v", 1024, 8192), ("o", 8192, 8192),
             ("gate", 28672, 8192), ("up", 28672, 8192), ("down", 8192, 28672)]


def fit_linreg(xs: torch.Tensor, est: torch.Tensor):
    """Least-squares (alpha, beta) of est ~ alpha * ||x||_2 + beta over the calibration activations: the
    linear-regression estimator's constants (Sec. 5.1 of the paper), as fp32 values."""
    nx = xs.double().norm(dim=1).cpu().numpy()
    e = est.detach().cpu().numpy().astype(np.float64)
    A = np.stack([nx, np.ones_like(nx)], axis=1)
    (alpha, beta), *_ = np.linalg.lstsq(A, e, rcond=None)
    return float(np.float32(alpha)), float(np.float32(beta))


def linreg_estimates_fp64(xs: torch.Tensor, alpha: float, beta: float) -> torch.Tensor:
    """Calibration-side alpha * ||x_t|| + beta (used only to place thresholds)."""
    return alpha * xs.double().norm(dim=1) + beta


def build_model(dp, shapes, n_blocks, p, pairs, n_x, seed=1234, keep_blocks=(0,), log=None, quantile=None, rank=64,
                linreg_every=0, kmin=3):
    """Harness helper: loads n_blocks x len(shapes) linears generated on the GPU into a model of the binding `dp`
    and attaches, for every candidate pair of `pairs` ((l, h) tuples; the first one is left in use), one selector
    per linear.  Thresholds: tau ~ U[0.05, 0.3] times the median of ||W_h x|| (default), or the `quantile` of the
    calibration estimates (Phase 3 of Algorithm 1).  linreg_every = m > 0: the linears with index % m == m - 1 take
    the linear-regression estimator (constants fitted to the calibration estimates), the others the projection.  Returns (model, meta); meta carries shapes, the activation
    sets, per pair the selector constants and calibration estimates, and host copies of the linears of
    `keep_blocks` for the oracle."""
    import time
    n = n_blocks * len(shapes)
    model = dp.Model(n)
    ins = sorted({in_ for _, _, in_ in shapes})
    xs_by_in = {in_: make_x(in_, n_x, seed=seed + in_, device="cuda") for in_ in ins}
    rng = np.random.default_rng(seed)
    taus = rng.uniform(0.05, 0.3, size=n)
    meta = {"shapes": [], "xs_by_in": xs_by_in, "host": {}, "pairs": list(pairs),
            "sel": {pr: [] for pr in pairs}}      # sel[(l,h)][i] = dict(kind, G, alpha, beta, T, est)
    t0 = time.time()
    for b in range(n_blocks):
        for j, (name, out, in_) in enumerate(shapes):
            i = b * len(shapes) + j
            lin = make_linear(out, in_, p, kmin, seed=seed + 7919 * i, device="cuda", keep_codes=True)
            model.dpllm_load_linear(i, lin["planes"], lin["luts"], kmin)
            xs = xs_by_in[in_]
            for pi, (l, h) in reversed(list(enumerate(pairs))):      # the first pair is attached last: it stays in use
                G = make_G(lin, l, h, rank, seed=seed + 104729 * i + 1 + pi)
                est = estimates_fp64(G, xs)
                kind, alpha, beta = 1, 0.0, 0.0
                if linreg_every and i % linreg_every == linreg_every - 1:
                    kind = 2
                    alpha, beta = fit_linreg(xs, est)
                    est = linreg_estimates_fp64(xs, alpha, beta)
                    G = None
                if quantile is None:
                    T = thresholds_from_tau(lin, h, xs, float(taus[i]))
                    if kind == 2:       # the fitted line is nearly flat on these activations: split its range
                        T = float(est.median())
                else:   # Phase-3 style: the rho-quantile of the calibration estimates
                    T = quantile_threshold(est, quantile)
                T = nudge_threshold(T, est, band=1e-6)
                model.dpllm_set_selector(i, l, h, kind, G=G, alpha=alpha, beta=beta, T=T)
                meta["sel"][(l, h)].append(None)
                meta["sel"][(l, h)][-1] = {"kind": kind, "G": G, "alpha": alpha, "beta": beta, "T": T, "est": est}
            meta["shapes"].append((out, in_))
            if b in keep_blocks:
                meta["host"][i] = {"planes": planes_np(lin["planes"]),
                                   "luts": {k: lut_np(v) for k, v in lin["luts"].items()}}
            del lin
        if log and (b % 8 == 7 or b == n_blocks - 1):
            log("built block %d/%d (%.0f s)" % (b + 1, n_blocks, time.time() - t0))
    return model, meta


def oracle_selector(meta, pair, i, T=None):
    """The selector dict the oracle's decode_step takes, for linear i under candidate pair `pair`."""
    s = meta["sel"][pair][i]
    d = {"l": pair[0], "h": pair[1], "kind": s["kind"], "alpha": s["alpha"], "beta": s["beta"],
         "T": s["T"] if T is None else T}
    if s["G"] is not None:
        d["G"] = lut_np(s["G"])
    return d


def to_np(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().contiguous().numpy()


def planes_np(planes: torch.Tensor) -> np.ndarray:
    """int32 plane tensor -> the canonical uint32 host array."""
    return to_np(planes).view(np.uint32)


def lut_np(lut: torch.Tensor) -> np.ndarray:
    """fp16 tensor -> uint16 bit patterns."""
    return to_np(lut).view(np.uint16)
