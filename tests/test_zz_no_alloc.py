"""The entry point that allocates nothing (dpllm_estimate_noalloc: partial results travel through a fixed array in
the library's device image) against the entry point it is a variant of (dpllm_estimate: through the model's
workspace), called through the C boundary.  Two calls in a row, the second on a smaller input (fewer columns,
lower rank: it leaves most of what the first call wrote in the array untouched), then the other estimator kinds."""
import math

import pytest
import torch

import synth

pytestmark = pytest.mark.gpu


def test_estimate_noalloc_matches_estimate_two_calls_in_a_row():
    import paper_2508_06041_amd as dp
    assert torch.cuda.is_available()
    cases = [(4096 + 256, 64), (1056, 17)]          # (columns, rank): the second input is the smaller one
    model = dp.Model(len(cases))
    Gs, xs = [], []
    for i, (in_, r) in enumerate(cases):
        lin = synth.make_linear(8, in_, 4, 3, seed=900 + i)
        model.dpllm_load_linear(i, synth.planes_np(lin["planes"]), {k: synth.lut_np(v) for k, v in lin["luts"].items()}, 3)
        g = torch.Generator().manual_seed(901 + i)
        G = (torch.randn(r, in_, generator=g) / math.sqrt(r)).half().cuda()
        x = synth.make_x(in_, 1, seed=902 + i)[0].cuda()
        est = float(synth.estimates_fp64(G, x[None])[0])
        model.dpllm_set_selector(i, 3, 4, dp.DPLLM_SEL_PROJ, G=G, T=est * (0.9 if i == 0 else 1.1))
        Gs.append(G)
        xs.append(x)
    ref = [model.dpllm_estimate(i, 3, 4, xs[i]) for i in range(len(cases))]      # through the workspace
    torch.cuda.synchronize()
    assert [int(k) for _, k in ref] == [4, 3]
    e_out = torch.full((len(cases),), -1.0, dtype=torch.float32, device="cuda")
    k_out = torch.full((len(cases),), -1, dtype=torch.int32, device="cuda")
    for rep in range(2):                            # and once more over the array the previous calls left behind
        e_out.fill_(-1.0)
        k_out.fill_(-1)
        for i in range(len(cases)):                 # the larger input first, then the smaller one, back to back
            model.dpllm_estimate_noalloc(i, 3, 4, xs[i], e_out[i:i + 1], k_out[i:i + 1])
        torch.cuda.synchronize()
        for i in range(len(cases)):
            assert torch.equal(e_out[i:i + 1], ref[i][0]), (rep, i, e_out[i].item(), ref[i][0].item())
            assert torch.equal(k_out[i:i + 1], ref[i][1]), (rep, i)
    # the other estimator kinds, and the size limit
    model.dpllm_set_selector(0, 3, 4, dp.DPLLM_SEL_LINREG, alpha=0.5, beta=-1.0, T=0.0)
    e_ref, k_ref = model.dpllm_estimate(0, 3, 4, xs[0])
    model.dpllm_estimate_noalloc(0, 3, 4, xs[0], e_out[0:1], k_out[0:1])
    torch.cuda.synchronize()
    assert torch.equal(e_out[0:1], e_ref) and torch.equal(k_out[0:1], k_ref)
    model.dpllm_set_selector(1, 3, 3, dp.DPLLM_SEL_NONE)
    model.dpllm_estimate_noalloc(1, 3, 3, xs[1], e_out[1:2], k_out[1:2])
    torch.cuda.synchronize()
    assert int(k_out[1]) == 3 and float(e_out[1]) == 0.0
    big = torch.zeros((257, cases[1][0]), dtype=torch.float16, device="cuda")
    model.dpllm_set_selector(1, 3, 4, dp.DPLLM_SEL_PROJ, G=big, T=0.0)
    with pytest.raises(dp.DpllmError) as ei:
        model.dpllm_estimate_noalloc(1, 3, 4, xs[1], e_out[1:2], k_out[1:2])
    assert ei.value.code == dp.DPLLM_ERANGE
    model.close()
