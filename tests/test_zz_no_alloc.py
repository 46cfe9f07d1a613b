"""swconv_forward_noalloc: the forward pass with its intermediates in the library's static device scratch.

Checked through the C ABI against swconv_forward (same kernels: bit-identical) and against the oracle
(the forward tolerance), on two calls in a row, the second on a smaller layer - the scratch then still
holds the first call's data - and a third on the first layer again; a layer whose intermediates do not
fit the scratch is refused before anything is launched.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_1702_08597_amd import binding as sw
from paper_1702_08597_amd import synth

pytestmark = pytest.mark.gpu


def make(N, C, H, W, K, m, r, pad, seed, density=0.2):
    P = (m + r - 1) ** 2
    x = synth.activations(N, C, H, W, seed)
    rp, ci, va = synth.bernoulli_weights(P, K, C, density, seed + 1)
    plan = sw.swconv_plan_create(N, C, H, W, K, m, r, pad)
    sw.swconv_set_weights(plan, rp, ci, va)
    _, _, Ho, Wo = sw.swconv_plan_sizes(plan)
    ref = oracle.forward_f64(x, rp, ci, va, K, m, r, pad, want_VM=False)[0]
    return dict(plan=plan, x=torch.from_numpy(x).cuda(), shape=(N, K, Ho, Wo), ref=ref,
                tol=1e-5 if (m, r) == (2, 3) else 1e-4)


def run(L, fn, stream):
    out = torch.full(L["shape"], float("nan"), device="cuda")
    fn(L["plan"], stream, L["x"].data_ptr(), out.data_ptr())
    torch.cuda.synchronize()
    return out.cpu().numpy()


def test_static_scratch_forward_equals_forward_and_oracle_on_calls_in_a_row():
    st = torch.cuda.current_stream().cuda_stream
    big = make(24, 96, 13, 13, 120, 4, 3, 1, 4100)          # several tile blocks, ragged 13 x 13 tiles
    small = make(3, 20, 9, 11, 14, 2, 3, 1, 4200)           # fewer tiles, other F(m,r): other offsets in the scratch
    fused = make(4, 24, 13, 13, 40, 2, 5, 2, 4300)          # steps 2 and 3 in one kernel: only V is used
    try:
        for L in (big, small, fused, big, small):
            print("static scratch: output shape", L["shape"], flush=True)
            got = run(L, sw.swconv_forward_noalloc, st)
            assert not np.isnan(got).any(), "output not fully overwritten"
            want = run(L, sw.swconv_forward, st)
            np.testing.assert_array_equal(got.view(np.uint32), want.view(np.uint32))
            assert np.abs(got - L["ref"]).max() <= L["tol"] * np.abs(L["ref"]).max()
        # the static pass leaves nothing in the plan's own workspaces
        run(small, sw.swconv_forward_noalloc, st)
        with pytest.raises(sw.SwconvError) as e:
            sw.swconv_debug_copy_V(small["plan"], 20)
        assert e.value.status == sw.SWCONV_ESTATE
    finally:
        for L in (big, small, fused):
            sw.swconv_plan_destroy(L["plan"])


def test_static_scratch_forward_refuses_what_does_not_fit_and_needs_weights():
    N, C, H, W, K = 64, 256, 13, 13, 384                    # V + M = 94 MB > 64 MiB
    plan = sw.swconv_plan_create(N, C, H, W, K, 4, 3, 1)
    try:
        x = torch.zeros((N, C, H, W), device="cuda")
        out = torch.full((N, K, 13, 13), 7.0, device="cuda")
        with pytest.raises(sw.SwconvError) as e:
            sw.swconv_forward_noalloc(plan, 0, x.data_ptr(), out.data_ptr())
        assert e.value.status == sw.SWCONV_ESTATE
        rp, ci, va = synth.bernoulli_weights(36, K, C, 0.05, 4400)
        sw.swconv_set_weights(plan, rp, ci, va)
        with pytest.raises(sw.SwconvError) as e:
            sw.swconv_forward_noalloc(plan, 0, x.data_ptr(), out.data_ptr())
        assert e.value.status == sw.SWCONV_EUNSUPPORTED
        torch.cuda.synchronize()
        assert torch.all(out == 7.0).item()                 # nothing was launched
    finally:
        sw.swconv_plan_destroy(plan)
