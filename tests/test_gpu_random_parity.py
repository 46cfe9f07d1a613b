"""GPU parity on randomly drawn layer shapes: forward and backward pass against the CPU oracle, through
the C ABI, for all four F(m x m, r x r) the library builds.

Every case is drawn from a fixed seed: filter size and output tile, padding 0 .. r-1, 1-39 images,
1-149 input and output channels (a few cases up to the 638 the panels hold), 1-33 pixels per side
(ragged tiles, images smaller than a tile, several images per 64-tile block and blocks that span
images), densities from empty to full, a quarter of the cases with the skewed row-density recipe.
Tolerance as in the fixed-shape tests: max|gpu - oracle64| <= rtol * max|oracle64| over a whole
tensor, rtol 1e-5 for F(2x2,3x3) and 1e-4 for the others; outputs are pre-filled with NaN, so an
element that is not written fails.  The backward pass reuses the transformed input of the forward
pass.  Run with -x: the first failing case names its shape.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_1702_08597_amd import binding as sw
from paper_1702_08597_amd import synth

pytestmark = pytest.mark.gpu

FMR = [(2, 3), (4, 3), (2, 5), (4, 5)]
CASES_PER_CHUNK = 30


def relerr(a, ref):
    s = np.abs(ref).max()
    return np.abs(a.astype(np.float64) - ref).max() / (s if s > 0 else 1.0)


def draw_case(rng, wide):
    while True:
        m, r = FMR[int(rng.integers(0, 4))]
        pad = int(rng.integers(0, r))
        top = 639 if wide else 150
        N, C, K = int(rng.integers(1, 40)), int(rng.integers(1, top)), int(rng.integers(1, top))
        if wide:
            N = int(rng.integers(1, 6))
        lo = max(1, r - 2 * pad)
        H, W = int(rng.integers(lo, 34)), int(rng.integers(lo, 34))
        dens = float(rng.choice([0.0, 0.03, 0.1, 0.3, 0.7, 1.0]))
        skew = bool(rng.random() < 0.25)
        seeds = [int(rng.integers(1 << 30)) for _ in range(3)]
        if H + 2 * pad - r + 1 >= 1 and W + 2 * pad - r + 1 >= 1:
            return dict(m=m, r=r, pad=pad, N=N, C=C, K=K, H=H, W=W, dens=dens, skew=skew, seeds=seeds)


def run_case(c):
    m, r, pad, N, C, K, H, W = (c[k] for k in ("m", "r", "pad", "N", "C", "K", "H", "W"))
    P = (m + r - 1) ** 2
    Ho, Wo = H + 2 * pad - r + 1, W + 2 * pad - r + 1
    x = synth.activations(N, C, H, W, c["seeds"][0])
    if c["skew"]:
        rp, ci, va = synth.skewed_weights(P, K, C, c["seeds"][1])
    else:
        rp, ci, va = synth.bernoulli_weights(P, K, C, c["dens"], c["seeds"][1])
    G = np.random.default_rng(c["seeds"][2]).standard_normal((N, K, Ho, Wo)).astype(np.float32)
    print("case F(%d,%d) pad=%d N=%d C=%d K=%d H=%d W=%d nnz=%d%s" % (m, r, pad, N, C, K, H, W, rp[-1],
                                                                     " skewed" if c["skew"] else ""), flush=True)
    o64, _, _ = oracle.forward_f64(x, rp, ci, va, K, m, r, pad, want_VM=False)
    din64, dv64, _, _ = oracle.backward_f64(x, rp, ci, va, G, K, m, r, pad, want_ZV=False)
    plan = sw.swconv_plan_create(N, C, H, W, K, m, r, pad)
    try:
        sw.swconv_set_weights(plan, rp, ci, va)
        sw.swconv_debug_check_schedule(plan)
        xd, gd = torch.from_numpy(x).cuda(), torch.from_numpy(G).cuda()
        out = torch.full((N, K, Ho, Wo), float("nan"), device="cuda")
        din = torch.full((N, C, H, W), float("nan"), device="cuda")
        dv = torch.full((max(1, len(va)),), float("nan"), device="cuda")
        sw.swconv_forward(plan, 0, xd.data_ptr(), out.data_ptr())
        sw.swconv_backward(plan, 0, 0, gd.data_ptr(), din.data_ptr(), dv.data_ptr())
        torch.cuda.synchronize()
        out_h, din_h, dv_h = out.cpu().numpy(), din.cpu().numpy(), dv.cpu().numpy()[:len(va)]
    finally:
        sw.swconv_plan_destroy(plan)
    assert not np.isnan(out_h).any(), "output not fully overwritten"
    assert not np.isnan(din_h).any(), "dL/dI not fully overwritten"
    tol = 1e-5 if (m, r) == (2, 3) else 1e-4
    errs = [relerr(out_h, o64), relerr(din_h, din64), relerr(dv_h, dv64) if len(va) else 0.0]
    assert max(errs) <= tol, (errs, tol)
    return max(errs) / tol


@pytest.mark.parametrize("chunk", range(8))
def test_random_shapes_forward_and_backward(chunk):
    rng = np.random.default_rng(170208597 + 31 * chunk)
    worst = 0.0
    for _ in range(CASES_PER_CHUNK):
        worst = max(worst, run_case(draw_case(rng, wide=False)))
    print("chunk %d: worst error / tolerance %.3f" % (chunk, worst), flush=True)


def test_random_shapes_with_many_channels():
    rng = np.random.default_rng(170208597 + 977)
    worst = 0.0
    for _ in range(16):
        worst = max(worst, run_case(draw_case(rng, wide=True)))
    print("worst error / tolerance %.3f" % worst, flush=True)
