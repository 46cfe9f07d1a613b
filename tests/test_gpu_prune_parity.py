"""GPU parity of the pruning step (Eq. 8, Eq. 9).  Two checks: against the oracle's float instantiation
(the keep/drop decision is taken in fp32 on both sides with one rounding per operation, so everything is
bit-exact), and against the double instantiation, which is the one pinned to the thresholds the paper
states: Eq. 8 fixes no rounding, so there the decision may differ only for entries whose score
|w'| (|g| + beta) lies within a few fp32 ulps of eps, and kept values agree to fp32 rounding."""
import numpy as np
import pytest
import torch

import oracle
from paper_1702_08597_amd import binding as sw
from paper_1702_08597_amd import synth

pytestmark = pytest.mark.gpu


def gpu_prune(rp, ci, va, g, eta, lam, eps, beta):
    d = lambda a: torch.from_numpy(a).cuda()
    rpd, cid, vad, gd = d(rp), d(ci), d(va), d(g)
    n = max(1, len(va))
    upd = torch.full((n,), float("nan"), device="cuda")
    rp2 = torch.full((len(rp),), -7, dtype=torch.int32, device="cuda")
    ci2 = torch.full((n,), -7, dtype=torch.int32, device="cuda")
    va2 = torch.full((n,), float("nan"), device="cuda")
    sw.swconv_prune_step(len(rp) - 1, rpd.data_ptr(), cid.data_ptr(), vad.data_ptr(), gd.data_ptr(), eta, lam, eps,
                         beta, torch.cuda.current_stream().cuda_stream, upd.data_ptr(), rp2.data_ptr(), ci2.data_ptr(),
                         va2.data_ptr())
    torch.cuda.synchronize()
    rp2_host = rp2.cpu().numpy()
    k = int(rp2_host[-1])
    return upd.cpu().numpy()[:len(va)], rp2_host, ci2.cpu().numpy()[:k], va2.cpu().numpy()[:k], (rp2, ci2, va2)


@pytest.mark.parametrize("P,K,C,density,seed", [(36, 384, 256, 0.1, 1), (16, 7, 5, 0.5, 2), (36, 2100, 3, 0.7, 3),
                                                (4, 3, 9, 0.0, 4), (36, 40, 600, 1.0, 5)])
def test_prune_step_bit_exact(P, K, C, density, seed):
    rng = np.random.default_rng(seed)
    rp, ci, va = synth.bernoulli_weights(P, K, C, density, seed + 10, sigma=2e-3)
    g = (rng.standard_normal(len(va)) * 0.05).astype(np.float32)
    g[::5] = 0.0
    eta, lam, eps, beta = 0.01, 1e-3, 1e-4, 0.1
    upd_o, (rp_o, ci_o, va_o) = oracle.prune_step(rp, ci, va, g, eta, lam, eps, beta, np.float32)
    upd, rp2, ci2, va2, _ = gpu_prune(rp, ci, va, g, eta, lam, eps, beta)
    if len(va):
        assert 0 < rp_o[-1] < len(va) or density in (0.0,)
    np.testing.assert_array_equal(upd.view(np.uint32), upd_o.view(np.uint32))
    np.testing.assert_array_equal(rp2, rp_o)
    np.testing.assert_array_equal(ci2, ci_o)
    np.testing.assert_array_equal(va2.view(np.uint32), va_o.view(np.uint32))


@pytest.mark.parametrize("P,K,C,density,seed", [(36, 384, 256, 0.1, 1), (16, 7, 5, 0.5, 2), (36, 40, 600, 1.0, 5)])
def test_prune_step_against_the_double_oracle(P, K, C, density, seed):
    rng = np.random.default_rng(seed)
    rp, ci, va = synth.bernoulli_weights(P, K, C, density, seed + 10, sigma=2e-3)
    g = (rng.standard_normal(len(va)) * 0.05).astype(np.float32)
    g[::5] = 0.0
    eta, lam, eps, beta = 0.01, 1e-3, 1e-4, 0.1
    # the double oracle gets the hyper-parameters as the floats the GPU entry point receives
    f = lambda v: float(np.float32(v))
    upd64, (rp64, ci64, va64) = oracle.prune_step(rp, ci, va.astype(np.float64), g.astype(np.float64), f(eta), f(lam),
                                                  f(eps), f(beta), np.float64)
    upd, rp2, ci2, va2, _ = gpu_prune(rp, ci, va, g, eta, lam, eps, beta)
    # the score in double, from the double update (before thresholding): w' = w - eta (g + lam sign w)
    w64, g64 = va.astype(np.float64), g.astype(np.float64)
    wp = w64 - f(eta) * (g64 + f(lam) * np.sign(w64))
    score = np.abs(wp) * (np.abs(g64) + f(beta))
    near = np.abs(score - f(eps)) <= 8 * np.spacing(np.float32(eps)).astype(np.float64)   # within a few fp32 ulps of eps
    keep64, keep = upd64 != 0.0, upd != 0.0
    # (an entry whose update is exactly 0 is dropped on both sides: its score is 0 < eps)
    disagree = keep64 != keep
    assert not (disagree & ~near).any(), "keep/drop differs away from the threshold"
    print("entries %d, near the threshold %d, decided differently %d" % (len(va), near.sum(), disagree.sum()), flush=True)
    both = keep64 & keep
    # kept values: fp32 rounds the sum g + lambda sign(w) (half an ulp of it, scaled by eta) and the fused
    # multiply-add (half an ulp of the result); the double result is exact to far below either
    step32 = np.abs(g + np.float32(lam) * np.sign(va))
    bound = 0.5 * np.spacing(np.abs(upd)).astype(np.float64) + f(eta) * 0.5 * np.spacing(step32).astype(np.float64)
    assert np.all(np.abs(upd[both].astype(np.float64) - upd64[both]) <= 1.01 * bound[both])
    if not disagree.any():
        np.testing.assert_array_equal(rp2, rp64)
        np.testing.assert_array_equal(ci2, ci64)
    # the compaction is consistent with the GPU's own decisions: survivors in order, row counts match
    np.testing.assert_array_equal(ci2, ci[keep])
    np.testing.assert_array_equal(va2.view(np.uint32), upd[keep].view(np.uint32))
    kept_before = np.concatenate([[0], np.cumsum(keep)])
    np.testing.assert_array_equal(rp2, kept_before[rp])


@pytest.mark.parametrize("m,r,N,C,K", [(4, 3, 3, 40, 30), (2, 5, 2, 24, 70), (2, 3, 4, 12, 9)])
def test_set_weights_device_round_trip_and_forward(m, r, N, C, K):
    """swconv_set_weights_device: the plan takes CSR arrays that live on the device; the export round trip
    returns them bit for bit and the forward pass matches the oracle (and a plan fed from the host)."""
    H = W = 13
    pad = r // 2
    P = (m + r - 1) ** 2
    x = synth.activations(N, C, H, W, 9100 + C)
    rp, ci, va = synth.bernoulli_weights(P, K, C, 0.3, 9101 + K)
    plan = sw.swconv_plan_create(N, C, H, W, K, m, r, pad)
    host_plan = sw.swconv_plan_create(N, C, H, W, K, m, r, pad)
    try:
        # first another pattern, so that the call below really replaces weights
        rp0, ci0, va0 = synth.bernoulli_weights(P, K, C, 0.5, 9102)
        sw.swconv_set_weights(plan, rp0, ci0, va0)
        dev = [torch.from_numpy(a).cuda() for a in (rp, ci, va)]
        st = torch.cuda.current_stream().cuda_stream
        sw.swconv_set_weights_device(plan, st, *(a.data_ptr() for a in dev))
        rp2, ci2, va2 = sw.swconv_debug_export_weights(plan, K, int(rp[-1]))
        np.testing.assert_array_equal(rp2, rp)
        np.testing.assert_array_equal(ci2, ci)
        np.testing.assert_array_equal(va2.view(np.uint32), va.view(np.uint32))
        xd = torch.from_numpy(x).cuda()
        Ho, Wo = sw.swconv_plan_sizes(plan)[2:]
        out = torch.full((N, K, Ho, Wo), float("nan"), device="cuda")
        sw.swconv_forward(plan, st, xd.data_ptr(), out.data_ptr())
        torch.cuda.synchronize()
        ref = oracle.forward_f64(x, rp, ci, va, K, m, r, pad, want_VM=False)[0]
        got = out.cpu().numpy()
        assert np.abs(got - ref).max() <= (1e-5 if (m, r) == (2, 3) else 1e-4) * np.abs(ref).max()
        sw.swconv_set_weights(host_plan, rp, ci, va)
        out2 = torch.full_like(out, float("nan"))
        sw.swconv_forward(host_plan, st, xd.data_ptr(), out2.data_ptr())
        torch.cuda.synchronize()
        np.testing.assert_array_equal(got.view(np.uint32), out2.cpu().numpy().view(np.uint32))
        # an empty weight set through the same door
        rpz = torch.zeros(P * K + 1, dtype=torch.int32, device="cuda")
        sw.swconv_set_weights_device(plan, st, rpz.data_ptr(), 0, 0)
        sw.swconv_forward(plan, st, xd.data_ptr(), out.data_ptr())
        torch.cuda.synchronize()
        assert torch.all(out == 0).item()
    finally:
        sw.swconv_plan_destroy(plan)
        sw.swconv_plan_destroy(host_plan)


def test_backward_prune_set_weights_forward_round():
    """One training-style round on the device: forward, backward, pruning step, new weights, forward."""
    cfg = dict(N=4, C=32, H=13, W=13, K=24, m=4, pad=1)
    N, C, H, W, K, m, pad = (cfg[k] for k in ("N", "C", "H", "W", "K", "m", "pad"))
    x = synth.activations(N, C, H, W, 50)
    rp, ci, va = synth.bernoulli_weights(36, K, C, 0.3, 51, sigma=2e-3)
    G = np.random.default_rng(52).standard_normal((N, K, 13, 13)).astype(np.float32)
    plan = sw.swconv_plan_create(N, C, H, W, K, m, 3, pad)
    try:
        sw.swconv_set_weights(plan, rp, ci, va)
        xd, gd = torch.from_numpy(x).cuda(), torch.from_numpy(G).cuda()
        out = torch.empty((N, K, 13, 13), device="cuda")
        dv = torch.empty((len(va),), device="cuda")
        st = torch.cuda.current_stream().cuda_stream
        sw.swconv_forward(plan, st, xd.data_ptr(), out.data_ptr())
        sw.swconv_backward(plan, st, 0, gd.data_ptr(), 0, dv.data_ptr())
        torch.cuda.synchronize()
        grad = dv.cpu().numpy()
        upd, rp2, ci2, va2, dev = gpu_prune(rp, ci, va, grad, 1e-4, 1e-3, 1e-4, 0.1)
        upd_o, (rp_o, ci_o, va_o) = oracle.prune_step(rp, ci, va, grad, 1e-4, 1e-3, 1e-4, 0.1, np.float32)
        np.testing.assert_array_equal(rp2, rp_o)
        np.testing.assert_array_equal(va2.view(np.uint32), va_o.view(np.uint32))
        assert 0 < rp2[-1] < len(va)
        # without re-packing: the thresholded values in the old pattern (zeros where an entry was dropped)
        # go into the packed weights in place; dropped entries then multiply as stored zeros
        sw.swconv_update_values(plan, st, torch.from_numpy(upd).cuda().data_ptr())
        sw.swconv_forward(plan, st, xd.data_ptr(), out.data_ptr())
        torch.cuda.synchronize()
        out_in_place = out.cpu().numpy()
        # with re-packing: the compacted CSR of the survivors, taken from the device arrays of the step
        sw.swconv_set_weights_device(plan, st, *(a.data_ptr() for a in dev))
        rp3, ci3, va3 = sw.swconv_debug_export_weights(plan, K, int(rp_o[-1]))
        np.testing.assert_array_equal(rp3, rp_o)
        np.testing.assert_array_equal(ci3, ci_o)
        np.testing.assert_array_equal(va3.view(np.uint32), va_o.view(np.uint32))
        out.fill_(float("nan"))
        sw.swconv_forward(plan, st, xd.data_ptr(), out.data_ptr())
        torch.cuda.synchronize()
        ref = oracle.forward_f64(x, rp_o, ci_o, va_o, K, m, 3, pad, want_VM=False)[0]
        assert np.abs(out.cpu().numpy() - ref).max() <= 1e-4 * np.abs(ref).max()
        # a stored zero adds exactly nothing to a row sum whose order is otherwise unchanged
        np.testing.assert_array_equal(out_in_place, out.cpu().numpy())
    finally:
        sw.swconv_plan_destroy(plan)


@pytest.mark.parametrize("m,r,C,K,backward_first", [(4, 3, 40, 30, True), (4, 3, 40, 30, False), (2, 5, 24, 70, True),
                                                     (2, 3, 12, 9, False)])
def test_update_values_equals_setting_the_weights_anew(m, r, C, K, backward_first):
    """Fine-tuning step (Section 4.3): new values, same pattern, written in place on the device - every
    result must be bit-identical to a plan that was given the new values with swconv_set_weights."""
    N, H, W, pad = 5, 13, 13, r // 2
    P = (m + r - 1) ** 2
    rng = np.random.default_rng(8800 + C)
    x = synth.activations(N, C, H, W, 8801)
    rp, ci, va1 = synth.bernoulli_weights(P, K, C, 0.3, 8802)
    va2 = rng.standard_normal(len(va1)).astype(np.float32)
    G = rng.standard_normal((N, K, 13, 13)).astype(np.float32)
    xd, gd = torch.from_numpy(x).cuda(), torch.from_numpy(G).cuda()

    def passes(plan):
        out = torch.full((N, K, 13, 13), float("nan"), device="cuda")
        din = torch.full((N, C, H, W), float("nan"), device="cuda")
        dv = torch.full((len(va1),), float("nan"), device="cuda")
        sw.swconv_forward(plan, 0, xd.data_ptr(), out.data_ptr())
        sw.swconv_backward(plan, 0, xd.data_ptr(), gd.data_ptr(), din.data_ptr(), dv.data_ptr())
        torch.cuda.synchronize()
        return out.cpu().numpy(), din.cpu().numpy(), dv.cpu().numpy()

    ref_plan = sw.swconv_plan_create(N, C, H, W, K, m, r, pad)
    plan = sw.swconv_plan_create(N, C, H, W, K, m, r, pad)
    try:
        sw.swconv_set_weights(ref_plan, rp, ci, va2)
        want = passes(ref_plan)
        sw.swconv_set_weights(plan, rp, ci, va1)
        if backward_first:
            passes(plan)                       # the transposed weights exist and are updated in place
        sw.swconv_update_values(plan, 0, torch.from_numpy(va2).cuda().data_ptr())
        got = passes(plan)                     # otherwise they are built from the updated values
        for g, w in zip(got, want):
            np.testing.assert_array_equal(g.view(np.uint32), w.view(np.uint32))
        rp3, ci3, va3 = sw.swconv_debug_export_weights(plan, K, int(rp[-1]))
        np.testing.assert_array_equal(rp3, rp)
        np.testing.assert_array_equal(ci3, ci)
        np.testing.assert_array_equal(va3.view(np.uint32), va2.view(np.uint32))
        o64, _, _ = oracle.forward_f64(x, rp, ci, va2, K, m, r, pad, want_VM=False)
        assert np.abs(got[0] - o64).max() <= 1e-4 * np.abs(o64).max()
    finally:
        sw.swconv_plan_destroy(plan)
        sw.swconv_plan_destroy(ref_plan)
