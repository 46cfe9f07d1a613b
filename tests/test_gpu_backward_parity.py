"""GPU parity of the backward pass (Eq. 5, Eq. 6) against the CPU oracle, through the C ABI.

Tolerances as for the forward pass: norm-relative over a whole tensor, 1e-5 for F(2x2,3x3) and 1e-4 for
F(4x4,3x3); integer-valued data must match bit for bit.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_1702_08597_amd import binding as sw
from paper_1702_08597_amd import synth

pytestmark = pytest.mark.gpu

RTOL = {2: 1e-5, 4: 1e-4}


def relerr(a, ref):
    scale = np.abs(ref).max()
    return np.abs(a.astype(np.float64) - ref).max() / (scale if scale > 0 else 1.0)


def run_backward(N, C, H, W, K, m, pad, x, rp, ci, va, G, want_dvals=True):
    plan = sw.swconv_plan_create(N, C, H, W, K, m, 3, pad)
    try:
        sw.swconv_set_weights(plan, rp, ci, va)
        xd = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).cuda()
        gd = torch.from_numpy(np.ascontiguousarray(G, dtype=np.float32)).cuda()
        din = torch.full((N, C, H, W), float("nan"), dtype=torch.float32, device="cuda")
        dvals = torch.full((max(1, len(va)),), float("nan"), dtype=torch.float32, device="cuda")
        st = torch.cuda.current_stream()
        torch.cuda.synchronize()
        sw.swconv_backward(plan, st.cuda_stream, xd.data_ptr(), gd.data_ptr(), din.data_ptr(),
                           dvals.data_ptr() if want_dvals else 0)
        st.synchronize()
        return din.cpu().numpy(), dvals.cpu().numpy()[:len(va)], sw.swconv_debug_copy_dZ(plan, K), \
            sw.swconv_debug_copy_dV(plan, C)
    finally:
        sw.swconv_plan_destroy(plan)


def check(N, C, H, W, K, m, pad, x, rp, ci, va, G, stages=True, want_dvals=True):
    print("backward case N=%d C=%d H=%d W=%d K=%d m=%d pad=%d nnz=%d" % (N, C, H, W, K, m, pad, rp[-1]), flush=True)
    din64, dvals64, dZ64, dV64 = oracle.backward_f64(x, rp, ci, va, G, K, m, 3, pad, want_ZV=stages)
    din, dvals, dZ, dV = run_backward(N, C, H, W, K, m, pad, x, rp, ci, va, G, want_dvals)
    assert not np.isnan(din).any(), "dL/dI not fully overwritten"
    if stages:
        assert relerr(dZ, dZ64) <= RTOL[m]
        assert relerr(dV, dV64) <= RTOL[m]
    e = relerr(din, din64)
    print("  dL/dI max rel err %.3g" % e, flush=True)
    assert e <= RTOL[m]
    if want_dvals and len(va):
        assert not np.isnan(dvals).any(), "dL/dW_F not fully overwritten"
        e = relerr(dvals, dvals64)
        print("  dL/dW_F max rel err %.3g" % e, flush=True)
        assert e <= RTOL[m]


SMALL = [
    (9, 19, 13, 13, 10, 2, 1),
    (5, 7, 13, 11, 13, 4, 1),
    (2, 3, 56, 40, 5, 4, 1),
    (3, 5, 9, 17, 6, 2, 0),
    (1, 1, 1, 1, 1, 2, 1),
    (1, 2, 3, 3, 3, 4, 0),
    (70, 4, 4, 4, 4, 4, 1),
    (1, 20, 6, 6, 638, 2, 1),   # largest K whose dL/dZ panel fits LDS
]


@pytest.mark.parametrize("N,C,H,W,K,m,pad", SMALL)
def test_small_shapes_all_stages(N, C, H, W, K, m, pad):
    P = (m + 2) ** 2
    rng = np.random.default_rng(7000 + N + K)
    x = synth.activations(N, C, H, W, 100 + N + C)
    rp, ci, va = synth.bernoulli_weights(P, K, C, 0.3, 200 + K)
    G = rng.standard_normal((N, K, H + 2 * pad - 2, W + 2 * pad - 2)).astype(np.float32)
    check(N, C, H, W, K, m, pad, x, rp, ci, va, G, want_dvals=WANT_DVALS)


@pytest.mark.parametrize("m", [2, 4])
def test_integer_data_bit_exact(m):
    N, C, H, W, K = 6, 24, 13, 13, 22
    x, rp, ci, va = synth.integer_case(N, C, H, W, K, m, 3, 0.4, 300 + m)
    G = np.random.default_rng(301).integers(-2, 3, size=(N, K, 13, 13)).astype(np.float32)
    din64, dvals64, dZ64, dV64 = oracle.backward_f64(x, rp, ci, va, G, K, m)
    din, dvals, dZ, dV = run_backward(N, C, H, W, K, m, 1, x, rp, ci, va, G, WANT_DVALS)
    np.testing.assert_array_equal(dZ.astype(np.float64), dZ64)
    np.testing.assert_array_equal(dV.astype(np.float64), dV64)
    np.testing.assert_array_equal(din.astype(np.float64), din64)
    if WANT_DVALS:
        np.testing.assert_array_equal(dvals.astype(np.float64), dvals64)


@pytest.mark.parametrize("name", ["alexnet_conv3_n32_f4", "alexnet_conv4_n64_f4", "conv4_skewed_n64_f4",
                                  "alexnet_conv3_n1_f2"])
def test_full_size_configs(name):
    cfg, x, rp, ci, va = synth.make_layer(name)
    G = np.random.default_rng(cfg["seed"] + 5).standard_normal((cfg["N"], cfg["K"], cfg["Ho"], cfg["Wo"])).astype(
        np.float32)
    check(cfg["N"], cfg["C"], cfg["H"], cfg["W"], cfg["K"], cfg["m"], cfg["pad"], x, rp, ci, va, G,
          stages=(cfg["N"] <= 32), want_dvals=WANT_DVALS)


def test_backward_can_reuse_the_forward_pass_transform():
    N, C, H, W, K, m = 5, 20, 13, 13, 18, 4
    rng = np.random.default_rng(9100)
    x = synth.activations(N, C, H, W, 9101)
    rp, ci, va = synth.bernoulli_weights(36, K, C, 0.3, 9102)
    G = rng.standard_normal((N, K, 13, 13)).astype(np.float32)
    din64, dvals64, _, _ = oracle.backward_f64(x, rp, ci, va, G, K, m, want_ZV=False)
    plan = sw.swconv_plan_create(N, C, H, W, K, m, 3, 1)
    try:
        sw.swconv_set_weights(plan, rp, ci, va)
        xd, gd = torch.from_numpy(x).cuda(), torch.from_numpy(G).cuda()
        out = torch.empty((N, K, 13, 13), device="cuda")
        din = torch.full((N, C, H, W), float("nan"), device="cuda")
        dv = torch.full((len(va),), float("nan"), device="cuda")
        with pytest.raises(sw.SwconvError) as e:     # nothing to reuse yet
            sw.swconv_backward(plan, 0, 0, gd.data_ptr(), din.data_ptr(), dv.data_ptr())
        assert e.value.status == sw.SWCONV_ESTATE
        sw.swconv_forward(plan, 0, xd.data_ptr(), out.data_ptr())
        sw.swconv_backward(plan, 0, 0, gd.data_ptr(), din.data_ptr(), dv.data_ptr())
        torch.cuda.synchronize()
        assert relerr(din.cpu().numpy(), din64) <= RTOL[m]
        assert relerr(dv.cpu().numpy(), dvals64) <= RTOL[m]
        with pytest.raises(sw.SwconvError):          # the backward pass used the workspace
            sw.swconv_backward(plan, 0, 0, gd.data_ptr(), din.data_ptr(), dv.data_ptr())
        # new weights: what the workspaces hold belongs to the old ones until a forward pass has run
        sw.swconv_forward(plan, 0, xd.data_ptr(), out.data_ptr())
        sw.swconv_set_weights(plan, rp, ci, va)
        with pytest.raises(sw.SwconvError) as e:
            sw.swconv_backward(plan, 0, 0, gd.data_ptr(), din.data_ptr(), dv.data_ptr())
        assert e.value.status == sw.SWCONV_ESTATE
        with pytest.raises(sw.SwconvError) as e:
            sw.swconv_debug_copy_M(plan, K)
        assert e.value.status == sw.SWCONV_ESTATE
        sw.swconv_forward(plan, 0, xd.data_ptr(), out.data_ptr())
        sw.swconv_backward(plan, 0, 0, gd.data_ptr(), din.data_ptr(), dv.data_ptr())
        torch.cuda.synchronize()
        assert relerr(dv.cpu().numpy(), dvals64) <= RTOL[m]
    finally:
        sw.swconv_plan_destroy(plan)


def test_profile_backward_reports_seven_kernels_and_skips_unwanted_ones(monkeypatch):
    monkeypatch.setenv("SWCONV_FUSE_INPUT_GRAD", "0")   # the seven-kernel pipeline
    N, C, H, W, K, m = 4, 16, 13, 13, 12, 4
    x = synth.activations(N, C, H, W, 1)
    rp, ci, va = synth.bernoulli_weights(36, K, C, 0.3, 2)
    plan = sw.swconv_plan_create(N, C, H, W, K, m, 3, 1)
    try:
        sw.swconv_set_weights(plan, rp, ci, va)
        xd = torch.from_numpy(x).cuda()
        gd = torch.ones((N, K, 13, 13), device="cuda")
        din = torch.empty_like(xd)
        dv = torch.empty((len(va),), device="cuda")
        ms = sw.swconv_profile_backward(plan, 0, xd.data_ptr(), gd.data_ptr(), din.data_ptr(), dv.data_ptr(), 3)
        assert ms.shape == (7,) and np.all(ms > 0) and np.all(ms < 50)
        ms = sw.swconv_profile_backward(plan, 0, xd.data_ptr(), gd.data_ptr(), din.data_ptr(), 0, 3)
        assert np.all(ms[1:4] == 0) and ms[0] > 0 and np.all(ms[4:] > 0)
        ms = sw.swconv_profile_backward(plan, 0, xd.data_ptr(), gd.data_ptr(), 0, dv.data_ptr(), 3)
        assert np.all(ms[5:] == 0) and np.all(ms[:5] > 0)
    finally:
        sw.swconv_plan_destroy(plan)


@pytest.mark.parametrize("N,C,H,W,K,m,r,pad", [
    (5, 7, 13, 13, 9, 4, 3, 1),     # four images per wave, a last group of one
    (3, 6, 13, 13, 5, 2, 3, 1),     # 49 tiles per image: one image per wave
    (2, 5, 56, 40, 4, 4, 3, 1),     # 140 tiles per image: three passes
    (3, 5, 27, 27, 6, 2, 5, 2),     # F(2x2,5x5): patches reach two tiles back, stays on two kernels
    (6, 4, 9, 17, 3, 2, 3, 0),      # no padding
])
def test_input_gradient_in_one_kernel_equals_the_two_kernel_path_and_the_oracle(N, C, H, W, K, m, r, pad, monkeypatch):
    print("input-grad case N=%d C=%d H=%d W=%d K=%d m=%d r=%d" % (N, C, H, W, K, m, r), flush=True)
    P = (m + r - 1) ** 2
    Ho, Wo = H + 2 * pad - r + 1, W + 2 * pad - r + 1
    x = synth.activations(N, C, H, W, 9300 + N)
    rp, ci, va = synth.bernoulli_weights(P, K, C, 0.3, 9301 + K)
    G = np.random.default_rng(9302).standard_normal((N, K, Ho, Wo)).astype(np.float32)
    din64, _, _, _ = oracle.backward_f64(x, rp, ci, va, G, K, m, r, pad, want_ZV=False)
    xd, gd = torch.from_numpy(x).cuda(), torch.from_numpy(G).cuda()
    got = []
    for fuse in (1, 0):
        monkeypatch.setenv("SWCONV_FUSE_INPUT_GRAD", str(fuse))
        plan = sw.swconv_plan_create(N, C, H, W, K, m, r, pad)
        try:
            sw.swconv_set_weights(plan, rp, ci, va)
            din = torch.full((N, C, H, W), float("nan"), device="cuda")
            ms = sw.swconv_profile_backward(plan, 0, xd.data_ptr(), gd.data_ptr(), din.data_ptr(), 0, 1)
            assert (ms[6] == 0) == (fuse == 1 and r == 3) and ms[5] > 0
            torch.cuda.synchronize()
            got.append(din.cpu().numpy())
        finally:
            sw.swconv_plan_destroy(plan)
    for d in got:
        assert not np.isnan(d).any()
        assert relerr(d, din64) <= RTOL[m]
    assert relerr(got[0], got[1].astype(np.float64)) <= 1e-5


def test_unsupported_K_is_refused():
    plan = sw.swconv_plan_create(1, 4, 6, 6, 700, 2, 3, 1)
    try:
        rp, ci, va = synth.bernoulli_weights(16, 700, 4, 0.5, 1)
        sw.swconv_set_weights(plan, rp, ci, va)
        x = torch.zeros((1, 4, 6, 6), device="cuda")
        g = torch.zeros((1, 700, 6, 6), device="cuda")
        d = torch.zeros((1, 4, 6, 6), device="cuda")
        with pytest.raises(sw.SwconvError) as e:
            sw.swconv_backward(plan, 0, x.data_ptr(), g.data_ptr(), d.data_ptr(), 0)
        assert e.value.status == sw.SWCONV_EUNSUPPORTED
    finally:
        sw.swconv_plan_destroy(plan)


WANT_DVALS = True
