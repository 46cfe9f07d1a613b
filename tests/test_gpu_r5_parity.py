"""GPU parity of the 5x5 layer, F(2x2,5x5) (t = 6, P = 36) and F(4x4,5x5) (t = 8, P = 64), forward and
backward, through the C ABI.

Tolerance: F(2,5) uses the input transform of F(4,3) (same interpolation points, same B^T with
entries up to 5), so the bound of F(4x4,3x3) applies: max|gpu - oracle64| <= 1e-4 * max|oracle64|
over a whole tensor; F(4,5) adds the points +-1/2 (entries up to 21/4 and 8) and the oracle's own
float instantiation stays below 1e-6 of the fp64 one on these inputs, so the same bound is kept.
Integer-valued data must match bit for bit for F(2,5); F(4,5) has entries down to 1/8, whose
products with integers need more than 24 bits at these magnitudes, so it is checked by tolerance.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_1702_08597_amd import binding as sw
from paper_1702_08597_amd import synth

pytestmark = pytest.mark.gpu

RTOL = 1e-4
M, R, P = 2, 5, 36


def relerr(a, ref):
    scale = np.abs(ref).max()
    return np.abs(a.astype(np.float64) - ref).max() / (scale if scale > 0 else 1.0)


def run_gpu(N, C, H, W, K, pad, x, rp, ci, va, G):
    """Forward, then backward with the input given again; returns every tensor the two passes leave."""
    plan = sw.swconv_plan_create(N, C, H, W, K, M, R, pad)
    try:
        _, _, Ho, Wo = sw.swconv_plan_sizes(plan)
        sw.swconv_set_weights(plan, rp, ci, va)
        xd = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).cuda()
        gd = torch.from_numpy(np.ascontiguousarray(G, dtype=np.float32)).cuda()
        out = torch.full((N, K, Ho, Wo), float("nan"), dtype=torch.float32, device="cuda")
        din = torch.full((N, C, H, W), float("nan"), dtype=torch.float32, device="cuda")
        dvals = torch.full((max(1, len(va)),), float("nan"), dtype=torch.float32, device="cuda")
        st = torch.cuda.current_stream()
        torch.cuda.synchronize()
        sw.swconv_forward(plan, st.cuda_stream, xd.data_ptr(), out.data_ptr())
        st.synchronize()
        res = dict(out=out.cpu().numpy(), V=sw.swconv_debug_copy_V(plan, C), M=sw.swconv_debug_copy_M(plan, K))
        sw.swconv_backward(plan, st.cuda_stream, xd.data_ptr(), gd.data_ptr(), din.data_ptr(), dvals.data_ptr())
        st.synchronize()
        res.update(din=din.cpu().numpy(), dvals=dvals.cpu().numpy()[:len(va)], dZ=sw.swconv_debug_copy_dZ(plan, K),
                   dV=sw.swconv_debug_copy_dV(plan, C))
        return res
    finally:
        sw.swconv_plan_destroy(plan)


def run_oracle(x, rp, ci, va, G, K, pad, stages=True):
    o64, V64, M64 = oracle.forward_f64(x, rp, ci, va, K, M, R, pad, want_VM=stages)
    din64, dvals64, dZ64, dV64 = oracle.backward_f64(x, rp, ci, va, G, K, M, R, pad, want_ZV=stages)
    return dict(out=o64, V=V64, M=M64, din=din64, dvals=dvals64, dZ=dZ64, dV=dV64)


SMALL = [
    # N, C, H, W, K, pad: several tile blocks, ragged tails, odd sizes
    (3, 7, 13, 11, 9, 2),
    (2, 5, 27, 27, 6, 2),
    (9, 4, 8, 9, 5, 0),      # no padding: Ho = 4, Wo = 5
    (1, 1, 5, 5, 1, 0),      # one output pixel
    (1, 2, 1, 1, 3, 2),      # one input pixel, every tile mostly padding
    (70, 3, 4, 4, 4, 2),     # four tiles per image, many images
    (2, 6, 6, 7, 300, 1),    # pad = 1: Ho = H - 2
]


@pytest.mark.parametrize("N,C,H,W,K,pad", SMALL)
def test_small_shapes_all_stages(N, C, H, W, K, pad):
    print("r5 case N=%d C=%d H=%d W=%d K=%d pad=%d" % (N, C, H, W, K, pad), flush=True)
    x = synth.activations(N, C, H, W, 500 + N + C)
    rp, ci, va = synth.bernoulli_weights(P, K, C, 0.3, 600 + K)
    Ho, Wo = H + 2 * pad - 4, W + 2 * pad - 4
    G = np.random.default_rng(700 + N).standard_normal((N, K, Ho, Wo)).astype(np.float32)
    ref = run_oracle(x, rp, ci, va, G, K, pad)
    got = run_gpu(N, C, H, W, K, pad, x, rp, ci, va, G)
    for name in ("V", "M", "out", "dZ", "dV", "din", "dvals"):
        assert not np.isnan(got[name]).any(), name + " not fully overwritten"
        e = relerr(got[name], ref[name])
        print("  %-5s max rel err %.3g" % (name, e), flush=True)
        assert e <= RTOL, name


def test_integer_data_bit_exact():
    # F(2,5)'s B^T, A^T and their transposes are integer matrices, so with integer weights given
    # in the Winograd domain every intermediate is an integer below 2**24
    N, C, H, W, K, pad = 5, 12, 13, 13, 10, 2
    x, rp, ci, va = synth.integer_case(N, C, H, W, K, M, R, 0.4, 305)
    G = np.random.default_rng(306).integers(-2, 3, size=(N, K, 13, 13)).astype(np.float32)
    ref = run_oracle(x, rp, ci, va, G, K, pad)
    got = run_gpu(N, C, H, W, K, pad, x, rp, ci, va, G)
    for name in ("V", "M", "out", "dZ", "dV", "din", "dvals"):
        assert np.abs(ref[name]).max() < 2 ** 24
        np.testing.assert_array_equal(got[name].astype(np.float64), ref[name], err_msg=name)


def test_alexnet_conv2_group_full_size():
    cfg, x, rp, ci, va = synth.make_layer("alexnet_conv2g_n32_f2r5")
    N, C, H, W, K, pad = (cfg[k] for k in ("N", "C", "H", "W", "K", "pad"))
    G = np.random.default_rng(cfg["seed"] + 5).standard_normal((N, K, cfg["Ho"], cfg["Wo"])).astype(np.float32)
    ref = run_oracle(x, rp, ci, va, G, K, pad, stages=False)
    got = run_gpu(N, C, H, W, K, pad, x, rp, ci, va, G)
    for name in ("out", "din", "dvals"):
        e = relerr(got[name], ref[name])
        print("  %-5s max rel err %.3g" % (name, e), flush=True)
        assert e <= RTOL, name


@pytest.mark.parametrize("m,r,pad,H", [(2, 5, 2, 27), (4, 3, 1, 13)])
def test_channel_groups_inside_the_whole_layers_tensors(m, r, pad, H):
    # AlexNet's 5x5 layer (and its last two 3x3 layers) have two channel groups: one plan per group,
    # both working in place on the whole layer's NCHW tensors through image strides.
    groups, N, Cg, Kg, W = 2, 5, 6, 10, H
    C, K, Pn = groups * Cg, groups * Kg, (m + r - 1) ** 2
    Ho = Wo = H + 2 * pad - r + 1
    rng = np.random.default_rng(4100 + r)
    x = synth.activations(N, C, H, W, 4101)
    G = rng.standard_normal((N, K, Ho, Wo)).astype(np.float32)
    xd, gd = torch.from_numpy(x).cuda(), torch.from_numpy(G).cuda()
    out = torch.full((N, K, Ho, Wo), float("nan"), device="cuda")
    din = torch.full((N, C, H, W), float("nan"), device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    for g in range(groups):
        print("group %d of F(%d,%d)" % (g, m, r), flush=True)
        rp, ci, va = synth.bernoulli_weights(Pn, Kg, Cg, 0.3, 4200 + g)
        xs = np.ascontiguousarray(x[:, g * Cg:(g + 1) * Cg])
        Gs = np.ascontiguousarray(G[:, g * Kg:(g + 1) * Kg])
        o64, _, _ = oracle.forward_f64(xs, rp, ci, va, Kg, m, r, pad, want_VM=False)
        din64, dvals64, _, _ = oracle.backward_f64(xs, rp, ci, va, Gs, Kg, m, r, pad, want_ZV=False)
        plan = sw.swconv_plan_create(N, Cg, H, W, Kg, m, r, pad)
        try:
            sw.swconv_plan_set_image_strides(plan, C * H * W, K * Ho * Wo)
            sw.swconv_set_weights(plan, rp, ci, va)
            dv = torch.full((len(va),), float("nan"), device="cuda")
            in_ptr = xd.data_ptr() + 4 * g * Cg * H * W
            out_ptr = out.data_ptr() + 4 * g * Kg * Ho * Wo
            sw.swconv_forward(plan, st, in_ptr, out_ptr)
            sw.swconv_backward(plan, st, in_ptr, gd.data_ptr() + 4 * g * Kg * Ho * Wo,
                               din.data_ptr() + 4 * g * Cg * H * W, dv.data_ptr())
            torch.cuda.synchronize()
        finally:
            sw.swconv_plan_destroy(plan)
        got_out, got_din = out.cpu().numpy(), din.cpu().numpy()
        assert relerr(got_out[:, g * Kg:(g + 1) * Kg], o64) <= RTOL
        assert relerr(got_din[:, g * Cg:(g + 1) * Cg], din64) <= RTOL
        assert relerr(dv.cpu().numpy(), dvals64) <= RTOL
        if g == 0:   # the other group's channels are untouched
            assert np.isnan(got_out[:, Kg:]).all() and np.isnan(got_din[:, Cg:]).all()
    assert not np.isnan(got_out).any() and not np.isnan(got_din).any()


FUSED = [
    # m = 2 layers with few input channels run steps 2 and 3 in one kernel: r, N, C, H, W, K, pad, density
    (5, 3, 48, 27, 27, 128, 2, 0.1),    # the conv2 group's shape, two row chunks
    (5, 2, 64, 9, 9, 65, 2, 0.3),       # one panel piece per thread exactly, rows longer than one batch, ragged chunk
    (5, 2, 100, 8, 8, 5, 2, 0.15),      # two pieces per thread, two batches
    (3, 4, 128, 13, 13, 130, 1, 0.1),   # F(2x2,3x3), the widest panel the kernel takes
    (3, 9, 19, 13, 13, 10, 1, 0.0),     # no stored entries at all
]


@pytest.mark.parametrize("r,N,C,H,W,K,pad,density", FUSED)
def test_fused_product_and_output_transform_against_oracle_and_three_kernel_path(r, N, C, H, W, K, pad, density,
                                                                                 monkeypatch):
    print("fused case r=%d N=%d C=%d H=%d W=%d K=%d" % (r, N, C, H, W, K), flush=True)
    Pn = (r + 1) ** 2
    x = synth.activations(N, C, H, W, 8100 + C)
    rp, ci, va = synth.bernoulli_weights(Pn, K, C, density, 8200 + K)
    o64, _, _ = oracle.forward_f64(x, rp, ci, va, K, 2, r, pad, want_VM=False)
    xd = torch.from_numpy(x).cuda()
    outs = []
    for fuse in (1, 0):
        monkeypatch.setenv("SWCONV_FUSE_OUTPUT", str(fuse))
        plan = sw.swconv_plan_create(N, C, H, W, K, 2, r, pad)
        try:
            sw.swconv_set_weights(plan, rp, ci, va)
            out = torch.full(o64.shape, float("nan"), dtype=torch.float32, device="cuda")
            ms = sw.swconv_profile_forward(plan, 0, xd.data_ptr(), out.data_ptr(), 2)
            assert (ms[2] == 0) == (fuse == 1), "which kernels ran"
            out.fill_(float("nan"))
            sw.swconv_forward(plan, 0, xd.data_ptr(), out.data_ptr())
            torch.cuda.synchronize()
            outs.append(out.cpu().numpy())
        finally:
            sw.swconv_plan_destroy(plan)
    for o in outs:
        assert not np.isnan(o).any()
        assert relerr(o, o64) <= RTOL
    assert relerr(outs[0], outs[1].astype(np.float64)) <= 1e-5


def test_rows_longer_than_the_fused_kernels_batches_fall_back():
    N, C, H, W, K = 2, 60, 9, 9, 8
    x = synth.activations(N, C, H, W, 8300)
    rp, ci, va = synth.bernoulli_weights(36, K, C, 0.9, 8301)     # rows of about 54 entries
    o64, _, _ = oracle.forward_f64(x, rp, ci, va, K, 2, 5, 2, want_VM=False)
    plan = sw.swconv_plan_create(N, C, H, W, K, 2, 5, 2)
    try:
        sw.swconv_set_weights(plan, rp, ci, va)
        xd = torch.from_numpy(x).cuda()
        out = torch.full(o64.shape, float("nan"), dtype=torch.float32, device="cuda")
        ms = sw.swconv_profile_forward(plan, 0, xd.data_ptr(), out.data_ptr(), 2)
        assert ms[2] > 0
        torch.cuda.synchronize()
        assert relerr(out.cpu().numpy(), o64) <= RTOL
    finally:
        sw.swconv_plan_destroy(plan)


F45 = [
    # N, C, H, W, K, pad
    (3, 7, 13, 11, 9, 2),
    (2, 5, 27, 27, 6, 2),
    (9, 4, 8, 9, 5, 0),
    (1, 1, 5, 5, 1, 0),      # one output pixel
    (1, 2, 1, 1, 3, 2),      # one input pixel
    (70, 3, 4, 4, 4, 2),     # one tile per image, many images
    (2, 6, 9, 12, 300, 1),
]


@pytest.mark.parametrize("N,C,H,W,K,pad", F45)
def test_f4x4_5x5_all_stages(N, C, H, W, K, pad):
    print("F(4,5) case N=%d C=%d H=%d W=%d K=%d pad=%d" % (N, C, H, W, K, pad), flush=True)
    x = synth.activations(N, C, H, W, 1500 + N + C)
    rp, ci, va = synth.bernoulli_weights(64, K, C, 0.3, 1600 + K)
    Ho, Wo = H + 2 * pad - 4, W + 2 * pad - 4
    G = np.random.default_rng(1700 + N).standard_normal((N, K, Ho, Wo)).astype(np.float32)
    o64, V64, M64 = oracle.forward_f64(x, rp, ci, va, K, 4, 5, pad)
    din64, dvals64, dZ64, dV64 = oracle.backward_f64(x, rp, ci, va, G, K, 4, 5, pad)
    ref = dict(out=o64, V=V64, M=M64, din=din64, dvals=dvals64, dZ=dZ64, dV=dV64)
    plan = sw.swconv_plan_create(N, C, H, W, K, 4, 5, pad)
    try:
        assert sw.swconv_plan_sizes(plan)[0] == 64
        sw.swconv_set_weights(plan, rp, ci, va)
        xd, gd = torch.from_numpy(x).cuda(), torch.from_numpy(G).cuda()
        out = torch.full((N, K, Ho, Wo), float("nan"), device="cuda")
        din = torch.full((N, C, H, W), float("nan"), device="cuda")
        dv = torch.full((max(1, len(va)),), float("nan"), device="cuda")
        sw.swconv_forward(plan, 0, xd.data_ptr(), out.data_ptr())
        torch.cuda.synchronize()
        got = dict(out=out.cpu().numpy(), V=sw.swconv_debug_copy_V(plan, C), M=sw.swconv_debug_copy_M(plan, K))
        sw.swconv_backward(plan, 0, xd.data_ptr(), gd.data_ptr(), din.data_ptr(), dv.data_ptr())
        torch.cuda.synchronize()
        got.update(din=din.cpu().numpy(), dvals=dv.cpu().numpy()[:len(va)], dZ=sw.swconv_debug_copy_dZ(plan, K),
                   dV=sw.swconv_debug_copy_dV(plan, C))
    finally:
        sw.swconv_plan_destroy(plan)
    for name in ("V", "M", "out", "dZ", "dV", "din", "dvals"):
        assert not np.isnan(got[name]).any(), name + " not fully overwritten"
        e = relerr(got[name], ref[name])
        print("  %-5s max rel err %.3g" % (name, e), flush=True)
        assert e <= RTOL, name


def test_alexnet_conv2_group_full_size_f4x4():
    cfg, x, rp, ci, va = synth.make_layer("alexnet_conv2g_n32_f4r5")
    N, C, H, W, K, pad = (cfg[k] for k in ("N", "C", "H", "W", "K", "pad"))
    G = np.random.default_rng(cfg["seed"] + 5).standard_normal((N, K, cfg["Ho"], cfg["Wo"])).astype(np.float32)
    o64, _, _ = oracle.forward_f64(x, rp, ci, va, K, 4, 5, pad, want_VM=False)
    din64, dvals64, _, _ = oracle.backward_f64(x, rp, ci, va, G, K, 4, 5, pad, want_ZV=False)
    plan = sw.swconv_plan_create(N, C, H, W, K, 4, 5, pad)
    try:
        sw.swconv_set_weights(plan, rp, ci, va)
        xd, gd = torch.from_numpy(x).cuda(), torch.from_numpy(G).cuda()
        out = torch.full(o64.shape, float("nan"), dtype=torch.float32, device="cuda")
        din = torch.full(x.shape, float("nan"), dtype=torch.float32, device="cuda")
        dv = torch.full((len(va),), float("nan"), device="cuda")
        sw.swconv_forward(plan, 0, xd.data_ptr(), out.data_ptr())
        sw.swconv_backward(plan, 0, 0, gd.data_ptr(), din.data_ptr(), dv.data_ptr())
        torch.cuda.synchronize()
        for name, got, ref in (("out", out, o64), ("din", din, din64), ("dvals", dv, dvals64)):
            e = relerr(got.cpu().numpy(), ref)
            print("  %-5s max rel err %.3g" % (name, e), flush=True)
            assert e <= RTOL, name
    finally:
        sw.swconv_plan_destroy(plan)


def test_other_filter_sizes_are_refused():
    for m, r in ((3, 5), (2, 7), (3, 3), (6, 3)):
        with pytest.raises(sw.SwconvError) as e:
            sw.swconv_plan_create(1, 4, 16, 16, 4, m, r, 1)
        assert e.value.status == sw.SWCONV_EUNSUPPORTED
