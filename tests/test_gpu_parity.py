"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element.

Tolerance (norm-relative over the whole tensor, as fp32 summation order is not fixed by the
paper): max|gpu - oracle64| <= rtol * max|oracle64| with rtol = 1e-5 for F(2x2,3x3) and 1e-4 for
F(4x4,3x3).  Integer-valued data must match bit for bit (V, M and the output).
"""
import numpy as np
import pytest
import torch

import oracle
from paper_1702_08597_amd import binding as sw
from paper_1702_08597_amd import synth

pytestmark = pytest.mark.gpu

RTOL = {2: 1e-5, 4: 1e-4}


class GpuLayer:
    """Plan + device buffers for one layer shape (torch is used for device memory and streams only)."""

    def __init__(self, N, C, H, W, K, m, r=3, pad=1):
        self.shape = (N, C, H, W, K, m, r, pad)
        self.plan = sw.swconv_plan_create(N, C, H, W, K, m, r, pad)
        self.P, self.T, self.Ho, self.Wo = sw.swconv_plan_sizes(self.plan)
        self.out = torch.full((N, K, self.Ho, self.Wo), float("nan"), dtype=torch.float32, device="cuda")

    def set_weights(self, rp, ci, va):
        sw.swconv_set_weights(self.plan, rp, ci, va)

    def forward(self, x, stream=None, dense=False):
        self.x = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).cuda()
        self.out.fill_(float("nan"))
        torch.cuda.synchronize()
        st = stream if stream is not None else torch.cuda.current_stream()
        fn = sw.swconv_forward_dense if dense else sw.swconv_forward
        fn(self.plan, st.cuda_stream, self.x.data_ptr(), self.out.data_ptr())
        st.synchronize()
        return self.out.cpu().numpy()

    def V(self):
        return sw.swconv_debug_copy_V(self.plan, self.shape[1])

    def M(self):
        return sw.swconv_debug_copy_M(self.plan, self.shape[4])

    def close(self):
        sw.swconv_plan_destroy(self.plan)


def relerr(a, ref):
    scale = np.abs(ref).max()
    return np.abs(a.astype(np.float64) - ref).max() / (scale if scale > 0 else 1.0)


def check_against_oracle(N, C, H, W, K, m, pad, x, rp, ci, va, stages=True):
    print("case N=%d C=%d H=%d W=%d K=%d m=%d pad=%d nnz=%d" % (N, C, H, W, K, m, pad, rp[-1]), flush=True)
    o64, V64, M64 = oracle.forward_f64(x, rp, ci, va, K, m, 3, pad, want_VM=stages)
    L = GpuLayer(N, C, H, W, K, m, 3, pad)
    try:
        L.set_weights(rp, ci, va)
        out = L.forward(x)
        assert not np.isnan(out).any(), "output not fully overwritten"
        if stages:
            assert relerr(L.V(), V64) <= RTOL[m]
            assert relerr(L.M(), M64) <= RTOL[m]
        err = relerr(out, o64)
        print("  max rel err %.3g (tol %.0e)" % (err, RTOL[m]), flush=True)
        assert err <= RTOL[m]
    finally:
        L.close()
    return out


SMALL = [
    # N, C, H, W, K, m, pad : several tile blocks + ragged tails, odd channel counts
    (9, 19, 13, 13, 10, 2, 1),
    (5, 7, 13, 11, 13, 4, 1),
    (2, 3, 56, 40, 5, 4, 1),
    (3, 5, 9, 17, 6, 2, 0),
    (1, 1, 1, 1, 1, 2, 1),     # one pixel, one tile
    (1, 2, 3, 3, 3, 4, 0),     # Ho = 1
    (70, 4, 4, 4, 4, 4, 1),    # one tile per image, many images
    (1, 638, 6, 6, 2, 2, 1),   # largest channel count the panel holds
    (1, 638, 6, 6, 70, 2, 1),  # ... with more slices per position than its LDS holds descriptors for
    (2, 6, 9, 9, 1100, 4, 1),  # more slices per position than one work item holds
]


@pytest.mark.parametrize("N,C,H,W,K,m,pad", SMALL)
def test_small_shapes_all_stages(N, C, H, W, K, m, pad):
    P = (m + 2) ** 2
    x = synth.activations(N, C, H, W, 100 + N + C)
    rp, ci, va = synth.bernoulli_weights(P, K, C, 0.3, 200 + K)
    check_against_oracle(N, C, H, W, K, m, pad, x, rp, ci, va)


@pytest.mark.parametrize("m", [2, 4])
def test_integer_data_bit_exact(m):
    N, C, H, W, K = 6, 24, 13, 13, 22
    x, rp, ci, va = synth.integer_case(N, C, H, W, K, m, 3, 0.4, 300 + m)
    o64, V64, M64 = oracle.forward_f64(x, rp, ci, va, K, m)
    L = GpuLayer(N, C, H, W, K, m)
    try:
        L.set_weights(rp, ci, va)
        out = L.forward(x)
        np.testing.assert_array_equal(L.V().astype(np.float64), V64)
        np.testing.assert_array_equal(L.M().astype(np.float64), M64)
        np.testing.assert_array_equal(out.astype(np.float64), o64)
        rp2, ci2, va2 = sw.swconv_debug_export_weights(L.plan, K, int(rp[-1]))
        np.testing.assert_array_equal(rp2, rp)
        np.testing.assert_array_equal(ci2, ci)
        np.testing.assert_array_equal(va2.view(np.uint32), va.view(np.uint32))
    finally:
        L.close()


@pytest.mark.parametrize("m", [2, 4])
def test_zero_weights_exact_zero_and_reset(m):
    N, C, H, W, K = 3, 8, 13, 13, 9
    P = (m + 2) ** 2
    x = synth.activations(N, C, H, W, 5)
    L = GpuLayer(N, C, H, W, K, m)
    try:
        L.set_weights(np.zeros(P * K + 1, dtype=np.int32), np.zeros(0, np.int32), np.zeros(0, np.float32))
        out = L.forward(x)
        assert np.all(out == 0.0)
        # new pattern on the same plan, then empty again
        rp, ci, va = synth.bernoulli_weights(P, K, C, 0.5, 6)
        L.set_weights(rp, ci, va)
        o64 = oracle.forward_f64(x, rp, ci, va, K, m, want_VM=False)[0]
        assert relerr(L.forward(x), o64) <= RTOL[m]
        L.set_weights(np.zeros(P * K + 1, dtype=np.int32), np.zeros(0, np.int32), np.zeros(0, np.float32))
        assert np.all(L.forward(x) == 0.0)
    finally:
        L.close()


def test_row_permutation_is_bit_exact_and_runs_are_deterministic():
    m, N, C, H, W, K = 4, 8, 32, 13, 13, 24
    P = 36
    x = synth.activations(N, C, H, W, 8)
    rp, ci, va = synth.bernoulli_weights(P, K, C, 0.2, 9)
    import scipy.sparse
    dense = scipy.sparse.csr_matrix((va, ci, rp), shape=(P * K, C)).toarray().reshape(P, K, C)
    perm = np.random.default_rng(10).permutation(K)
    csr_p = synth.dense_to_csr(dense[:, perm] != 0, dense[:, perm])
    L = GpuLayer(N, C, H, W, K, m)
    try:
        L.set_weights(rp, ci, va)
        a = L.forward(x)
        b = L.forward(x)
        np.testing.assert_array_equal(a, b)
        side = torch.cuda.Stream()
        c = L.forward(x, stream=side)
        np.testing.assert_array_equal(a, c)
        L.set_weights(*csr_p)
        d = L.forward(x)
        np.testing.assert_array_equal(d, a[:, perm])
    finally:
        L.close()


def test_full_rows_stored_zeros_and_lone_rows_through_the_sparse_path():
    """Stream edge cases of the packed layout: every row full (many batches per slice), explicit
    stored zeros, and positions where one row is full and all others are empty (a slice whose
    other rows are pure padding; all-empty slices next to it)."""
    m, N, C, H, W, K = 4, 5, 70, 9, 9, 9
    P = 36
    rng = np.random.default_rng(77)
    x = synth.activations(N, C, H, W, 78)
    dense = rng.normal(0, 0.05, size=(P, K, C)).astype(np.float32)
    mask = np.ones((P, K, C), dtype=bool)
    dense[:, :, ::7] = 0.0          # stored zeros: kept in the pattern
    mask[1::2] = False              # odd positions: only row 3 is populated
    mask[1::2, 3, :] = True
    rp, ci, va = synth.dense_to_csr(mask, dense)
    assert (va == 0).any()
    check_against_oracle(N, C, H, W, K, m, 1, x, rp, ci, va)


FULL = ["alexnet_conv3_n1_f2", "alexnet_conv3_n32_f4", "alexnet_conv4_n64_f4", "alexnet_conv5_n64_f4",
        "conv4_skewed_n64_f4"]


@pytest.mark.parametrize("name", FULL)
def test_full_size_configs(name):
    cfg, x, rp, ci, va = synth.make_layer(name)
    check_against_oracle(cfg["N"], cfg["C"], cfg["H"], cfg["W"], cfg["K"], cfg["m"], cfg["pad"], x, rp, ci, va,
                         stages=(cfg["N"] <= 32))


@pytest.mark.parametrize("density", synth.DENSITY_SWEEP)
@pytest.mark.parametrize("name", ["alexnet_conv3_n64_f4", "alexnet_conv4_n64_f4", "alexnet_conv5_n64_f4"])
def test_density_sweep(name, density):
    # the three 3x3 layers at batch 64, each at every density of the sweep (Table 1's sparsity range)
    cfg, x, rp, ci, va = synth.make_layer(name, density=density)
    check_against_oracle(cfg["N"], cfg["C"], cfg["H"], cfg["W"], cfg["K"], cfg["m"], cfg["pad"], x, rp, ci, va,
                         stages=False)


FUSED4 = [
    # N, C, H, W, K, pad, density: F(4x4,3x3) with steps 2 and 3 in one kernel (C a multiple of 4, at most 256)
    (5, 8, 13, 13, 10, 1, 0.3),       # ragged 13 x 13 tiles, one row chunk, K below a slice multiple
    (3, 64, 16, 16, 70, 1, 0.1),      # whole tiles (Wo = 16), two row chunks, the second mostly padding rows
    (2, 256, 9, 12, 130, 1, 0.3),     # rows longer than two batches (mean 77 entries), three row chunks
    (9, 4, 8, 8, 64, 0, 1.0),         # one direct load per panel, full rows, no padding: Ho = Wo = 6
    (1, 256, 5, 7, 5, 1, 0.05),       # the largest C the two panel arrays hold; many empty rows
    (2, 200, 6, 6, 9, 1, 0.2),        # C not a multiple of 64: waves without a row group in the last direct load
    (30, 12, 4, 4, 4, 1, 0.5),        # one tile per image: 30 image parts in the staging area of a wave
]


@pytest.mark.parametrize("N,C,H,W,K,pad,density", FUSED4)
def test_f4x4_product_and_output_transform_in_one_kernel(N, C, H, W, K, pad, density, monkeypatch):
    m = 4
    x = synth.activations(N, C, H, W, 8100 + C)
    rp, ci, va = synth.bernoulli_weights(36, K, C, density, 8200 + K)
    outs = {}
    for mode in ("2", "0"):
        with monkeypatch.context() as mp:
            mp.setenv("SWCONV_FUSE_OUTPUT", mode)
            L = GpuLayer(N, C, H, W, K, m, 3, pad)
            try:
                L.set_weights(rp, ci, va)
                outs[mode] = L.forward(x).copy()
                ms = sw.swconv_profile_forward(L.plan, torch.cuda.current_stream().cuda_stream, L.x.data_ptr(),
                                               L.out.data_ptr(), 2)
                assert (ms[2] == 0) == (mode == "2"), "the fused kernel must run exactly when asked for"
                if mode == "2":
                    np.testing.assert_array_equal(L.out.cpu().numpy(), outs[mode])   # deterministic
            finally:
                L.close()
    with monkeypatch.context() as mp:
        mp.setenv("SWCONV_FUSE_OUTPUT", "2")
        got = check_against_oracle(N, C, H, W, K, m, pad, x, rp, ci, va)            # V, M (step 2 run alone) and output
    np.testing.assert_array_equal(got, outs["2"])
    scale = np.abs(outs["0"]).max()
    assert np.abs(outs["2"] - outs["0"]).max() <= 2 * RTOL[m] * scale


def test_f4x4_fused_kernel_integer_data_bit_exact_and_skewed_rows(monkeypatch):
    monkeypatch.setenv("SWCONV_FUSE_OUTPUT", "2")
    N, C, H, W, K, m = 6, 24, 13, 13, 150, 4
    x, rp, ci, va = synth.integer_case(N, C, H, W, K, m, 3, 0.4, 8301)
    o64, _, _ = oracle.forward_f64(x, rp, ci, va, K, m, want_VM=False)
    L = GpuLayer(N, C, H, W, K, m)
    try:
        L.set_weights(rp, ci, va)
        np.testing.assert_array_equal(L.forward(x).astype(np.float64), o64)
        ms = sw.swconv_profile_forward(L.plan, 0, L.x.data_ptr(), L.out.data_ptr(), 1)
        assert ms[2] == 0
    finally:
        L.close()
    # rows from empty to full inside one position (slices whose rows differ widely in length)
    N, C, K = 4, 128, 96
    x = synth.activations(N, C, H, W, 8302)
    rp, ci, va = synth.skewed_weights(36, K, C, 8303)
    check_against_oracle(N, C, H, W, K, m, 1, x, rp, ci, va)


def test_vgg_shaped_layer_full_size_through_the_fused_f4x4_kernel(monkeypatch):
    # the launch configuration the profiles of the fused kernel were taken in: 98 tile blocks x 4 row chunks
    monkeypatch.setenv("SWCONV_FUSE_OUTPUT", "2")
    cfg, x, rp, ci, va = synth.make_layer("vgg_56_n32_f4")
    out = check_against_oracle(cfg["N"], cfg["C"], cfg["H"], cfg["W"], cfg["K"], cfg["m"], cfg["pad"], x, rp, ci, va,
                               stages=False)
    plan = sw.swconv_plan_create(cfg["N"], cfg["C"], cfg["H"], cfg["W"], cfg["K"], cfg["m"], 3, cfg["pad"])
    try:
        sw.swconv_set_weights(plan, rp, ci, va)
        xd = torch.from_numpy(x).cuda()
        od = torch.empty(out.shape, device="cuda")
        ms = sw.swconv_profile_forward(plan, 0, xd.data_ptr(), od.data_ptr(), 1)
        assert ms[2] == 0, "the fused kernel did not run"
        np.testing.assert_array_equal(od.cpu().numpy(), out)
    finally:
        sw.swconv_plan_destroy(plan)


def test_vgg_shaped_layer_full_size():
    cfg, x, rp, ci, va = synth.make_layer("vgg_56_n32_f4")
    check_against_oracle(cfg["N"], cfg["C"], cfg["H"], cfg["W"], cfg["K"], cfg["m"], cfg["pad"], x, rp, ci, va,
                         stages=False)


@pytest.mark.parametrize("N,C,H,W,K,m", [(4, 40, 13, 13, 50, 4), (3, 17, 10, 9, 130, 2), (64, 384, 13, 13, 384, 4)])
def test_dense_mfma_comparison_path(N, C, H, W, K, m):
    P = (m + 2) ** 2
    x = synth.activations(N, C, H, W, 50)
    wf = synth.dense_weights(P, K, C, 51)
    rowptr = (np.arange(P * K + 1, dtype=np.int64) * C).astype(np.int32)
    colidx = np.tile(np.arange(C, dtype=np.int32), P * K)
    o64 = oracle.forward_f64(x, rowptr, colidx, wf.reshape(-1), K, m, want_VM=False)[0]
    L = GpuLayer(N, C, H, W, K, m)
    try:
        sw.swconv_set_weights_dense(L.plan, wf)
        out = L.forward(x, dense=True)
        err = relerr(out, o64)
        print("dense path max rel err %.3g" % err, flush=True)
        assert err <= RTOL[m]
    finally:
        L.close()


def test_profile_forward_returns_positive_stage_times_and_same_output():
    cfg, x, rp, ci, va = synth.make_layer("alexnet_conv3_n32_f4")
    L = GpuLayer(cfg["N"], cfg["C"], cfg["H"], cfg["W"], cfg["K"], cfg["m"])
    try:
        L.set_weights(rp, ci, va)
        ref = L.forward(x)
        L.out.fill_(0)
        torch.cuda.synchronize()
        ms = sw.swconv_profile_forward(L.plan, torch.cuda.current_stream().cuda_stream, L.x.data_ptr(),
                                       L.out.data_ptr(), 5)
        assert np.all(ms > 0) and np.all(ms < 100)
        np.testing.assert_array_equal(L.out.cpu().numpy(), ref)
    finally:
        L.close()


def test_workspaces_just_below_the_4_gib_offset_limit_on_sampled_images():
    # V and M are addressed with 32-bit byte offsets; this plan's workspaces are 4.13e9 bytes each
    # (2**32 = 4.29e9).  The layer treats images independently, so the oracle checks the first, a
    # middle and the last images - the last ones sit at the top of the offset range.
    N, C, H, W, K, m = 28000, 64, 13, 13, 64, 4
    P, T, Ho, Wo = 36, N * 16, 13, 13
    assert 36 * 64 * T * 4 > 0.96 * 2 ** 32
    plan = sw.swconv_plan_create(N, C, H, W, K, m, 3, 1)
    try:
        assert sw.swconv_plan_sizes(plan) == (P, T, Ho, Wo)
        rp, ci, va = synth.bernoulli_weights(P, K, C, 0.2, 4401)
        sw.swconv_set_weights(plan, rp, ci, va)
        gen = torch.Generator(device="cuda").manual_seed(4402)
        xd = torch.randn((N, C, H, W), device="cuda", generator=gen).clamp_(min=0)
        gd = torch.randn((N, K, Ho, Wo), device="cuda", generator=gen)
        out = torch.full((N, K, Ho, Wo), float("nan"), device="cuda")
        din = torch.full((N, C, H, W), float("nan"), device="cuda")
        print("forward", flush=True)
        sw.swconv_forward(plan, 0, xd.data_ptr(), out.data_ptr())
        torch.cuda.synchronize()
        print("backward", flush=True)
        sw.swconv_backward(plan, 0, xd.data_ptr(), gd.data_ptr(), din.data_ptr(), 0)
        torch.cuda.synchronize()
        assert not torch.isnan(out).any().item() and not torch.isnan(din).any().item()
        for n0 in (0, 13999, N - 3):
            xs, gs = xd[n0:n0 + 3].cpu().numpy(), gd[n0:n0 + 3].cpu().numpy()
            o64, _, _ = oracle.forward_f64(xs, rp, ci, va, K, m, 3, 1, want_VM=False)
            din64, _, _, _ = oracle.backward_f64(xs, rp, ci, va, gs, K, m, 3, 1, want_ZV=False)
            assert relerr(out[n0:n0 + 3].cpu().numpy(), o64) <= RTOL[m]
            assert relerr(din[n0:n0 + 3].cpu().numpy(), din64) <= RTOL[m]
    finally:
        sw.swconv_plan_destroy(plan)
    # one more image row of tiles and the plan is refused, not wrapped around
    with pytest.raises(sw.SwconvError) as e:
        sw.swconv_plan_create(30000, C, H, W, K, m, 3, 1)
    assert e.value.status == sw.SWCONV_EUNSUPPORTED


def test_schedule_settings_do_not_change_a_single_bit(monkeypatch):
    # how the work is cut into ranges decides who computes a row, not how the row is summed
    N, C, H, W, K, m = 9, 40, 13, 13, 70, 4
    x = synth.activations(N, C, H, W, 5101)
    rp, ci, va = synth.skewed_weights(36, K, C, 5102)
    outs = []
    for env in ({}, {"SWCONV_SPMM_WGS": "37"}, {"SWCONV_SPMM_SECOND_SHARE": "40"},
                {"SWCONV_SPMM_WAVES": "8", "SWCONV_SPMM_WGS": "301", "SWCONV_SPMM_SLICE_COST": "5"}):
        with monkeypatch.context() as mp:
            for k, v in env.items():
                mp.setenv(k, v)
            L = GpuLayer(N, C, H, W, K, m)
            try:
                L.set_weights(rp, ci, va)
                sw.swconv_debug_check_schedule(L.plan)
                outs.append(L.forward(x).copy())
            finally:
                L.close()
    for o in outs[1:]:
        np.testing.assert_array_equal(o.view(np.uint32), outs[0].view(np.uint32))
    o64, _, _ = oracle.forward_f64(x, rp, ci, va, K, m, 3, 1, want_VM=False)
    assert relerr(outs[0], o64) <= RTOL[m]


def test_two_plans_on_two_streams_at_once():
    # plans own their workspaces and schedules; nothing is shared between them, so two layers
    # may be in flight together (forward and backward), each on a stream of its own
    shapes = [(6, 24, 13, 13, 20, 4, 3, 1), (4, 12, 27, 27, 16, 2, 5, 2)]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    jobs = []
    for (N, C, H, W, K, m, r, pad), st in zip(shapes, streams):
        P = (m + r - 1) ** 2
        Ho, Wo = H + 2 * pad - r + 1, W + 2 * pad - r + 1
        x = synth.activations(N, C, H, W, 6100 + C)
        rp, ci, va = synth.bernoulli_weights(P, K, C, 0.3, 6200 + K)
        G = np.random.default_rng(6300 + K).standard_normal((N, K, Ho, Wo)).astype(np.float32)
        plan = sw.swconv_plan_create(N, C, H, W, K, m, r, pad)
        sw.swconv_set_weights(plan, rp, ci, va)
        jobs.append(dict(plan=plan, st=st, x=x, rp=rp, ci=ci, va=va, G=G, K=K, m=m, r=r, pad=pad,
                         xd=torch.from_numpy(x).cuda(), gd=torch.from_numpy(G).cuda(),
                         out=torch.full((N, K, Ho, Wo), float("nan"), device="cuda"),
                         din=torch.full((N, C, H, W), float("nan"), device="cuda"),
                         dv=torch.full((len(va),), float("nan"), device="cuda")))
    torch.cuda.synchronize()
    try:
        for rep in range(3):                      # interleaved launches, no synchronisation in between
            for j in jobs:
                sw.swconv_forward(j["plan"], j["st"].cuda_stream, j["xd"].data_ptr(), j["out"].data_ptr())
            for j in jobs:
                sw.swconv_backward(j["plan"], j["st"].cuda_stream, j["xd"].data_ptr(), j["gd"].data_ptr(),
                                   j["din"].data_ptr(), j["dv"].data_ptr())
        torch.cuda.synchronize()
        for j in jobs:
            tol = 1e-4
            o64, _, _ = oracle.forward_f64(j["x"], j["rp"], j["ci"], j["va"], j["K"], j["m"], j["r"], j["pad"], want_VM=False)
            din64, dv64, _, _ = oracle.backward_f64(j["x"], j["rp"], j["ci"], j["va"], j["G"], j["K"], j["m"], j["r"],
                                                    j["pad"], want_ZV=False)
            assert relerr(j["out"].cpu().numpy(), o64) <= tol
            assert relerr(j["din"].cpu().numpy(), din64) <= tol
            assert relerr(j["dv"].cpu().numpy(), dv64) <= tol
    finally:
        for j in jobs:
            sw.swconv_plan_destroy(j["plan"])


def test_forward_and_backward_replay_from_a_hip_graph():
    # the passes only launch kernels (no allocation, no memset), so a caller may capture them;
    # every replay must give what the eager call gives, bit for bit, with fresh inputs each time
    N, C, H, W, K, m = 6, 32, 13, 13, 24, 4
    rp, ci, va = synth.bernoulli_weights(36, K, C, 0.3, 7001)
    plan = sw.swconv_plan_create(N, C, H, W, K, m, 3, 1)
    try:
        sw.swconv_set_weights(plan, rp, ci, va)
        xs = [torch.from_numpy(synth.activations(N, C, H, W, 7100 + i)).cuda() for i in range(3)]
        gs = [torch.randn((N, K, 13, 13), device="cuda", generator=torch.Generator(device="cuda").manual_seed(7200 + i))
              for i in range(3)]
        x_in, g_in = torch.empty_like(xs[0]), torch.empty_like(gs[0])
        out, din = torch.empty((N, K, 13, 13), device="cuda"), torch.empty((N, C, H, W), device="cuda")
        dv = torch.empty((len(va),), device="cuda")

        def passes(stream):
            sw.swconv_forward(plan, stream, x_in.data_ptr(), out.data_ptr())
            sw.swconv_backward(plan, stream, 0, g_in.data_ptr(), din.data_ptr(), dv.data_ptr())   # reuses I_F

        eager = []
        for x, g in zip(xs, gs):        # also the warm-up: first-call set-up happens outside the capture
            x_in.copy_(x); g_in.copy_(g)
            passes(torch.cuda.current_stream().cuda_stream)
            torch.cuda.synchronize()
            eager.append((out.clone(), din.clone(), dv.clone()))
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            passes(torch.cuda.current_stream().cuda_stream)
        for rep in range(2):
            for (x, g), want in zip(zip(xs, gs), eager):
                x_in.copy_(x); g_in.copy_(g)
                out.fill_(float("nan")); din.fill_(float("nan")); dv.fill_(float("nan"))
                graph.replay()
                torch.cuda.synchronize()
                for got, ref in zip((out, din, dv), want):
                    assert torch.equal(got.view(torch.int32), ref.view(torch.int32))
    finally:
        sw.swconv_plan_destroy(plan)
