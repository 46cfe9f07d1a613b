"""Host-side logic of libswconv that needs no GPU: exported symbols, argument checking, CSR
validation, and the bit-exact round trip of the re-packed weight layout."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_1702_08597_amd import binding as sw
from paper_1702_08597_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "swconv.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = sorted(set(re.findall(r"\b(swconv_[a-z_A-Z0-9]+)\s*\(", header)))
    assert sorted(sw.EXPORTS) == declared
    L = sw.lib()
    for name in declared:
        assert getattr(L, name) is not None


def test_status_strings():
    for s in range(6):
        assert isinstance(sw.swconv_status_string(s), str) and sw.swconv_status_string(s)
    assert "unknown" in sw.swconv_status_string(99)


@pytest.mark.parametrize("args,status", [
    ((0, 4, 8, 8, 4, 4, 3, 1), sw.SWCONV_EINVAL),
    ((1, 4, 8, 8, 0, 4, 3, 1), sw.SWCONV_EINVAL),
    ((1, 4, 8, 8, 4, 4, 3, -1), sw.SWCONV_EINVAL),
    ((1, 4, 2, 8, 4, 4, 3, 0), sw.SWCONV_EINVAL),      # Ho < 1
    ((1, 4, 8, 8, 4, 3, 3, 1), sw.SWCONV_EUNSUPPORTED),  # F(3,3)
    ((1, 4, 8, 8, 4, 6, 5, 1), sw.SWCONV_EUNSUPPORTED),  # F(6,5): m = 2 and 4 are built for r = 5
    ((1, 4096, 8, 8, 4, 4, 3, 1), sw.SWCONV_EUNSUPPORTED),  # panel beyond LDS
    ((1, 639, 8, 8, 4, 4, 3, 1), sw.SWCONV_EUNSUPPORTED),   # the first channel count whose panel does not fit
])
def test_plan_create_rejects(args, status):
    with pytest.raises(sw.SwconvError) as e:
        sw.swconv_plan_create(*args)
    assert e.value.status == status


def test_largest_panel_is_accepted_and_packs():
    # C = 638: the 64-tile panel, the slice counter and the fewest slice descriptors just fit LDS
    pl = sw.swconv_plan_create(1, 638, 6, 6, 9, 4, 3, 1)
    try:
        rp, ci, va = synth.bernoulli_weights(36, 9, 638, 0.2, 12)
        assert sw.swconv_set_weights_status(pl, rp, ci, va) in (sw.SWCONV_OK, sw.SWCONV_EHIP)   # EHIP: no device here
        rp2, ci2, va2 = sw.swconv_debug_export_weights(pl, 9, int(rp[-1]))
        np.testing.assert_array_equal(ci2, ci)
        sw.swconv_debug_check_schedule(pl)
    finally:
        sw.swconv_plan_destroy(pl)


def test_plan_sizes():
    pl = sw.swconv_plan_create(32, 256, 13, 13, 384, 4, 3, 1)
    assert sw.swconv_plan_sizes(pl) == (36, 512, 13, 13)
    sw.swconv_plan_destroy(pl)
    pl = sw.swconv_plan_create(1, 256, 13, 13, 384, 2, 3, 1)
    assert sw.swconv_plan_sizes(pl) == (16, 49, 13, 13)
    sw.swconv_plan_destroy(pl)
    pl = sw.swconv_plan_create(32, 48, 27, 27, 128, 2, 5, 2)   # F(2x2,5x5): t = 6
    assert sw.swconv_plan_sizes(pl) == (36, 32 * 14 * 14, 27, 27)
    sw.swconv_plan_destroy(pl)
    sw.swconv_plan_destroy(None)


def test_image_strides_are_validated():
    pl = sw.swconv_plan_create(2, 4, 6, 6, 3, 2, 3, 1)
    try:
        sw.swconv_plan_set_image_strides(pl, 2 * 4 * 36, 2 * 3 * 36)
        sw.swconv_plan_set_image_strides(pl, 0, 0)                     # back to dense
        for bad in ((4 * 36 - 1, 0), (0, 3 * 36 - 1), (-5, 0), (2 ** 40, 0), (0, 2 ** 40)):
            with pytest.raises(sw.SwconvError) as e:
                sw.swconv_plan_set_image_strides(pl, *bad)
            assert e.value.status == sw.SWCONV_EINVAL
    finally:
        sw.swconv_plan_destroy(pl)


def _tiny_plan():
    return sw.swconv_plan_create(1, 4, 6, 6, 3, 2, 3, 1), 16, 3, 4


def test_set_weights_rejects_malformed_csr():
    pl, P, K, C = _tiny_plan()
    rows = P * K
    good_rp = np.arange(rows + 1, dtype=np.int32) * 2
    good_ci = np.tile(np.array([1, 3], dtype=np.int32), rows)
    good_va = np.ones(2 * rows, dtype=np.float32)
    ok = (sw.SWCONV_OK, sw.SWCONV_EHIP)  # EHIP: validated and packed, but no device to upload to
    assert sw.swconv_set_weights_status(pl, good_rp, good_ci, good_va) in ok

    bad = good_rp.copy(); bad[0] = 1
    assert sw.swconv_set_weights_status(pl, bad, good_ci, good_va) == sw.SWCONV_EINVAL
    bad = good_rp.copy(); bad[5] = bad[4] - 1
    assert sw.swconv_set_weights_status(pl, bad, good_ci, good_va) == sw.SWCONV_EINVAL
    bad = good_ci.copy(); bad[0:2] = [3, 1]          # unsorted
    assert sw.swconv_set_weights_status(pl, good_rp, bad, good_va) == sw.SWCONV_EINVAL
    bad = good_ci.copy(); bad[0:2] = [1, 1]          # duplicate
    assert sw.swconv_set_weights_status(pl, good_rp, bad, good_va) == sw.SWCONV_EINVAL
    bad = good_ci.copy(); bad[7] = C                 # out of range
    assert sw.swconv_set_weights_status(pl, good_rp, bad, good_va) == sw.SWCONV_EINVAL
    bad = good_ci.copy(); bad[6] = -1
    assert sw.swconv_set_weights_status(pl, good_rp, bad, good_va) == sw.SWCONV_EINVAL
    assert sw.lib().swconv_set_weights(pl, None, None, None) == sw.SWCONV_EINVAL
    # the earlier good weights survive failed calls
    rp, ci, va = sw.swconv_debug_export_weights(pl, K, 2 * rows)
    np.testing.assert_array_equal(rp, good_rp)
    np.testing.assert_array_equal(ci, good_ci)
    sw.swconv_plan_destroy(pl)


def test_export_before_set_weights_is_a_state_error():
    pl, P, K, C = _tiny_plan()
    with pytest.raises(sw.SwconvError) as e:
        sw.swconv_debug_export_weights(pl, K, 0)
    assert e.value.status == sw.SWCONV_ESTATE
    with pytest.raises(sw.SwconvError) as e:
        sw.swconv_plan_weight_stats(pl)
    assert e.value.status == sw.SWCONV_ESTATE
    assert sw.lib().swconv_forward(pl, None, ctypes.c_void_p(8), ctypes.c_void_p(16)) == sw.SWCONV_ESTATE
    assert sw.lib().swconv_forward(pl, None, None, None) == sw.SWCONV_EINVAL
    sw.swconv_plan_destroy(pl)


@pytest.mark.parametrize("K,C,m,density,seed", [(384, 256, 4, 0.10, 1), (7, 5, 2, 0.5, 2), (13, 33, 4, 0.9, 3),
                                                (5, 9, 4, 0.0, 4), (6, 6, 2, 1.0, 5)])
def test_packed_weights_round_trip_bit_exact(K, C, m, density, seed):
    P = (m + 2) ** 2
    pl = sw.swconv_plan_create(2, C, 13, 13, K, m, 3, 1)
    rp, ci, va = synth.bernoulli_weights(P, K, C, density, seed)
    # include stored zeros and negative zeros: they must survive as stored entries
    if va.size > 4:
        va[1], va[3] = 0.0, -0.0
    assert sw.swconv_set_weights_status(pl, rp, ci, va) in (sw.SWCONV_OK, sw.SWCONV_EHIP)
    rp2, ci2, va2 = sw.swconv_debug_export_weights(pl, K, int(rp[-1]))
    np.testing.assert_array_equal(rp2, rp)
    np.testing.assert_array_equal(ci2, ci)
    np.testing.assert_array_equal(va2.view(np.uint32), va.view(np.uint32))
    st = sw.swconv_plan_weight_stats(pl)
    assert st["nnz"] == int(rp[-1]) and st["padded_nnz"] >= st["nnz"] and st["work_items"] >= 1
    sw.swconv_debug_check_schedule(pl)
    sw.swconv_plan_destroy(pl)


def test_skewed_weights_pack_and_balance():
    K, C, P = 384, 384, 36
    pl = sw.swconv_plan_create(64, C, 13, 13, K, 4, 3, 1)
    rp, ci, va = synth.skewed_weights(P, K, C, 77)
    assert sw.swconv_set_weights_status(pl, rp, ci, va) in (sw.SWCONV_OK, sw.SWCONV_EHIP)
    rp2, ci2, va2 = sw.swconv_debug_export_weights(pl, K, int(rp[-1]))
    np.testing.assert_array_equal(rp2, rp)
    np.testing.assert_array_equal(ci2, ci)
    np.testing.assert_array_equal(va2.view(np.uint32), va.view(np.uint32))
    st = sw.swconv_plan_weight_stats(pl)
    # sorted slices keep the padding small even with a Zipf row-length profile
    assert st["padded_nnz"] <= 1.25 * st["nnz"]
    sw.swconv_debug_check_schedule(pl)
    sw.swconv_plan_destroy(pl)


@pytest.mark.parametrize("N,C,H,W,K,m", [(1, 3, 5, 5, 1, 2), (64, 384, 13, 13, 384, 4), (3, 638, 6, 6, 7, 2),
                                         (2, 16, 56, 56, 9, 4), (200, 8, 4, 4, 5, 4),
                                         (1, 8, 6, 6, 2100, 2),      # more slices per position than one item holds
                                         (1, 638, 6, 6, 70, 2)])     # little LDS left for descriptors
@pytest.mark.parametrize("density", [0.0, 0.1, 1.0])
def test_schedule_is_a_partition(N, C, H, W, K, m, density):
    P = (m + 2) ** 2
    pl = sw.swconv_plan_create(N, C, H, W, K, m, 3, 1)
    rp, ci, va = synth.bernoulli_weights(P, K, C, density, 11)
    assert sw.swconv_set_weights_status(pl, rp, ci, va) in (sw.SWCONV_OK, sw.SWCONV_EHIP)
    sw.swconv_debug_check_schedule(pl)
    sw.swconv_plan_destroy(pl)


@pytest.mark.parametrize("seed", range(6))
@pytest.mark.parametrize("env", [{}, {"SWCONV_SPMM_SECOND_SHARE": "40"}, {"SWCONV_SPMM_WGS": "37"},
                                 {"SWCONV_SPMM_WGS": "301", "SWCONV_SPMM_SECOND_SHARE": "55", "SWCONV_SPMM_WAVES": "8"}])
def test_schedule_is_a_partition_for_random_shapes_and_cost_settings(seed, env, monkeypatch):
    # the cut into ranges (budgets that depend on where a range's workgroup sits, the re-cut when
    # fewer workgroups are used than assumed) must hand out every (position, tile block, slice) once
    for k, v in env.items():
        monkeypatch.setenv(k, v)
    rng = np.random.default_rng(9000 + seed)
    for _ in range(4):
        m, r = [(2, 3), (4, 3), (2, 5), (4, 5)][int(rng.integers(0, 4))]
        N, C, K = int(rng.integers(1, 70)), int(rng.integers(1, 400)), int(rng.integers(1, 500))
        H, W = int(rng.integers(r, 30)), int(rng.integers(r, 30))
        P = (m + r - 1) ** 2
        pl = sw.swconv_plan_create(N, C, H, W, K, m, r, r // 2)
        if rng.random() < 0.3:
            rp, ci, va = synth.skewed_weights(P, K, C, int(rng.integers(1 << 30)))
        else:
            rp, ci, va = synth.bernoulli_weights(P, K, C, float(rng.choice([0.0, 0.02, 0.1, 0.5, 1.0])),
                                                 int(rng.integers(1 << 30)))
        assert sw.swconv_set_weights_status(pl, rp, ci, va) in (sw.SWCONV_OK, sw.SWCONV_EHIP)
        sw.swconv_debug_check_schedule(pl)
        rp2, ci2, va2 = sw.swconv_debug_export_weights(pl, K, int(rp[-1]))
        np.testing.assert_array_equal(rp2, rp)
        np.testing.assert_array_equal(ci2, ci)
        np.testing.assert_array_equal(va2.view(np.uint32), va.view(np.uint32))
        sw.swconv_plan_destroy(pl)


def test_product_path_never_touches_the_oracle():
    """The package (binding, build script, input generators, kernels) must not import, include, load or run
    anything under oracle/: the oracle is the checker, and a product path through it would void every parity test."""
    pkg = os.path.join(ROOT, "paper_1702_08597_amd")
    for folder, _, files in os.walk(pkg):
        for name in files:
            if not name.endswith((".py", ".hip", ".hpp", ".inc", ".h")):
                continue
            text = open(os.path.join(folder, name), encoding="utf-8", errors="replace").read()
            assert not re.search(r"\boracle\b(?!s)", text.replace("the CPU oracle", "")), "%s names the oracle" % name
    header = open(os.path.join(ROOT, "include", "swconv.h")).read()
    assert "oracle" not in header
