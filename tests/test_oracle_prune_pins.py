"""Pins of the oracle's pruning step (Section 4.2, Eq. 8 and Eq. 9) to what the paper states.

The paper gives the thresholding function T_{eps,beta} in closed form and three values of the effective
threshold on |w|: eps/beta at gradient magnitude 0, eps at 1 - beta, 0 as the magnitude goes to infinity,
with eps = 1e-4 and beta = 0.1 the values it recommends.  The update is plain SGD on L + lambda*|w|_1.
"""
import numpy as np

import oracle

EPS, BETA = 1e-4, 0.1


def one_row(vals, grad, eta=0.0, lam=0.0, dtype=np.float64):
    n = len(vals)
    rp = np.array([0, n], dtype=np.int32)
    ci = np.arange(n, dtype=np.int32)
    return oracle.prune_step(rp, ci, np.asarray(vals), np.asarray(grad), eta, lam, EPS, BETA, dtype)


def test_threshold_values_the_paper_states():
    # eta = 0: the step leaves w alone and only T acts.  Effective threshold on |w| is eps / (|g| + beta).
    for g, thr in ((0.0, EPS / BETA), (1.0 - BETA, EPS), (1e9, 1e-13)):
        below, above = thr * (1 - 1e-6), thr * (1 + 1e-6)
        upd, (rp, ci, va) = one_row([below, -below, above, -above], [g, -g, g, -g])
        assert list(upd[:2]) == [0.0, 0.0] and list(upd[2:]) == [above, -above]
        assert list(rp) == [0, 2] and list(ci) == [2, 3] and list(va) == [above, -above]


def test_update_is_sgd_on_loss_plus_l1():
    w = np.array([0.5, -0.25, 0.125, 0.0])
    g = np.array([0.1, 0.2, -0.3, 0.05])
    eta, lam = 0.01, 0.5
    upd, _ = one_row(w, g, eta, lam)
    want = w - eta * (g + lam * np.sign(w))
    np.testing.assert_allclose(upd[:3], want[:3], rtol=1e-15)
    # a stored zero has subgradient 0 of the L1 term: it moves by -eta*g = -5e-4, and |w'|(|g|+beta) = 7.5e-5 < eps
    assert upd[3] == 0.0


def test_compaction_keeps_order_and_row_structure():
    rng = np.random.default_rng(1)
    rows, C = 37, 23
    mask = rng.random((rows, C)) < 0.4
    counts = mask.sum(1)
    rp = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    ci = np.nonzero(mask)[1].astype(np.int32)
    w = rng.standard_normal(len(ci)) * 2e-3
    g = rng.standard_normal(len(ci)) * 0.05
    upd, (rp2, ci2, va2) = oracle.prune_step(rp, ci, w, g, 0.01, 1e-3, EPS, BETA, np.float64)
    wn = w - 0.01 * (g + 1e-3 * np.sign(w))
    keep = ~(np.abs(wn) * (np.abs(g) + BETA) < EPS)
    assert 0 < keep.sum() < len(w)
    # the oracle fuses w - eta*(.) into one rounding, numpy rounds twice: values agree to an ulp
    np.testing.assert_array_equal(upd != 0, keep)
    np.testing.assert_allclose(upd, np.where(keep, wn, 0.0), rtol=1e-14, atol=0)
    np.testing.assert_array_equal(ci2, ci[keep])
    np.testing.assert_array_equal(va2, upd[keep])
    np.testing.assert_array_equal(rp2, np.concatenate([[0], np.cumsum(np.add.reduceat(keep, rp[:-1]) * (counts > 0))]))


def test_float_instantiation_rounds_like_float():
    rng = np.random.default_rng(2)
    n = 5000
    w = (rng.standard_normal(n) * 2e-3).astype(np.float32)
    g = (rng.standard_normal(n) * 0.05).astype(np.float32)
    eta, lam = np.float32(0.01), np.float32(1e-3)
    upd, (rp, ci, va) = one_row(w, g, eta, lam, np.float32)
    step = g + lam * np.sign(w)                                        # one rounding
    wn = (w.astype(np.float64) - eta.astype(np.float64) * step.astype(np.float64)).astype(np.float32)  # fused
    keep = ~(np.abs(wn) * (np.abs(g) + np.float32(BETA)) < np.float32(EPS))
    np.testing.assert_array_equal(upd, np.where(keep, wn, np.float32(0)))
    assert rp[1] == keep.sum()
