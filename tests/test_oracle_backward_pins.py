"""Pins of the oracle's backward pass (Section 3, Eq. 5 and Eq. 6) to what the mathematics fixes.

The forward oracle is pinned in test_oracle_pins.py.  The layer is linear in its input and linear in
W_F, so its backward pass is the adjoint of two linear maps: <f(x; W), G> = <x, dL/dI> and
<f(x; W), G> = <W, dL/dW_F> for L = <O, G>, which holds to rounding only if every transposition, sign and
index map of Eq. 5/6 is right.  Independently of the forward oracle, with W_F = G w G^T the gradients
must reduce to those of the textbook direct convolution (brute force here), the weight gradient through
dL/dw = G^T dL/dW_F G (chain rule through Eq. 3).  Finite differences on a tiny case close the loop.
"""
import numpy as np
import pytest

import oracle
from paper_1702_08597_amd import synth


def dense_csr(P, K, C):
    rowptr = (np.arange(P * K + 1, dtype=np.int64) * C).astype(np.int32)
    colidx = np.tile(np.arange(C, dtype=np.int32), P * K)
    return rowptr, colidx


def random_case(m, N, C, H, W, K, pad, density, seed):
    rng = np.random.default_rng(seed)
    P = (m + 2) ** 2
    x = rng.standard_normal((N, C, H, W))
    rp, ci, va = synth.bernoulli_weights(P, K, C, density, seed + 1)
    va = rng.standard_normal(va.shape)
    Ho, Wo = H + 2 * pad - 2, W + 2 * pad - 2
    G = rng.standard_normal((N, K, Ho, Wo))
    return x, rp, ci, va, G


@pytest.mark.parametrize("m", [2, 4])
@pytest.mark.parametrize("pad,H,W", [(1, 13, 13), (0, 9, 11), (1, 5, 6), (2, 4, 4)])
def test_backward_is_the_adjoint_of_the_forward_maps(m, pad, H, W):
    N, C, K = 2, 5, 4
    x, rp, ci, va, G = random_case(m, N, C, H, W, K, pad, 0.6, 1000 + 10 * m + pad)
    out, V, M = oracle.forward_f64(x, rp, ci, va, K, m, 3, pad)
    din, dvals, dZ, dV = oracle.backward_f64(x, rp, ci, va, G, K, m, 3, pad)
    L = float((out * G).sum())
    scale = np.abs(out).max() * np.abs(G).max() * out.size
    assert abs(L - float((x * din).sum())) <= 1e-12 * scale       # adjoint w.r.t. the input (Eq. 6)
    assert abs(L - float((va * dvals).sum())) <= 1e-12 * scale    # adjoint w.r.t. the stored W_F entries (Eq. 5)
    assert abs(L - float((M * dZ).sum())) <= 1e-12 * scale        # O~ = A^T Z A  <->  dZ = A dO~ A^T
    assert abs(L - float((V * dV).sum())) <= 1e-12 * scale        # Z = W_F I_F  <->  dI_F = W_F^T dZ


def direct_conv_grads(x, w, G, pad):
    """Brute-force gradients of L = <O, G>, O = cross-correlation of x with w (Eq. 1), zero padding."""
    N, C, H, W = x.shape
    K, _, r, _ = w.shape
    Ho, Wo = G.shape[2:]
    xp = np.zeros((N, C, H + 2 * pad, W + 2 * pad))
    xp[:, :, pad:pad + H, pad:pad + W] = x
    dw = np.zeros_like(w)
    dxp = np.zeros_like(xp)
    for u in range(r):
        for v in range(r):
            win = xp[:, :, u:u + Ho, v:v + Wo]                      # [N][C][Ho][Wo]
            dw[:, :, u, v] = np.einsum("nkyx,ncyx->kc", G, win)
            dxp[:, :, u:u + Ho, v:v + Wo] += np.einsum("nkyx,kc->ncyx", G, w[:, :, u, v])
    return dxp[:, :, pad:pad + H, pad:pad + W], dw


@pytest.mark.parametrize("m", [2, 4])
@pytest.mark.parametrize("pad,H,W", [(1, 13, 13), (0, 7, 10), (1, 6, 5)])
def test_with_GwGT_backward_equals_direct_convolution_gradients(m, pad, H, W):
    rng = np.random.default_rng(2000 + m + pad)
    N, C, K = 2, 3, 4
    t = m + 2
    P = t * t
    x = rng.standard_normal((N, C, H, W))
    w = rng.standard_normal((K, C, 3, 3))
    G = rng.standard_normal((N, K, H + 2 * pad - 2, W + 2 * pad - 2))
    wf = oracle.wf_from_spatial_f64(w, m)                                  # [p][K][C], p = i*t + j
    vals = wf.reshape(-1)
    rp, ci = dense_csr(P, K, C)
    din, dvals, _, _ = oracle.backward_f64(x, rp, ci, vals, G, K, m, 3, pad, want_ZV=False)
    dx_ref, dw_ref = direct_conv_grads(x, w, G, pad)
    np.testing.assert_allclose(din, dx_ref, rtol=0, atol=1e-11 * np.abs(dx_ref).max())
    _, _, Gm = oracle.winograd_matrices(m)                                 # t x r
    dwf = dvals.reshape(t, t, K, C)                                        # [i][j][K][C]
    dw = np.einsum("iu,ijkc,jv->kcuv", Gm, dwf, Gm)                        # G^T dW_F G (chain rule through Eq. 3)
    np.testing.assert_allclose(dw, dw_ref, rtol=0, atol=1e-11 * np.abs(dw_ref).max())


def test_finite_differences_tiny_case():
    m, N, C, H, W, K, pad = 4, 1, 2, 6, 5, 2, 1
    x, rp, ci, va, G = random_case(m, N, C, H, W, K, pad, 0.7, 3000)
    din, dvals, _, _ = oracle.backward_f64(x, rp, ci, va, G, K, m, 3, pad, want_ZV=False)
    loss = lambda xx, vv: float((oracle.forward_f64(xx, rp, ci, vv, K, m, 3, pad, want_VM=False)[0] * G).sum())
    eps = 1e-6
    rng = np.random.default_rng(3001)
    for idx in rng.choice(x.size, size=12, replace=False):
        e = np.zeros(x.size); e[idx] = eps
        fd = (loss(x + e.reshape(x.shape), va) - loss(x - e.reshape(x.shape), va)) / (2 * eps)
        assert abs(fd - din.reshape(-1)[idx]) <= 1e-6 * max(1.0, abs(fd))
    for idx in rng.choice(va.size, size=12, replace=False):
        e = np.zeros(va.size); e[idx] = eps
        fd = (loss(x, va + e) - loss(x, va - e)) / (2 * eps)
        assert abs(fd - dvals[idx]) <= 1e-6 * max(1.0, abs(fd))


def test_gradient_of_dropped_outputs_is_ignored_and_zero_weights_give_zero_input_gradient():
    # 13 with m = 4: the last tile row/column computes outputs that are dropped; they carry no gradient
    m, N, C, H, W, K, pad = 4, 1, 2, 13, 13, 3, 1
    x, rp, ci, va, G = random_case(m, N, C, H, W, K, pad, 0.5, 4000)
    P = 36
    empty = np.zeros(P * K + 1, dtype=np.int32)
    din, dvals, dZ, dV = oracle.backward_f64(x, empty, np.zeros(0, np.int32), np.zeros(0), G, K, m, 3, pad)
    assert np.all(din == 0) and dvals.size == 0 and np.all(dV == 0)
    # dZ of a tile equals A g A^T with g zero outside the 13 x 13 output: corner tile keeps one pixel
    AT, _, _ = oracle.winograd_matrices(m)
    g = np.zeros((4, 4)); g[0, 0] = G[0, 1, 12, 12]
    want = AT.T @ g @ AT
    tau = 3 * 4 + 3
    np.testing.assert_allclose(dZ[:, 1, tau].reshape(6, 6), want, rtol=0, atol=1e-14)


def test_float_instantiation_agrees_with_double():
    m, N, C, H, W, K, pad = 4, 4, 24, 13, 13, 20, 1
    rng = np.random.default_rng(5000)
    x = synth.activations(N, C, H, W, 5001)
    rp, ci, va = synth.bernoulli_weights(36, K, C, 0.3, 5002)
    G = rng.standard_normal((N, K, 13, 13)).astype(np.float32)
    d64 = oracle.backward_f64(x, rp, ci, va, G, K, m, want_ZV=False)
    d32 = oracle.backward_f32(x, rp, ci, va, G, K, m)
    for a, b in zip(d32[:2], d64[:2]):
        assert np.abs(a - b).max() <= 1e-4 * np.abs(b).max()
