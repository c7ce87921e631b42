"""Pins of the oracle's primitives against things other than itself: library routines
(numpy matmul, scipy correlate2d), closed forms, adjoint identities, brute force."""
import numpy as np
import pytest
from scipy.signal import correlate2d

from oracle import lpref

rng = np.random.default_rng(1234)


def _brute_conv(x, w, stride, pad):
    """Pure-Python 7-loop convolution on a zero-padded copy (tiny inputs only)."""
    N, H, W, Cin = x.shape
    Cout, R, S, _ = w.shape
    xp = np.zeros((N, H + 2 * pad, W + 2 * pad, Cin))
    xp[:, pad:pad + H, pad:pad + W, :] = x
    Ho, Wo = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1
    y = np.zeros((N, Ho, Wo, Cout))
    for n in range(N):
        for ho in range(Ho):
            for wo in range(Wo):
                for co in range(Cout):
                    acc = 0.0
                    for r in range(R):
                        for s in range(S):
                            for ci in range(Cin):
                                acc += xp[n, ho * stride + r, wo * stride + s, ci] * w[co, r, s, ci]
                    y[n, ho, wo, co] = acc
    return y


CASES = [(2, 5, 6, 3, 4, 3, 1, 1), (1, 6, 6, 2, 3, 3, 2, 1), (2, 4, 4, 5, 2, 1, 1, 0),
         (1, 6, 4, 3, 2, 1, 2, 0), (1, 9, 9, 2, 2, 7, 2, 3)]


@pytest.mark.parametrize("N,H,W,Cin,Cout,R,stride,pad", CASES)
def test_conv_fwd_brute_force(N, H, W, Cin, Cout, R, stride, pad):
    x = rng.standard_normal((N, H, W, Cin))
    w = rng.standard_normal((Cout, R, R, Cin))
    np.testing.assert_allclose(lpref.conv_fwd(x, w, stride, pad), _brute_conv(x, w, stride, pad), rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("stride,pad,R", [(1, 1, 3), (2, 1, 3), (2, 3, 7), (1, 0, 1)])
def test_conv_fwd_vs_scipy_correlate(stride, pad, R):
    """Cross-correlation per (cout, cin) channel pair with a library routine, then subsample by the stride."""
    N, H, W, Cin, Cout = 2, 10, 8, 3, 2
    x = rng.standard_normal((N, H, W, Cin))
    w = rng.standard_normal((Cout, R, R, Cin))
    y = lpref.conv_fwd(x, w, stride, pad)
    xp = np.pad(x, ((0, 0), (pad, pad), (pad, pad), (0, 0)))
    for n in range(N):
        for co in range(Cout):
            full = sum(correlate2d(xp[n, :, :, ci], w[co, :, :, ci], mode="valid") for ci in range(Cin))
            np.testing.assert_allclose(y[n, :, :, co], full[::stride, ::stride], rtol=1e-11, atol=1e-11)


def test_conv_1x1_is_matmul():
    x = rng.standard_normal((3, 4, 5, 6))
    w = rng.standard_normal((7, 1, 1, 6))
    y = lpref.conv_fwd(x, w, 1, 0)
    np.testing.assert_allclose(y.reshape(-1, 7), x.reshape(-1, 6) @ w.reshape(7, 6).T, rtol=1e-12, atol=1e-12)


def test_conv_unit_impulse_returns_flipped_filter():
    """An impulse at (h0,w0,c0) makes y[h0+p-r, w0+p-s, co] = w[co,r,s,c0]."""
    H = W = 7
    x = np.zeros((1, H, W, 3))
    x[0, 3, 3, 1] = 1.0
    w = rng.standard_normal((2, 3, 3, 3))
    y = lpref.conv_fwd(x, w, 1, 1)
    for r in range(3):
        for s in range(3):
            np.testing.assert_allclose(y[0, 3 + 1 - r, 3 + 1 - s, :], w[:, r, s, 1], rtol=0, atol=0)
    assert np.count_nonzero(y) == 2 * 9


@pytest.mark.parametrize("N,H,W,Cin,Cout,R,stride,pad", CASES)
def test_conv_adjoint_identities(N, H, W, Cin, Cout, R, stride, pad):
    """<conv(x,w), g> = <x, dgrad(g,w)> = <w, wgrad(x,g)> (bilinearity)."""
    x = rng.standard_normal((N, H, W, Cin))
    w = rng.standard_normal((Cout, R, R, Cin))
    y = lpref.conv_fwd(x, w, stride, pad)
    g = rng.standard_normal(y.shape)
    lhs = np.sum(y * g)
    dx = lpref.conv_dgrad(g, w, x.shape, stride, pad)
    dw = lpref.conv_wgrad(x, g, w.shape, stride, pad)
    assert abs(lhs - np.sum(x * dx)) <= 1e-11 * abs(lhs) + 1e-11
    assert abs(lhs - np.sum(w * dw)) <= 1e-11 * abs(lhs) + 1e-11


def test_conv_dgrad_wgrad_elementwise_brute():
    """dgrad / wgrad entries equal derivatives of <conv(x,w), g> computed by perturbing one entry
    (exact, because the map is linear in each argument)."""
    N, H, W, Cin, Cout, R, stride, pad = 1, 5, 5, 2, 3, 3, 2, 1
    x = rng.standard_normal((N, H, W, Cin))
    w = rng.standard_normal((Cout, R, R, Cin))
    g = rng.standard_normal(lpref.conv_fwd(x, w, stride, pad).shape)
    dx = lpref.conv_dgrad(g, w, x.shape, stride, pad)
    dw = lpref.conv_wgrad(x, g, w.shape, stride, pad)
    for idx in np.ndindex(x.shape):
        e = np.zeros_like(x); e[idx] = 1.0
        assert abs(np.sum(_brute_conv(e, w, stride, pad) * g) - dx[idx]) < 1e-12
    for idx in np.ndindex(w.shape):
        e = np.zeros_like(w); e[idx] = 1.0
        assert abs(np.sum(_brute_conv(x, e, stride, pad) * g) - dw[idx]) < 1e-12


@pytest.mark.parametrize("N,H,W,Cin,Cout,R,stride,pad", CASES)
def test_im2col_index_reproduces_conv(N, H, W, Cin, Cout, R, stride, pad):
    """Gathering with the canonical index function and a plain GEMM gives the direct convolution; every
    index is in range or -1; and -1 occurs exactly for taps in the padding."""
    x = rng.standard_normal((N, H, W, Cin))
    w = rng.standard_normal((Cout, R, R, Cin))
    Ho, Wo = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - R) // stride + 1
    M, Kg = N * Ho * Wo, R * R * Cin
    A = np.zeros((M, Kg))
    flat = x.reshape(-1)
    n_pad = 0
    for m in range(M):
        for q in range(Kg):
            o = lpref.im2col_index(m, q, H, W, Cin, R, R, stride, pad)
            assert -1 <= o < flat.size
            if o >= 0:
                A[m, q] = flat[o]
            else:
                n_pad += 1
    y = (A @ w.reshape(Cout, Kg).T).reshape(N, Ho, Wo, Cout)
    np.testing.assert_allclose(y, lpref.conv_fwd(x, w, stride, pad), rtol=1e-12, atol=1e-12)
    # count of padded taps by direct enumeration
    cnt = 0
    for ho in range(Ho):
        for wo in range(Wo):
            for r in range(R):
                for s in range(R):
                    hi, wi = ho * stride - pad + r, wo * stride - pad + s
                    cnt += (hi < 0 or hi >= H or wi < 0 or wi >= W)
    assert n_pad == cnt * N * Cin


def test_im2col_index_hand_values():
    # 1 image 4x4, Cin=2, 3x3 stride 1 pad 1: output pixel (1,2) tap (0,0) ci=1 reads input (0,1,ch1)
    m = 1 * 4 + 2
    assert lpref.im2col_index(m, 1, 4, 4, 2, 3, 3, 1, 1) == (0 * 4 + 1) * 2 + 1
    # corner pixel (0,0) tap (0,0) is padding; tap (1,1) is the pixel itself
    assert lpref.im2col_index(0, 0, 4, 4, 2, 3, 3, 1, 1) == -1
    assert lpref.im2col_index(0, (1 * 3 + 1) * 2, 4, 4, 2, 3, 3, 1, 1) == 0
    # stride 2: output (1,1) tap (2,2) ci 0 -> input (2*1-1+2, 2*1-1+2) = (3,3); second image adds H*W*Cin
    assert lpref.im2col_index(1 * 2 + 1, (2 * 3 + 2) * 2, 4, 4, 2, 3, 3, 2, 1) == (3 * 4 + 3) * 2
    assert lpref.im2col_index(4 + 3, (2 * 3 + 2) * 2, 4, 4, 2, 3, 3, 2, 1) == 32 + (3 * 4 + 3) * 2


def test_conv_fwd_at_matches_full():
    x = rng.standard_normal((2, 6, 6, 3)); w = rng.standard_normal((4, 3, 3, 3))
    y = lpref.conv_fwd(x, w, 2, 1)
    for idx in np.ndindex(y.shape):
        assert lpref.conv_fwd_at(x, w, 2, 1, *idx) == y[idx]


def test_bn_forward_moments_and_backward_orthogonality():
    y = rng.standard_normal((4, 5, 6, 7)) * 3.0 + 2.0
    gamma, beta, eps = rng.standard_normal(7) + 1.5, rng.standard_normal(7), 1e-5
    z, cache = lpref.bn_fwd(y, gamma, beta, eps)
    var = y.var(axis=(0, 1, 2))
    np.testing.assert_allclose(z.mean(axis=(0, 1, 2)), beta, atol=1e-12)
    np.testing.assert_allclose(z.var(axis=(0, 1, 2)), gamma ** 2 * var / (var + eps), rtol=1e-11)
    dz = rng.standard_normal(z.shape)
    dy, dgamma, dbeta = lpref.bn_bwd(dz, cache, gamma)
    np.testing.assert_allclose(dy.sum(axis=(0, 1, 2)), 0.0, atol=1e-11)
    # sum dy*yhat = gamma*invstd*dgamma*eps/(var+eps): zero only in the limit eps -> 0
    np.testing.assert_allclose((dy * cache[0]).sum(axis=(0, 1, 2)),
                               gamma * cache[1] * dgamma * eps / (var + eps), atol=1e-11)
    np.testing.assert_allclose(dgamma, (dz * (y - y.mean(axis=(0, 1, 2))) / np.sqrt(var + eps)).sum(axis=(0, 1, 2)), rtol=1e-11)
    np.testing.assert_allclose(dbeta, dz.sum(axis=(0, 1, 2)), rtol=1e-12)
    # statistics are over N*H*W only: channels do not mix
    y2 = y.copy(); y2[..., 0] *= 10.0
    z2, _ = lpref.bn_fwd(y2, gamma, beta, eps)
    np.testing.assert_allclose(z2[..., 1:], z[..., 1:], rtol=0, atol=0)


def test_bn_backward_finite_difference():
    y = rng.standard_normal((2, 3, 3, 4))
    gamma, beta, eps = rng.standard_normal(4) + 1.0, rng.standard_normal(4), 1e-3
    g = rng.standard_normal(y.shape)
    f = lambda yy, ga, be: np.sum(lpref.bn_fwd(yy, ga, be, eps)[0] * g)
    _, cache = lpref.bn_fwd(y, gamma, beta, eps)
    dy, dgamma, dbeta = lpref.bn_bwd(g, cache, gamma)
    h = 1e-6
    for idx in np.ndindex(y.shape):
        e = np.zeros_like(y); e[idx] = h
        assert abs((f(y + e, gamma, beta) - f(y - e, gamma, beta)) / (2 * h) - dy[idx]) < 1e-7
    for c in range(4):
        e = np.zeros(4); e[c] = h
        assert abs((f(y, gamma + e, beta) - f(y, gamma - e, beta)) / (2 * h) - dgamma[c]) < 1e-7
        assert abs((f(y, gamma, beta + e) - f(y, gamma, beta - e)) / (2 * h) - dbeta[c]) < 1e-7


def test_ce_closed_forms():
    N, C = 5, 7
    labels = np.array([0, 3, 6, 2, 2])
    loss, dz = lpref.ce_loss_grad(np.full((N, C), 0.37), labels)
    assert abs(loss - np.log(C)) < 1e-14
    z = rng.standard_normal((N, C)) * 4
    loss, dz = lpref.ce_loss_grad(z, labels)
    np.testing.assert_allclose(dz.sum(axis=1), 0.0, atol=1e-15)
    loss2, dz2 = lpref.ce_loss_grad(z + rng.standard_normal((N, 1)) * 50, labels)
    assert abs(loss - loss2) < 1e-12
    np.testing.assert_allclose(dz, dz2, atol=1e-13)
    # two-class case is the logistic loss: log(1+exp(-(z_y - z_other)))
    z2 = rng.standard_normal((4, 2)); l2 = np.array([0, 1, 1, 0])
    d = z2[np.arange(4), l2] - z2[np.arange(4), 1 - l2]
    assert abs(lpref.ce_loss_grad(z2, l2)[0] - np.mean(np.log1p(np.exp(-d)))) < 1e-14
    # finite differences
    h = 1e-6
    for idx in np.ndindex(z.shape):
        e = np.zeros_like(z); e[idx] = h
        fd = (lpref.ce_loss_grad(z + e, labels)[0] - lpref.ce_loss_grad(z - e, labels)[0]) / (2 * h)
        assert abs(fd - dz[idx]) < 1e-8
    # huge logits stay finite
    assert np.isfinite(lpref.ce_loss_grad(z * 1e4, labels)[0])


def test_local_loss_hand_example_and_limits():
    """rho=2, r=(1,2), lam=(0.5,-1): loss = 1*(1+4) + (0.5-2) = 3.5, dy = 2r+lam = (2.5,3)."""
    y = np.array([1.0, 2.0]).reshape(1, 1, 1, 2); x = np.zeros_like(y)
    lam = np.array([0.5, -1.0]).reshape(1, 1, 1, 2)
    loss, dy = lpref.local_loss_grad(y, x, lam, 2.0)
    assert loss == 3.5
    np.testing.assert_array_equal(dy.reshape(-1), [2.5, 3.0])
    loss, dy = lpref.local_loss_grad(y, x, lam, 2.0, scale=0.5)
    assert loss == 1.75
    np.testing.assert_array_equal(dy.reshape(-1), [1.25, 1.5])
    # zero multiplier is the penalty method
    lp, dp = lpref.local_loss_grad(y, x, None, 2.0)
    l0, d0 = lpref.local_loss_grad(y, x, np.zeros_like(y), 2.0)
    assert lp == l0 == 5.0 and np.array_equal(dp, d0)
    # consistent auxiliary variable and zero multiplier: everything vanishes
    lv, dv = lpref.local_loss_grad(y, y.copy(), None, 7.0)
    assert lv == 0.0 and not dv.any()
    # sign convention: r = F_k(x_k) - x_{k+1}
    l1, d1 = lpref.local_loss_grad(x, y, lam, 2.0)
    assert l1 == 5.0 - (0.5 - 2.0)
    np.testing.assert_array_equal(d1.reshape(-1), [-2.0 + 0.5, -4.0 - 1.0])


def test_local_loss_finite_difference():
    y = rng.standard_normal((2, 3, 3, 4)); x = rng.standard_normal(y.shape); lam = rng.standard_normal(y.shape)
    _, dy = lpref.local_loss_grad(y, x, lam, 1.7, 0.3)
    h = 1e-6
    for idx in list(np.ndindex(y.shape))[::5]:
        e = np.zeros_like(y); e[idx] = h
        fd = (lpref.local_loss_grad(y + e, x, lam, 1.7, 0.3)[0] - lpref.local_loss_grad(y - e, x, lam, 1.7, 0.3)[0]) / (2 * h)
        assert abs(fd - dy[idx]) < 1e-8


def test_multiplier_update_closed_form():
    lam = rng.standard_normal((2, 2, 2, 3)); y = rng.standard_normal(lam.shape); x = rng.standard_normal(lam.shape)
    np.testing.assert_array_equal(lpref.multiplier_update(lam, y, x, 0.0), lam)
    np.testing.assert_array_equal(lpref.multiplier_update(lam, y, y, 0.9), lam)
    out = lpref.multiplier_update(lam, y, x, 0.25)
    for idx in np.ndindex(lam.shape):
        assert out[idx] == lam[idx] + 0.25 * (y[idx] - x[idx])
    # ascent direction of the multiplier term <lam, r>: d/dlam = r
    assert np.sum((out - lam) * (y - x)) > 0


def test_maxpool_first_max_and_adjoint():
    x = np.zeros((1, 4, 4, 1)); x[0, 0, 0, 0] = 5.0; x[0, 0, 1, 0] = 5.0; x[0, 1, 0, 0] = 5.0
    y, idx = lpref.maxpool_fwd(x, 3, 2, 1)
    assert y.shape == (1, 2, 2, 1) and y[0, 0, 0, 0] == 5.0 and idx[0, 0, 0, 0] == 0   # first in row-major window order
    x = rng.standard_normal((2, 7, 6, 3))
    y, idx = lpref.maxpool_fwd(x, 3, 2, 1)
    xp = np.pad(x, ((0, 0), (1, 1), (1, 1), (0, 0)), constant_values=-np.inf)
    for n, ho, wo, c in np.ndindex(y.shape):
        assert y[n, ho, wo, c] == xp[n, 2 * ho:2 * ho + 3, 2 * wo:2 * wo + 3, c].max()
        assert x.reshape(-1)[idx[n, ho, wo, c]] == y[n, ho, wo, c]
    g = rng.standard_normal(y.shape)
    dx = lpref.maxpool_bwd(g, idx, x.shape)
    assert abs(dx.sum() - g.sum()) < 1e-12
    h = 1e-7
    e = rng.standard_normal(x.shape)
    fd = (np.sum(lpref.maxpool_fwd(x + h * e)[0] * g) - np.sum(lpref.maxpool_fwd(x - h * e)[0] * g)) / (2 * h)
    assert abs(fd - np.sum(dx * e)) < 1e-6


def test_residual_norm_hand_example_and_penalty_relation():
    """|r|^2 by hand (3-4-12 -> 169), and its relation to the penalty term: with no multiplier loss = rho/2 * |r|^2."""
    y = np.array([[[[3.0, 1.0]], [[5.0, -2.0]]]])
    x = np.array([[[[0.0, 1.0]], [[1.0, 10.0]]]])
    assert lpref.residual_norm2(y, x) == 169.0
    loss, _ = lpref.local_loss_grad(y, x, None, rho=0.5, scale=2.0)
    assert abs(loss - 2.0 * 0.25 * 169.0) < 1e-12
    assert lpref.residual_norm2(x, x) == 0.0


def test_c_routines_under_address_and_undefined_behaviour_sanitizers():
    """The C part of the oracle, compiled with -fsanitize=address,undefined into a self-check executable that runs
    every routine over small ragged shapes (see oracle/lpref_selfcheck.c): no out-of-bounds access, no undefined
    behaviour, and the self-check's own comparisons hold."""
    import os
    import subprocess
    from oracle.build import build_selfcheck
    exe = build_selfcheck()
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="halt_on_error=1", OMP_NUM_THREADS="4")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "0 failure(s)" in r.stdout
    assert "ERROR" not in r.stderr and "runtime error" not in r.stderr, r.stderr
