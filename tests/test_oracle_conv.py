"""Pins for the oracle's convolution trio (no GPU).

Each pin fixes the oracle to something other than itself: hand-worked values, closed
forms, library routines, scatter-form brute force written independently here, the
paper's padding and FFT identities (Section II-A), adjointness and finite differences.
"""
import os

import numpy as np
import pytest
import scipy.signal

from oracle import oracle as orc

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def load_golden(path):
    out, cur, rows = {}, None, 0
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        tok = line.split()
        if tok[0][0].isalpha():
            cur, rows = tok[0], int(tok[1])
            out[cur] = []
        else:
            out[cur].append([float(t) for t in tok])
    return {k: np.array(v) for k, v in out.items()}


def scatter_xcorr(x, w, pad):
    """Forward layer written the other way round (scatter form): every input pixel adds its
    contribution to every output it touches."""
    N, C, H, W = x.shape
    K, _, R, S = w.shape
    Ho, Wo = H + 2 * pad - R + 1, W + 2 * pad - S + 1
    z = np.zeros((N, K, Ho, Wo))
    for n in range(N):
        for c in range(C):
            for ii in range(H):
                for jj in range(W):
                    for k in range(K):
                        for r in range(R):
                            for s in range(S):
                                i, j = ii + pad - r, jj + pad - s
                                if 0 <= i < Ho and 0 <= j < Wo:
                                    z[n, k, i, j] += x[n, c, ii, jj] * w[k, c, r, s]
    return z


def stamp_full(dz, w, pad):
    """Full convolution as 'each dz element stamps the kernel', then cropped by pad."""
    N, K, Ho, Wo = dz.shape
    _, C, R, S = w.shape
    big = np.zeros((N, C, Ho + R - 1, Wo + S - 1))
    for n in range(N):
        for k in range(K):
            for i in range(Ho):
                for j in range(Wo):
                    big[n, :, i:i + R, j:j + S] += dz[n, k, i, j] * w[k]
    H, W = Ho + R - 1 - 2 * pad, Wo + S - 1 - 2 * pad
    return big[:, :, pad:pad + H, pad:pad + W]


def ident(N, C, H, W, K, R, S, pad=0):
    return orc.conv_desc(N, C, H, W, K, R, S, pad, orc.ACT_IDENTITY, 1)


# ---------------------------------------------------------------- forward (valid)

def test_handworked_valid():
    g = load_golden(os.path.join(GOLD, "handworked_3x3_2x2.txt"))
    x, w = g["x"][None, None], g["w"][None, None]
    d = ident(1, 1, 3, 3, 1, 2, 2)
    y, _ = orc.conv_valid_fwd(d, x, w)
    np.testing.assert_array_equal(y[0, 0], g["xcorr_valid"])
    yf, _ = orc.conv_valid_fwd(d, x, w[:, :, ::-1, ::-1])
    np.testing.assert_array_equal(yf[0, 0], g["conv_valid_flipped"])


@pytest.mark.parametrize("pad", [0, 1, 2])
def test_valid_vs_scatter_bruteforce(pad):
    r = np.random.default_rng(7 + pad)
    N, C, H, W, K, R, S = 2, 2, 6, 5, 3, 3, 3
    x, w, b = r.normal(size=(N, C, H, W)), r.normal(size=(K, C, R, S)), r.normal(size=(K,))
    d = ident(N, C, H, W, K, R, S, pad)
    y, _ = orc.conv_valid_fwd(d, x, w, b, f64=True)
    ref = scatter_xcorr(x, w, pad) + b[None, :, None, None]
    np.testing.assert_allclose(y, ref, rtol=0, atol=1e-12)


def test_valid_nonsquare_filter_vs_scipy():
    r = np.random.default_rng(11)
    N, C, H, W, K, R, S = 2, 3, 9, 7, 2, 4, 2
    x, w = r.normal(size=(N, C, H, W)), r.normal(size=(K, C, R, S))
    y, _ = orc.conv_valid_fwd(ident(N, C, H, W, K, R, S), x, w, f64=True)
    for n in range(N):
        for k in range(K):
            ref = sum(scipy.signal.correlate2d(x[n, c], w[k, c], mode="valid") for c in range(C))
            np.testing.assert_allclose(y[n, k], ref, atol=1e-12)


def test_delta_filter_is_crop_shift():
    r = np.random.default_rng(3)
    x = r.normal(size=(1, 1, 8, 9))
    for (a, b) in [(0, 0), (1, 2), (2, 0), (2, 2)]:
        w = np.zeros((1, 1, 3, 3))
        w[0, 0, a, b] = 1.0
        y, _ = orc.conv_valid_fwd(ident(1, 1, 8, 9, 1, 3, 3), x, w, f64=True)
        np.testing.assert_array_equal(y[0, 0], x[0, 0, a:a + 6, b:b + 7])


def test_box_filter_vs_summed_area_table():
    r = np.random.default_rng(5)
    H, W, R, S = 10, 11, 5, 3
    x = r.integers(-4, 5, size=(1, 1, H, W)).astype(np.float64)
    y, _ = orc.conv_valid_fwd(ident(1, 1, H, W, 1, R, S), x, np.ones((1, 1, R, S)), f64=True)
    sat = np.zeros((H + 1, W + 1))
    sat[1:, 1:] = x[0, 0].cumsum(0).cumsum(1)
    ref = sat[R:, S:] - sat[:-R, S:] - sat[R:, :-S] + sat[:-R, :-S]
    np.testing.assert_array_equal(y[0, 0], ref)


def test_valid_linearity():
    r = np.random.default_rng(9)
    d = ident(2, 2, 7, 7, 3, 3, 3, 1)
    x1, x2 = r.normal(size=(2, 2, 2, 7, 7))
    w1, w2 = r.normal(size=(2, 3, 2, 3, 3))
    f = lambda x, w: orc.conv_valid_fwd(d, x, w, f64=True)[0]
    np.testing.assert_allclose(f(2 * x1 - 3 * x2, w1), 2 * f(x1, w1) - 3 * f(x2, w1), atol=1e-12)
    np.testing.assert_allclose(f(x1, w1 + 0.5 * w2), f(x1, w1) + 0.5 * f(x1, w2), atol=1e-12)


def test_padding_equals_explicit_zero_border():
    r = np.random.default_rng(13)
    x, w = r.normal(size=(2, 3, 6, 8)), r.normal(size=(4, 3, 5, 5))
    y, _ = orc.conv_valid_fwd(ident(2, 3, 6, 8, 4, 5, 5, 2), x, w, f64=True)
    xp = np.pad(x, ((0, 0), (0, 0), (2, 2), (2, 2)))
    y0, _ = orc.conv_valid_fwd(ident(2, 3, 10, 12, 4, 5, 5, 0), xp, w, f64=True)
    np.testing.assert_array_equal(y, y0)


def test_fp32_storage_rounds_once():
    """fp32 instantiation == the fp64 instantiation on the same fp32 inputs, rounded once."""
    r = np.random.default_rng(17)
    x = r.normal(size=(2, 3, 9, 9)).astype(np.float32)
    w = r.normal(size=(5, 3, 3, 3)).astype(np.float32)
    b = r.normal(size=(5,)).astype(np.float32)
    d = orc.conv_desc(2, 3, 9, 9, 5, 3, 3, 1, orc.ACT_SIGMOID, 1)
    y32, _ = orc.conv_valid_fwd(d, x, w, b)
    y64, _ = orc.conv_valid_fwd(d, x, w, b, f64=True)
    assert y32.dtype == np.float32
    np.testing.assert_array_equal(y32, y64.astype(np.float32))


# ---------------------------------------------------------------- backward (full)

def test_handworked_full():
    g = load_golden(os.path.join(GOLD, "handworked_3x3_2x2.txt"))
    # the 3x3 array plays the role of dz; the layer input is then 4x4
    d = ident(1, 1, 4, 4, 1, 2, 2)
    dx = orc.conv_full_bwd(d, g["x"][None, None], None, None, g["w"][None, None])
    np.testing.assert_array_equal(dx[0, 0], g["full"])
    assert dx.sum() == g["x"].sum() * g["w"].sum()


@pytest.mark.parametrize("pad", [0, 1, 2])
def test_full_vs_stamp_bruteforce(pad):
    r = np.random.default_rng(21 + pad)
    N, C, H, W, K, R, S = 2, 3, 7, 6, 2, 3, 3
    d = ident(N, C, H, W, K, R, S, pad)
    dz, w = r.normal(size=d.out_shape), r.normal(size=(K, C, R, S))
    dx = orc.conv_full_bwd(d, dz, None, None, w, f64=True)
    np.testing.assert_allclose(dx, stamp_full(dz, w, pad), atol=1e-12)


def test_full_delta_filter_is_zero_filled_shift():
    r = np.random.default_rng(23)
    dz = r.normal(size=(1, 1, 5, 6))
    for (a, b) in [(0, 0), (1, 2), (2, 1)]:
        w = np.zeros((1, 1, 3, 3))
        w[0, 0, a, b] = 1.0
        dx = orc.conv_full_bwd(ident(1, 1, 7, 8, 1, 3, 3), dz, None, None, w, f64=True)
        ref = np.zeros((7, 8))
        ref[a:a + 5, b:b + 6] = dz[0, 0]
        np.testing.assert_array_equal(dx[0, 0], ref)


def test_full_sum_identity_and_scipy():
    r = np.random.default_rng(25)
    dz, w = r.normal(size=(1, 1, 6, 5)), r.normal(size=(1, 1, 4, 3))
    dx = orc.conv_full_bwd(ident(1, 1, 9, 7, 1, 4, 3), dz, None, None, w, f64=True)
    np.testing.assert_allclose(dx.sum(), dz.sum() * w.sum(), rtol=1e-12)
    np.testing.assert_allclose(dx[0, 0], scipy.signal.convolve2d(dz[0, 0], w[0, 0], mode="full"), atol=1e-12)


def test_full_equals_valid_on_padded_input_with_rotated_kernel():
    """Section II-A: a full convolution is a valid convolution with some amount of padding."""
    r = np.random.default_rng(27)
    N, C, K, R, S, Ho, Wo = 2, 3, 4, 3, 5, 6, 7
    dz, w = r.normal(size=(N, K, Ho, Wo)), r.normal(size=(K, C, R, S))
    dx = orc.conv_full_bwd(ident(N, C, Ho + R - 1, Wo + S - 1, K, R, S), dz, None, None, w, f64=True)
    dzp = np.pad(dz, ((0, 0), (0, 0), (R - 1, R - 1), (S - 1, S - 1)))
    wt = np.ascontiguousarray(w[:, :, ::-1, ::-1].transpose(1, 0, 2, 3))  # [C][K][R][S], rot180
    v, _ = orc.conv_valid_fwd(ident(N, K, Ho + 2 * R - 2, Wo + 2 * S - 2, C, R, S), dzp, wt, f64=True)
    np.testing.assert_allclose(dx, v, atol=1e-12)


def test_full_equals_fft_product():
    """Section II-A: pad image and kernel to the output size, multiply the transforms, invert."""
    r = np.random.default_rng(29)
    Ho, Wo, R, S = 12, 9, 5, 5
    dz, w = r.normal(size=(1, 1, Ho, Wo)), r.normal(size=(1, 1, R, S))
    dx = orc.conv_full_bwd(ident(1, 1, Ho + R - 1, Wo + S - 1, 1, R, S), dz, None, None, w, f64=True)
    shape = (Ho + R - 1, Wo + S - 1)
    ref = np.fft.irfft2(np.fft.rfft2(dz[0, 0], shape) * np.fft.rfft2(w[0, 0], shape), shape)
    np.testing.assert_allclose(dx[0, 0], ref, atol=1e-10)


@pytest.mark.parametrize("pad", [0, 1, 2])
def test_adjoint_fwd_full_wgrad(pad):
    """<valid(x;w), g> == <x, full(g;w)> == <w, wgrad(x,g)> (the forward map is bilinear)."""
    r = np.random.default_rng(31 + pad)
    N, C, H, W, K, R, S = 3, 2, 8, 7, 4, 3, 3
    d = ident(N, C, H, W, K, R, S, pad)
    x, w, g = r.normal(size=(N, C, H, W)), r.normal(size=(K, C, R, S)), r.normal(size=d.out_shape)
    z, _ = orc.conv_valid_fwd(d, x, w, f64=True)
    dx = orc.conv_full_bwd(d, g, None, None, w, f64=True)
    dw, db = orc.conv_valid_wgrad(d, x, g, None, None, f64=True)
    lhs = (z * g).sum()
    np.testing.assert_allclose((x * dx).sum(), lhs, rtol=1e-12)
    np.testing.assert_allclose((w * dw).sum(), lhs, rtol=1e-12)
    np.testing.assert_allclose(db, g.sum(axis=(0, 2, 3)), rtol=1e-12)


def test_wgrad_vs_scipy():
    r = np.random.default_rng(37)
    N, C, H, W, K, R, S = 2, 2, 8, 8, 3, 3, 3
    d = ident(N, C, H, W, K, R, S)
    x, g = r.normal(size=(N, C, H, W)), r.normal(size=d.out_shape)
    dw, _ = orc.conv_valid_wgrad(d, x, g, None, None, f64=True)
    for k in range(K):
        for c in range(C):
            ref = sum(scipy.signal.correlate2d(x[n, c], g[n, k], mode="valid") for n in range(N))
            np.testing.assert_allclose(dw[k, c], ref, atol=1e-12)


# ---------------------------------------------------------------- activation, pooling, prologue

@pytest.mark.parametrize("act", [orc.ACT_SIGMOID, orc.ACT_RELU])
def test_act_and_pool_bruteforce(act):
    r = np.random.default_rng(41 + act)
    N, C, H, W, K, R, S = 2, 2, 8, 10, 3, 3, 3
    x, w, b = r.normal(size=(N, C, H, W)), r.normal(size=(K, C, R, S)), r.normal(size=(K,))
    z, _ = orc.conv_valid_fwd(ident(N, C, H, W, K, R, S), x, w, b, f64=True)
    a = 1 / (1 + np.exp(-z)) if act == orc.ACT_SIGMOID else np.maximum(z, 0)
    ya, _ = orc.conv_valid_fwd(orc.conv_desc(N, C, H, W, K, R, S, 0, act, 1), x, w, b, f64=True)
    np.testing.assert_allclose(ya, a, atol=1e-15)
    yp, idx = orc.conv_valid_fwd(orc.conv_desc(N, C, H, W, K, R, S, 0, act, 2), x, w, b, f64=True)
    win = a.reshape(N, K, 3, 2, 4, 2).transpose(0, 1, 2, 4, 3, 5).reshape(N, K, 3, 4, 4)
    np.testing.assert_allclose(yp, win.max(-1), atol=1e-15)
    np.testing.assert_array_equal(idx, win.argmax(-1))  # numpy argmax = first maximum
    # bias and a monotone activation commute with max: pool(act(z+b)) == act(pool(z)+b)
    z0, _ = orc.conv_valid_fwd(orc.conv_desc(N, C, H, W, K, R, S, 0, orc.ACT_IDENTITY, 2), x, w, None, f64=True)
    zb = z0 + b[None, :, None, None]
    np.testing.assert_allclose(yp, 1 / (1 + np.exp(-zb)) if act == orc.ACT_SIGMOID else np.maximum(zb, 0), atol=1e-12)


def test_pool_tie_takes_first_and_relu_zero_has_no_gradient():
    x = np.zeros((1, 1, 4, 4))
    x[0, 0, 0:2, 0:2] = [[1, 5], [5, 2]]      # tie between (0,1) and (1,0) -> first = (0,1)
    x[0, 0, 2:4, 2:4] = -1.0                  # all clamp to 0 under ReLU -> idx 0, gradient 0
    w = np.ones((1, 1, 1, 1))
    d = orc.conv_desc(1, 1, 4, 4, 1, 1, 1, 0, orc.ACT_RELU, 2)
    y, idx = orc.conv_valid_fwd(d, x, w, f64=True)
    assert idx[0, 0, 0, 0] == 1 and y[0, 0, 0, 0] == 5
    assert idx[0, 0, 1, 1] == 0 and y[0, 0, 1, 1] == 0
    dx = orc.conv_full_bwd(d, np.ones_like(y), y, idx, w, f64=True)
    assert dx[0, 0, 0, 1] == 1 and dx[0, 0, 1, 0] == 0
    assert np.all(dx[0, 0, 2:4, 2:4] == 0)


def test_unpooled_gradient_sums_to_dy():
    r = np.random.default_rng(43)
    N, C, H, W, K = 2, 1, 6, 6, 2
    d = orc.conv_desc(N, C, H, W, K, 1, 1, 0, orc.ACT_IDENTITY, 2)
    x, w = r.normal(size=(N, C, H, W)), np.ones((K, C, 1, 1))
    y, idx = orc.conv_valid_fwd(d, x, w, f64=True)
    dy = r.normal(size=y.shape)
    # with 1x1 unit filters and C = 1 the full conv returns sum_k dz[n,k,i,j]
    dx = orc.conv_full_bwd(d, dy, y, idx, w, f64=True)
    win = dx.reshape(N, 1, 3, 2, 3, 2).sum(axis=(3, 5))
    np.testing.assert_allclose(win[:, 0], dy.sum(axis=1), atol=1e-12)


@pytest.mark.parametrize("act,pool", [(orc.ACT_SIGMOID, 1), (orc.ACT_SIGMOID, 2), (orc.ACT_RELU, 2),
                                      (orc.ACT_IDENTITY, 2)])
def test_finite_differences_through_layer(act, pool):
    """Central differences in double of L = <y(x,w,b), g> against dx, dw, db."""
    r = np.random.default_rng(47 + act + 10 * pool)
    N, C, H, W, K, R, S, pad = 2, 2, 6, 6, 3, 3, 3, 1
    d = orc.conv_desc(N, C, H, W, K, R, S, pad, act, pool)
    x, w, b = r.normal(size=(N, C, H, W)), r.normal(size=(K, C, R, S)), r.normal(size=(K,))
    g = r.normal(size=d.out_shape)
    y, idx = orc.conv_valid_fwd(d, x, w, b, f64=True)
    dx = orc.conv_full_bwd(d, g, y, idx, w, f64=True)
    dw, db = orc.conv_valid_wgrad(d, x, g, y, idx, f64=True)
    L = lambda xx, ww, bb: (orc.conv_valid_fwd(d, xx, ww, bb, f64=True)[0] * g).sum()
    h = 1e-5
    for arr, grad, which in ((x, dx, 0), (w, dw, 1), (b, db, 2)):
        flat = arr.reshape(-1)
        for t in r.choice(flat.size, size=min(12, flat.size), replace=False):
            args = [x.copy(), w.copy(), b.copy()]
            args[which].reshape(-1)[t] += h
            up = L(*args)
            args[which].reshape(-1)[t] -= 2 * h
            fd = (up - L(*args)) / (2 * h)
            np.testing.assert_allclose(grad.reshape(-1)[t], fd, rtol=2e-6, atol=1e-8)


def test_rejects_bad_shapes():
    x, w = np.zeros((1, 1, 5, 5)), np.zeros((1, 1, 3, 3))
    with pytest.raises(ValueError):
        orc.conv_valid_fwd(orc.conv_desc(1, 1, 5, 5, 1, 3, 3, 0, 0, 2), x, w)   # odd map + pool
    with pytest.raises(ValueError):
        orc.conv_valid_fwd(orc.conv_desc(1, 1, 5, 5, 1, 3, 3, 3, 0, 1), x, w)   # pad > R-1
    with pytest.raises(ValueError):
        orc.conv_valid_fwd(orc.conv_desc(1, 1, 5, 5, 1, 3, 3, 0, 7, 1), x, w)   # unknown act
