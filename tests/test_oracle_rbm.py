"""Pins for the oracle's CRBM variants (probabilistic max pooling, Gaussian visible units), its
fully-connected RBM CD-1 step and its fully-connected network step (no GPU): brute-force
Boltzmann enumeration from the energy function, closed forms, limits that reduce to the sigmoid
unit, exact sampling intervals, degenerate shapes in which the convolutional and the
fully-connected models coincide, composition from the separately pinned conv trio and finite
differences in double."""
import itertools

import numpy as np
import pytest

from oracle import oracle as orc


def sigmoid(z):
    return 1 / (1 + np.exp(-z))


def unit_filter_crbm(I):
    """A CRBM whose hidden inputs are the visible values themselves: one channel, one 1x1 filter
    of weight 1, zero bias.  I: [N, Ho, Wo] -> (desc, v0, W, b, c)."""
    N, H, W = I.shape
    d = orc.conv_desc(N, 1, H, W, 1, 1, 1)
    return d, I[:, None].astype(np.float64), np.ones((1, 1, 1, 1)), np.zeros(1), np.zeros(1)


# ---------------------------------------------------------------- probabilistic max pooling

def test_pmp_matches_boltzmann_enumeration_of_the_energy():
    """P(h | v) of a block from the model's energy E(v,h) = -sum_k sum_ij h_ij (b_k + (W_k * v)_ij):
    enumerate all 16 on/off patterns of a 2x2 block, keep the 5 with at most one unit on, weight
    each by exp(-E) and read the marginals off."""
    r = np.random.default_rng(11)
    N, C, K, R, S = 2, 2, 3, 3, 2
    H, W = R + 3, S + 3                       # 4x4 hidden map = four blocks per filter
    d = orc.conv_desc(N, C, H, W, K, R, S)
    v0 = r.normal(size=(N, C, H, W))
    Wt, b, c = r.normal(size=(K, C, R, S)) * 0.7, r.normal(size=K), r.normal(size=C) * 0.1
    u = r.random((N, K, 2, 2))
    res = orc.crbm_cd1_step_units(d, orc.VIS_GAUSSIAN, 2, v0, Wt.copy(), b.copy(), c.copy(), u, f64=True)
    for n, k, pi, pj in itertools.product(range(N), range(K), range(2), range(2)):
        I = np.empty(4)
        for a, bb in itertools.product(range(2), range(2)):
            i, j = 2 * pi + a, 2 * pj + bb
            I[2 * a + bb] = b[k] + (v0[n, :, i:i + R, j:j + S] * Wt[k]).sum()
        marg, off, Z = np.zeros(4), 0.0, 0.0
        for pattern in itertools.product((0, 1), repeat=4):
            if sum(pattern) > 1:
                continue                      # excluded by the pooling constraint
            wgt = np.exp(np.dot(pattern, I))
            Z += wgt
            marg += wgt * np.array(pattern)
            off += wgt * (sum(pattern) == 0)
        got = res.h0_prob[n, k, 2 * pi:2 * pi + 2, 2 * pj:2 * pj + 2].reshape(4)
        np.testing.assert_allclose(got, marg / Z, rtol=1e-12)
        np.testing.assert_allclose(res.pool_prob[n, k, pi, pj], 1 - off / Z, rtol=1e-12)


def test_pmp_closed_forms_and_limits():
    # all inputs zero: five equally likely states
    d, v0, W, b, c = unit_filter_crbm(np.zeros((1, 4, 6)))
    u = np.full((1, 1, 2, 3), 0.5)
    res = orc.crbm_cd1_step_units(d, orc.VIS_GAUSSIAN, 2, v0, W, b, c, u, f64=True)
    np.testing.assert_allclose(res.h0_prob, 0.2, rtol=1e-15)
    np.testing.assert_allclose(res.pool_prob, 0.8, rtol=1e-15)
    # three units of a block silenced: the fourth is an ordinary sigmoid unit, wherever it sits
    for pos in range(4):
        for z in (-3.0, 0.25, 7.0):
            I = np.full((1, 2, 2), -800.0)
            I[0, pos // 2, pos % 2] = z
            d, v0, W, b, c = unit_filter_crbm(I)
            res = orc.crbm_cd1_step_units(d, orc.VIS_GAUSSIAN, 2, v0, W, b, c, np.full((1, 1, 1, 1), 0.5), f64=True)
            want = np.zeros(4)
            want[pos] = sigmoid(z)
            np.testing.assert_allclose(res.h0_prob.reshape(4), want, rtol=1e-14, atol=1e-300)
            np.testing.assert_allclose(res.pool_prob.reshape(()), sigmoid(z), rtol=1e-14)
    # huge inputs neither overflow nor lose the ratio: exp(1000)/(exp(1000)+exp(999)+...) = softmax
    I = np.array([[[1000.0, 999.0], [998.0, -5.0]]])
    d, v0, W, b, c = unit_filter_crbm(I)
    res = orc.crbm_cd1_step_units(d, orc.VIS_GAUSSIAN, 2, v0, W, b, c, np.full((1, 1, 1, 1), 0.5), f64=True)
    e = np.exp(np.array([0.0, -1.0, -2.0, -1005.0]))
    np.testing.assert_allclose(res.h0_prob.reshape(4), e / e.sum(), rtol=1e-14)
    # odd hidden maps cannot be pooled
    d = orc.conv_desc(1, 1, 5, 4, 1, 1, 1)
    with pytest.raises(ValueError):
        orc.crbm_cd1_step_units(d, 0, 2, np.zeros((1, 1, 5, 4)), np.ones((1, 1, 1, 1)), np.zeros(1), np.zeros(1),
                                np.zeros((1, 1, 2, 2)), f64=True)


def test_pmp_sampling_intervals():
    """One uniform number per block picks the state: unit i (order 2a+b) is on for u in
    [q0+..+q_{i-1}, q0+..+q_i), nothing is on above q0+..+q3.  A fine grid of u over identical
    images must hit every state with its probability (to 1/n) and never two units at once."""
    n = 2000
    block = np.array([[0.3, -1.2], [1.1, 0.0]])
    I = np.broadcast_to(block, (n, 2, 2)).copy()
    d, v0, W, b, c = unit_filter_crbm(I)
    u = ((np.arange(n) + 0.5) / n).reshape(n, 1, 1, 1)
    res = orc.crbm_cd1_step_units(d, orc.VIS_GAUSSIAN, 2, v0, W, b, c, u, f64=True)
    q = res.h0_prob[0, 0].reshape(4)
    hs = res.h0_sample.reshape(n, 4)
    assert set(np.unique(hs)) <= {0.0, 1.0}
    assert hs.sum(axis=1).max() == 1.0
    np.testing.assert_allclose(hs.mean(axis=0), q, atol=1.0 / n)
    np.testing.assert_allclose((hs.sum(axis=1) == 0).mean(), 1 - q.sum(), atol=1.0 / n)
    edges = np.concatenate([[0.0], np.cumsum(q)])
    uu = u.reshape(n)
    for i in range(4):
        np.testing.assert_array_equal(hs[:, i] == 1.0, (edges[i] <= uu) & (uu < edges[i + 1]))


def crbm_inputs(seed, N=3, C=2, H=10, W=8, K=4, R=3, S=3, binary=True):
    r = np.random.default_rng(seed)
    d = orc.conv_desc(N, C, H, W, K, R, S)
    v0 = (r.random((N, C, H, W)) < 0.3).astype(np.float64) if binary else r.normal(size=(N, C, H, W))
    Wt = r.normal(size=(K, C, R, S)) * 0.3
    b, c = r.normal(size=(K,)) * 0.2, r.normal(size=(C,)) * 0.2
    return d, v0, Wt, b, c, r


@pytest.mark.parametrize("visible", [orc.VIS_BINARY, orc.VIS_GAUSSIAN])
@pytest.mark.parametrize("hidden_pool", [1, 2])
def test_crbm_variants_are_compositions_of_the_trio(visible, hidden_pool):
    """Reconstruction = full convolution of the sampled states (+ c, then the visible unit's mean),
    statistics = filter gradients with the hidden probabilities in place of dz, negative phase =
    the positive phase's hidden rule applied to the reconstruction."""
    d, v0, W, b, c, r = crbm_inputs(410 + 2 * visible + hidden_pool, binary=(visible == 0))
    u = r.random((d.N, d.K, d.Ho // hidden_pool, d.Wo // hidden_pool))
    res = orc.crbm_cd1_step_units(d, visible, hidden_pool, v0, W.copy(), b.copy(), c.copy(), u, f64=True)
    di = orc.conv_desc(d.N, d.C, d.H, d.W, d.K, d.R, d.S, 0, orc.ACT_IDENTITY, 1)
    lin = orc.conv_full_bwd(di, res.h0_sample, None, None, W, f64=True) + c[None, :, None, None]
    v1 = sigmoid(lin) if visible == 0 else lin
    np.testing.assert_allclose(res.v1, v1, rtol=1e-13, atol=1e-15)
    again = orc.crbm_cd1_step_units(d, visible, hidden_pool, res.v1, W.copy(), b.copy(), c.copy(), u, f64=True)
    np.testing.assert_array_equal(again.h0_prob, res.h1_prob)
    pos, bp = orc.conv_valid_wgrad(di, v0, res.h0_prob, None, None, f64=True)
    neg, bn = orc.conv_valid_wgrad(di, res.v1, res.h1_prob, None, None, f64=True)
    np.testing.assert_allclose(res.dW, (pos - neg) / d.N, atol=1e-13)
    np.testing.assert_allclose(res.db, (bp - bn) / d.N, atol=1e-13)
    np.testing.assert_allclose(res.dc, (v0 - res.v1).sum(axis=(0, 2, 3)) / d.N, atol=1e-13)
    np.testing.assert_allclose(res.recon_mse, ((v0 - res.v1) ** 2).mean(), rtol=1e-13)
    if hidden_pool == 1:
        z, _ = orc.conv_valid_fwd(di, v0, W, b, f64=True)
        np.testing.assert_allclose(res.h0_prob, sigmoid(z), rtol=1e-13)
        np.testing.assert_array_equal(res.h0_sample, (u < res.h0_prob) * 1.0)
    else:
        blocks = res.h0_prob.reshape(d.N, d.K, d.Ho // 2, 2, d.Wo // 2, 2).sum(axis=(3, 5))
        np.testing.assert_allclose(blocks, res.pool_prob, rtol=1e-13)
        assert np.all(blocks < 1.0)
        assert res.h0_sample.reshape(d.N, d.K, d.Ho // 2, 2, d.Wo // 2, 2).sum(axis=(3, 5)).max() <= 1.0
    # supplied samples override the uniforms; lr applies theta += lr * grad
    forced = orc.crbm_cd1_step_units(d, visible, hidden_pool, v0, W.copy(), b.copy(), c.copy(), None,
                                     h0_sample_in=res.h0_sample, f64=True)
    np.testing.assert_array_equal(forced.dW, res.dW)
    W2, b2, c2 = W.copy(), b.copy(), c.copy()
    orc.crbm_cd1_step_units(d, visible, hidden_pool, v0, W2, b2, c2, u, lr=0.25, f64=True)
    np.testing.assert_allclose(W2, W + 0.25 * res.dW, rtol=1e-14)
    np.testing.assert_allclose(b2, b + 0.25 * res.db, rtol=1e-14)
    np.testing.assert_allclose(c2, c + 0.25 * res.dc, rtol=1e-14)


def test_crbm_binary_variant_is_the_original_step():
    d, v0, W, b, c, r = crbm_inputs(420)
    u = r.random((d.N, d.K, d.Ho, d.Wo))
    a = orc.crbm_cd1_step(d, v0, W.copy(), b.copy(), c.copy(), u, f64=True)
    bb = orc.crbm_cd1_step_units(d, orc.VIS_BINARY, 1, v0, W.copy(), b.copy(), c.copy(), u, f64=True)
    for f in ("dW", "db", "dc", "h0_prob", "h0_sample", "v1", "h1_prob"):
        np.testing.assert_array_equal(getattr(a, f), getattr(bb, f))


def test_gaussian_visible_closed_form_at_zero_weights():
    """W = 0: the reconstruction is the visible bias itself, whatever was sampled."""
    d, v0, _, _, c, r = crbm_inputs(421, binary=False)
    W, b = np.zeros((d.K, d.C, d.R, d.S)), np.zeros(d.K)
    u = r.random((d.N, d.K, d.Ho // 2, d.Wo // 2))
    res = orc.crbm_cd1_step_units(d, orc.VIS_GAUSSIAN, 2, v0, W, b, c.copy(), u, f64=True)
    np.testing.assert_array_equal(res.v1, np.broadcast_to(c[None, :, None, None], v0.shape))
    np.testing.assert_allclose(res.h1_prob, 0.2, rtol=1e-15)
    np.testing.assert_allclose(res.db, 0.0, atol=1e-15)
    ref = np.zeros_like(W)
    for rr in range(d.R):
        for s in range(d.S):
            ref[:, :, rr, s] = 0.2 * (v0[:, :, rr:rr + d.Ho, s:s + d.Wo] - c[None, :, None, None]).sum(axis=(0, 2, 3))[None, :] / d.N
    np.testing.assert_allclose(res.dW, ref, atol=1e-13)


# ---------------------------------------------------------------- fully-connected RBM

def rbm_inputs(seed, B=5, nv=7, nh=4, binary=True):
    r = np.random.default_rng(seed)
    v0 = (r.random((B, nv)) < 0.4).astype(np.float64) if binary else r.normal(size=(B, nv))
    return v0, r.normal(size=(nh, nv)) * 0.4, r.normal(size=nh) * 0.3, r.normal(size=nv) * 0.3, r.random((B, nh))


@pytest.mark.parametrize("visible", [orc.VIS_BINARY, orc.VIS_GAUSSIAN])
def test_rbm_equals_crbm_on_one_pixel_images(visible):
    """A CRBM on 1x1 images with 1x1 filters is a fully-connected RBM over its channels,
    visible biases included."""
    B, nv, nh = 5, 7, 4
    v0, W, b, c, u = rbm_inputs(500 + visible, B, nv, nh, binary=(visible == 0))
    a = orc.rbm_cd1_step(B, nv, nh, visible, v0, W.copy(), b.copy(), c.copy(), u, f64=True)
    d = orc.conv_desc(B, nv, 1, 1, nh, 1, 1)
    cr = orc.crbm_cd1_step_units(d, visible, 1, v0.reshape(B, nv, 1, 1), W.reshape(nh, nv, 1, 1).copy(), b.copy(),
                                 c.copy(), u.reshape(B, nh, 1, 1), f64=True)
    np.testing.assert_array_equal(a.h0_sample, cr.h0_sample.reshape(B, nh))
    for f, shape in (("dW", (nh, nv)), ("db", (nh,)), ("dc", (nv,)), ("h0_prob", (B, nh)), ("v1", (B, nv)),
                     ("h1_prob", (B, nh))):
        np.testing.assert_allclose(getattr(a, f), getattr(cr, f).reshape(shape), rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(a.recon_mse, cr.recon_mse, rtol=1e-12)


def test_rbm_equals_crbm_with_image_sized_filters():
    """Filters as large as the image give one hidden unit per filter: a fully-connected RBM over
    the pixels (with one shared visible bias, as the CRBM has one per channel)."""
    B, H, Wd, nh = 4, 3, 5, 6
    nv = H * Wd
    v0, W, b, _, u = rbm_inputs(510, B, nv, nh)
    c = np.full(nv, 0.37)
    a = orc.rbm_cd1_step(B, nv, nh, 0, v0, W.copy(), b.copy(), c.copy(), u, f64=True)
    d = orc.conv_desc(B, 1, H, Wd, nh, H, Wd)
    cr = orc.crbm_cd1_step(d, v0.reshape(B, 1, H, Wd), W.reshape(nh, 1, H, Wd).copy(), b.copy(), np.array([0.37]),
                           u.reshape(B, nh, 1, 1), f64=True)
    np.testing.assert_allclose(a.dW, cr.dW.reshape(nh, nv), rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(a.db, cr.db, rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(a.dc.sum(), cr.dc[0], rtol=1e-12)
    np.testing.assert_allclose(a.v1, cr.v1.reshape(B, nv), rtol=1e-13)


def test_rbm_closed_forms_and_update():
    B, nv, nh = 6, 5, 3
    v0, W, b, c, u = rbm_inputs(520, B, nv, nh)
    z = np.zeros
    res = orc.rbm_cd1_step(B, nv, nh, 0, v0, z((nh, nv)), z(nh), z(nv), u, f64=True)
    assert np.all(res.h0_prob == 0.5) and np.all(res.v1 == 0.5) and np.all(res.h1_prob == 0.5)
    np.testing.assert_array_equal(res.h0_sample, (u < 0.5) * 1.0)
    np.testing.assert_allclose(res.dW, np.broadcast_to(0.5 * (v0 - 0.5).mean(axis=0), (nh, nv)), atol=1e-15)
    np.testing.assert_allclose(res.dc, (v0 - 0.5).mean(axis=0), atol=1e-15)
    # library matmul for the general case, with forced samples
    hs = (u < 0.3) * 1.0
    res = orc.rbm_cd1_step(B, nv, nh, 1, v0, W.copy(), b.copy(), c.copy(), None, h0_sample_in=hs, f64=True)
    h0p = sigmoid(v0 @ W.T + b)
    v1 = hs @ W + c
    h1p = sigmoid(v1 @ W.T + b)
    np.testing.assert_allclose(res.h0_prob, h0p, rtol=1e-13)
    np.testing.assert_allclose(res.v1, v1, rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(res.dW, (h0p.T @ v0 - h1p.T @ v1) / B, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(res.db, (h0p - h1p).mean(axis=0), rtol=1e-12, atol=1e-15)
    W2, b2, c2 = W.copy(), b.copy(), c.copy()
    orc.rbm_cd1_step(B, nv, nh, 1, v0, W2, b2, c2, None, h0_sample_in=hs, lr=0.5, f64=True)
    np.testing.assert_allclose(W2, W + 0.5 * res.dW, rtol=1e-14)
    np.testing.assert_allclose(b2, b + 0.5 * res.db, rtol=1e-14)
    np.testing.assert_allclose(c2, c + 0.5 * res.dc, rtol=1e-14)


# ---------------------------------------------------------------- fully-connected network

def dense_net(B=4, act=orc.ACT_SIGMOID):
    return orc.Net([], [(9, 7, act), (7, 6, act), (6, 5, orc.ACT_IDENTITY)], 5, batch=B)


def dense_inputs(net, seed):
    r = np.random.default_rng(seed)
    params = [np.ascontiguousarray(r.normal(size=s) * 0.6) for s in net.param_shapes()]
    x = r.normal(size=(net.batch, net.dense[0][0]))
    labels = r.integers(0, net.classes, net.batch).astype(np.int32)
    return params, x, labels


def test_dense_net_finite_differences():
    net = dense_net()
    params, x, labels = dense_inputs(net, 600)
    res = orc.cnn_train_step(net, [p.copy() for p in params], x, labels, 0.0, f64=True)
    h = 1e-5
    r = np.random.default_rng(6)
    for pi, p in enumerate(params):
        for t in r.choice(p.size, size=min(12, p.size), replace=False):
            pp = [q.copy() for q in params]
            pp[pi].reshape(-1)[t] += h
            up = orc.cnn_train_step(net, pp, x, labels, 0.0, f64=True).loss
            pp[pi].reshape(-1)[t] -= 2 * h
            dn = orc.cnn_train_step(net, pp, x, labels, 0.0, f64=True).loss
            np.testing.assert_allclose(res.grads[pi].reshape(-1)[t], (up - dn) / (2 * h), rtol=5e-6, atol=1e-9)


@pytest.mark.parametrize("act", [orc.ACT_SIGMOID, orc.ACT_RELU])
def test_dense_net_equals_cnn_behind_an_identity_convolution(act):
    """The same dense stack behind a 1x1 identity convolution over one-pixel images is a CNN the
    (separately pinned) CNN step accepts: loss, logits and dense gradients must agree."""
    net = dense_net(act=act)
    params, x, labels = dense_inputs(net, 601)
    a = orc.cnn_train_step(net, [p.copy() for p in params], x, labels, 0.0, f64=True)
    nin = net.dense[0][0]
    cnn = orc.Net([orc.conv_desc(net.batch, nin, 1, 1, nin, 1, 1, 0, orc.ACT_IDENTITY, 1)], net.dense, net.classes)
    cparams = [np.eye(nin).reshape(nin, nin, 1, 1).copy(), np.zeros(nin)] + [p.copy() for p in params]
    b = orc.cnn_train_step(cnn, cparams, x.reshape(net.batch, nin, 1, 1), labels, 0.0, f64=True)
    np.testing.assert_allclose(a.loss, b.loss, rtol=1e-14)
    np.testing.assert_allclose(a.logits, b.logits, rtol=1e-14)
    for ga, gb in zip(a.grads, b.grads[2:]):
        np.testing.assert_allclose(ga, gb, rtol=1e-13, atol=1e-16)
    lg, prob = orc.cnn_forward(net, params, x, f64=True)
    np.testing.assert_array_equal(lg, a.logits)
    h = x
    for q, (i, o, ac) in enumerate(net.dense):
        h = h @ params[2 * q].T + params[2 * q + 1]
        if q < len(net.dense) - 1:
            h = sigmoid(h) if ac == orc.ACT_SIGMOID else np.maximum(h, 0)
    np.testing.assert_allclose(lg, h, rtol=1e-12)
    e = np.exp(h - h.max(axis=1, keepdims=True))
    np.testing.assert_allclose(prob, e / e.sum(axis=1, keepdims=True), rtol=1e-12)


def test_dense_net_needs_a_batch_size():
    net = orc.Net([], [(4, 3, 0)], 3, batch=0)
    with pytest.raises(ValueError):
        orc.cnn_train_step(net, [np.zeros((3, 4)), np.zeros(3)], np.zeros((1, 4)), np.zeros(1, np.int32), 0.0, f64=True)
