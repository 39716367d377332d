"""Pins for the oracle's dense layers, softmax cross-entropy, SGD, the CNN step and the
CRBM CD-1 step (no GPU): library matmul, closed forms, invariants, composition from the
separately pinned conv trio, and finite differences of the whole network in double."""
import os

import numpy as np
import pytest

from oracle import oracle as orc

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def sigmoid(z):
    return 1 / (1 + np.exp(-z))


# ---------------------------------------------------------------- dense, loss, update

@pytest.mark.parametrize("act", [orc.ACT_IDENTITY, orc.ACT_SIGMOID, orc.ACT_RELU])
def test_dense_vs_numpy_matmul(act):
    r = np.random.default_rng(100 + act)
    B, nin, nout = 5, 7, 4
    a, W, b, dh = r.normal(size=(B, nin)), r.normal(size=(nout, nin)), r.normal(size=(nout,)), r.normal(size=(B, nout))
    z = a @ W.T + b
    h_ref = {0: z, 1: sigmoid(z), 2: np.maximum(z, 0)}[act]
    h = orc.dense_fwd(a, W, b, act, f64=True)
    np.testing.assert_allclose(h, h_ref, atol=1e-13)
    dzh = dh * {0: np.ones_like(z), 1: h_ref * (1 - h_ref), 2: (z > 0) * 1.0}[act]
    da, dW, db = orc.dense_bwd(a, W, h, dh, act, f64=True)
    np.testing.assert_allclose(da, dzh @ W, atol=1e-13)
    np.testing.assert_allclose(dW, dzh.T @ a, atol=1e-13)
    np.testing.assert_allclose(db, dzh.sum(0), atol=1e-13)


def test_softmax_ce_invariants_and_closed_form():
    for line in open(os.path.join(GOLD, "loss_at_zero_logits.txt")):
        if line.startswith("#"):
            continue
        classes, expect = int(line.split()[0]), float(line.split()[1])
        loss, prob, dl = orc.softmax_ce(np.zeros((4, classes)), np.arange(4) % classes, f64=True)
        assert abs(loss - expect) < 1e-14
        np.testing.assert_allclose(prob, 1.0 / classes, rtol=1e-14)
    r = np.random.default_rng(101)
    B, classes = 6, 9
    logits, labels = r.normal(size=(B, classes)) * 5, r.integers(0, classes, B)
    loss, prob, dl = orc.softmax_ce(logits, labels, f64=True)
    np.testing.assert_allclose(prob.sum(1), 1.0, rtol=1e-14)
    np.testing.assert_allclose(dl.sum(1), 0.0, atol=1e-15)
    e = np.exp(logits)
    np.testing.assert_allclose(prob, e / e.sum(1, keepdims=True), rtol=1e-12)
    np.testing.assert_allclose(loss, -np.log(prob[np.arange(B), labels]).mean(), rtol=1e-13)
    # shift invariance and no overflow at large logits
    loss2, _, _ = orc.softmax_ce(logits + 1000.0, labels, f64=True)
    np.testing.assert_allclose(loss2, loss, rtol=1e-10)
    # gradient by central differences
    h = 1e-6
    for (n, j) in [(0, 0), (3, 4), (5, 8)]:
        lp, lm = logits.copy(), logits.copy()
        lp[n, j] += h
        lm[n, j] -= h
        fd = (orc.softmax_ce(lp, labels, f64=True)[0] - orc.softmax_ce(lm, labels, f64=True)[0]) / (2 * h)
        np.testing.assert_allclose(dl[n, j], fd, rtol=1e-6, atol=1e-10)


def test_sgd_update():
    r = np.random.default_rng(102)
    t, g = r.normal(size=(3, 4)), r.normal(size=(3, 4))
    t0 = t.copy()
    orc.sgd(t, g, 0.25, f64=True)
    np.testing.assert_allclose(t, t0 - 0.25 * g, rtol=1e-15)
    t32 = t0.astype(np.float32)
    keep = t32.copy()
    orc.sgd(t32, g.astype(np.float32), 0.0)
    np.testing.assert_array_equal(t32, keep)


# ---------------------------------------------------------------- CNN step

def tiny_net(B=3, act=orc.ACT_SIGMOID):
    conv = [orc.conv_desc(B, 2, 10, 10, 3, 3, 3, 1, act, 2), orc.conv_desc(B, 3, 5, 5, 4, 2, 2, 0, act, 2)]
    dense = [(4 * 2 * 2, 6, act), (6, 5, orc.ACT_IDENTITY)]
    return orc.Net(conv, dense, 5)


def tiny_inputs(net, seed, dt=np.float64):
    r = np.random.default_rng(seed)
    params = [np.ascontiguousarray(r.normal(size=s) * 0.5, dtype=dt) for s in net.param_shapes()]
    d0 = net.conv[0]
    x = r.normal(size=(d0.N, d0.C, d0.H, d0.W)).astype(dt)
    labels = r.integers(0, net.classes, d0.N).astype(np.int32)
    return params, x, labels


def test_cnn_step_is_the_composition_of_its_layers():
    net = tiny_net(act=orc.ACT_RELU)
    params, x, labels = tiny_inputs(net, 200)
    res = orc.cnn_train_step(net, [p.copy() for p in params], x, labels, 0.0, f64=True)
    a, idxs, acts = x, [], [x]
    for l, d in enumerate(net.conv):
        a, idx = orc.conv_valid_fwd(d, a, params[2 * l], params[2 * l + 1], f64=True)
        acts.append(a)
        idxs.append(idx)
    flat = a.reshape(a.shape[0], -1)           # NCHW row-major flatten
    h1 = orc.dense_fwd(flat, params[4], params[5], orc.ACT_RELU, f64=True)
    logits = orc.dense_fwd(h1, params[6], params[7], orc.ACT_IDENTITY, f64=True)
    np.testing.assert_array_equal(res.logits, logits)
    loss, _, dl = orc.softmax_ce(logits, labels, f64=True)
    assert res.loss == loss
    dh1, dW2, db2 = orc.dense_bwd(h1, params[6], logits, dl, orc.ACT_IDENTITY, f64=True)
    dflat, dW1, db1 = orc.dense_bwd(flat, params[4], h1, dh1, orc.ACT_RELU, f64=True)
    g = dflat.reshape(a.shape)
    dw1, dbc1 = orc.conv_valid_wgrad(net.conv[1], acts[1], g, acts[2], idxs[1], f64=True)
    g0 = orc.conv_full_bwd(net.conv[1], g, acts[2], idxs[1], params[2], f64=True)
    dw0, dbc0 = orc.conv_valid_wgrad(net.conv[0], acts[0], g0, acts[1], idxs[0], f64=True)
    for got, ref in zip(res.grads, [dw0, dbc0, dw1, dbc1, dW1, db1, dW2, db2]):
        np.testing.assert_array_equal(got, ref)
    for got, ref in zip(res.pool_idx, idxs):
        np.testing.assert_array_equal(got, ref)


def test_cnn_step_finite_differences_whole_network():
    """Loss gradient w.r.t. 20 random entries of every parameter tensor, central differences in
    double (sigmoid net: smooth everywhere except pooling ties, which have measure zero)."""
    net = tiny_net()
    params, x, labels = tiny_inputs(net, 201)
    res = orc.cnn_train_step(net, [p.copy() for p in params], x, labels, 0.0, f64=True)
    r = np.random.default_rng(5)
    h = 1e-5
    for pi, p in enumerate(params):
        for t in r.choice(p.size, size=min(20, p.size), replace=False):
            pp = [q.copy() for q in params]
            pp[pi].reshape(-1)[t] += h
            up = orc.cnn_train_step(net, pp, x, labels, 0.0, f64=True).loss
            pp[pi].reshape(-1)[t] -= 2 * h
            dn = orc.cnn_train_step(net, pp, x, labels, 0.0, f64=True).loss
            np.testing.assert_allclose(res.grads[pi].reshape(-1)[t], (up - dn) / (2 * h), rtol=5e-6, atol=1e-9)


def test_cnn_step_sgd_update_and_lr_zero():
    net = tiny_net(act=orc.ACT_RELU)
    params, x, labels = tiny_inputs(net, 202, np.float32)
    p0 = [p.copy() for p in params]
    res = orc.cnn_train_step(net, p0, x, labels, 0.0)
    for a, b in zip(p0, params):
        np.testing.assert_array_equal(a, b)        # lr = 0 leaves parameters bit-identical
    p1 = [p.copy() for p in params]
    res1 = orc.cnn_train_step(net, p1, x, labels, 0.1)
    assert res1.loss == res.loss
    for new, old, g in zip(p1, params, res.grads):
        ref = (old.astype(np.float64) - np.float64(np.float32(0.1)) * g.astype(np.float64)).astype(np.float32)
        np.testing.assert_array_equal(new, ref)
    # one step downhill reduces the loss on the same batch
    assert orc.cnn_train_step(net, p1, x, labels, 0.0).loss < res.loss


def test_cnn_step_pool_idx_override_routes_gradient():
    net = tiny_net(act=orc.ACT_RELU)
    params, x, labels = tiny_inputs(net, 203)
    base = orc.cnn_train_step(net, [p.copy() for p in params], x, labels, 0.0, f64=True)
    same = orc.cnn_train_step(net, [p.copy() for p in params], x, labels, 0.0, pool_idx_in=base.pool_idx, f64=True)
    for a, b in zip(base.grads, same.grads):
        np.testing.assert_array_equal(a, b)
    moved = [i.copy() for i in base.pool_idx]
    moved[1] = (moved[1] + 1) % 4
    other = orc.cnn_train_step(net, [p.copy() for p in params], x, labels, 0.0, pool_idx_in=moved, f64=True)
    assert not np.array_equal(other.grads[2], base.grads[2])
    np.testing.assert_array_equal(other.grads[6], base.grads[6])   # layers above are unaffected


def test_cnn_step_activity_override_decides_relu_derivative():
    """The handed-in activity record replaces "output > 0" of a ReLU layer: the layer's own record
    changes nothing; switching one active unit off removes exactly that unit's share of the bias
    gradient (its pooled gradient, read off a composition of the separately pinned layers);
    switching an inactive one on adds it; layers above are unaffected; an all-zero record kills
    every gradient below the layer; a sigmoid layer ignores the record."""
    B = 2
    conv = [orc.conv_desc(B, 2, 10, 10, 3, 3, 3, 1, orc.ACT_RELU, 2), orc.conv_desc(B, 3, 5, 5, 4, 2, 2, 0, orc.ACT_RELU, 1)]
    net = orc.Net(conv, [(4 * 4 * 4, 6, orc.ACT_RELU), (6, 5, orc.ACT_IDENTITY)], 5)
    params, x, labels = tiny_inputs(net, 204)
    run = lambda **kw: orc.cnn_train_step(net, [p.copy() for p in params], x, labels, 0.0, f64=True, **kw)
    base = run()
    y1, _ = orc.conv_valid_fwd(conv[0], x, params[0], params[1], f64=True)
    y2, _ = orc.conv_valid_fwd(conv[1], y1, params[2], params[3], f64=True)
    own = [(y1 > 0).astype(np.uint8), (y2 > 0).astype(np.uint8)]
    same = run(active_in=own)
    for a, b in zip(base.grads, same.grads):
        np.testing.assert_array_equal(a, b)
    # the gradient that reaches layer 2's output, from the dense layers
    flat = y2.reshape(B, -1)
    h1 = orc.dense_fwd(flat, params[4], params[5], orc.ACT_RELU, f64=True)
    logits = orc.dense_fwd(h1, params[6], params[7], orc.ACT_IDENTITY, f64=True)
    _, _, dl = orc.softmax_ce(logits, labels, f64=True)
    dh1, _, _ = orc.dense_bwd(h1, params[6], logits, dl, orc.ACT_IDENTITY, f64=True)
    dflat, _, _ = orc.dense_bwd(flat, params[4], h1, dh1, orc.ACT_RELU, f64=True)
    dy2 = dflat.reshape(y2.shape)
    on = np.argwhere(own[1] == 1)[0]
    off = np.argwhere(own[1] == 0)[0]
    for pos, sign in ((on, -1.0), (off, +1.0)):
        rec = [own[0], own[1].copy()]
        rec[1][tuple(pos)] ^= 1
        got = run(active_in=rec)
        k = pos[1]
        expect = base.grads[3].copy()
        expect[k] += sign * dy2[tuple(pos)]
        np.testing.assert_allclose(got.grads[3], expect, rtol=1e-12, atol=1e-15)
        for p in (4, 5, 6, 7):
            np.testing.assert_array_equal(got.grads[p], base.grads[p])
    dead = run(active_in=[None, np.zeros_like(own[1])])
    for p in (0, 1, 2, 3):
        assert not dead.grads[p].any()
    np.testing.assert_array_equal(dead.grads[4], base.grads[4])
    # only layer 1 overridden (pooled layer): switching a unit with non-zero gradient off changes dw0
    rec0 = own[0].copy()
    rec0[tuple(np.argwhere(own[0] == 1)[0])] = 0
    assert not np.array_equal(run(active_in=[rec0, None]).grads[0], base.grads[0])
    np.testing.assert_array_equal(run(active_in=[rec0, None]).grads[2], base.grads[2])
    # a sigmoid layer's derivative does not look at the record
    snet = tiny_net()
    sp, sx, sl = tiny_inputs(snet, 205)
    a = orc.cnn_train_step(snet, [p.copy() for p in sp], sx, sl, 0.0, f64=True)
    zeros = [np.zeros(d.out_shape, np.uint8) for d in snet.conv]
    b = orc.cnn_train_step(snet, [p.copy() for p in sp], sx, sl, 0.0, f64=True, active_in=zeros)
    for u, v in zip(a.grads, b.grads):
        np.testing.assert_array_equal(u, v)


# ---------------------------------------------------------------- CRBM CD-1

def crbm_inputs(seed, N=3, C=2, H=9, W=8, K=4, R=3, S=3):
    r = np.random.default_rng(seed)
    d = orc.conv_desc(N, C, H, W, K, R, S)
    v0 = (r.random((N, C, H, W)) < 0.3).astype(np.float64)
    Wt = r.normal(size=(K, C, R, S)) * 0.3
    b, c = r.normal(size=(K,)) * 0.2, r.normal(size=(C,)) * 0.2
    u = r.random((N, K, d.Ho, d.Wo))
    return d, v0, Wt, b, c, u


def test_crbm_closed_form_at_zero_weights():
    d, v0, _, _, _, u = crbm_inputs(300)
    W, b, c = np.zeros((d.K, d.C, d.R, d.S)), np.zeros(d.K), np.zeros(d.C)
    res = orc.crbm_cd1_step(d, v0, W, b, c, u, f64=True)
    assert np.all(res.h0_prob == 0.5) and np.all(res.h1_prob == 0.5)
    np.testing.assert_array_equal(res.h0_sample, (u < 0.5) * 1.0)
    # v1 = sigmoid(0) = 1/2 everywhere because W = 0, whatever was sampled
    assert np.all(res.v1 == 0.5)
    ref = np.zeros_like(W)
    for r in range(d.R):
        for s in range(d.S):
            ref[:, :, r, s] = 0.5 * (v0[:, :, r:r + d.Ho, s:s + d.Wo] - 0.5).sum(axis=(0, 2, 3))[None, :] / d.N
    np.testing.assert_allclose(res.dW, ref, atol=1e-13)
    np.testing.assert_allclose(res.db, 0.0, atol=1e-15)
    np.testing.assert_allclose(res.dc, (v0 - 0.5).sum(axis=(0, 2, 3)) / d.N, atol=1e-13)
    np.testing.assert_allclose(res.recon_mse, ((v0 - 0.5) ** 2).mean(), rtol=1e-13)


def test_crbm_forced_samples():
    d, v0, W, b, c, u = crbm_inputs(301)
    # u == 1 -> nothing fires -> v1 = sigmoid(c)
    res = orc.crbm_cd1_step(d, v0, W.copy(), b.copy(), c.copy(), np.ones_like(u), f64=True)
    assert np.all(res.h0_sample == 0)
    np.testing.assert_allclose(res.v1, np.broadcast_to(sigmoid(c)[None, :, None, None], v0.shape), rtol=1e-14)
    # u == 0 -> every unit fires -> v1 = sigmoid(c + sum of the taps that reach the pixel)
    res = orc.crbm_cd1_step(d, v0, W.copy(), b.copy(), c.copy(), np.zeros_like(u), f64=True)
    assert np.all(res.h0_sample == 1)
    ref = np.zeros(v0.shape[1:])
    for i in range(d.H):
        for j in range(d.W):
            for r in range(d.R):
                for s in range(d.S):
                    if 0 <= i - r < d.Ho and 0 <= j - s < d.Wo:
                        ref[:, i, j] += W[:, :, r, s].sum(0)
    np.testing.assert_allclose(res.v1[0], sigmoid(c[:, None, None] + ref), rtol=1e-13)
    assert 0.0 <= res.recon_mse <= 1.0


def test_crbm_is_the_composition_of_the_trio():
    d, v0, W, b, c, u = crbm_inputs(302)
    res = orc.crbm_cd1_step(d, v0, W.copy(), b.copy(), c.copy(), u, f64=True)
    ds = orc.conv_desc(d.N, d.C, d.H, d.W, d.K, d.R, d.S, 0, orc.ACT_SIGMOID, 1)
    di = orc.conv_desc(d.N, d.C, d.H, d.W, d.K, d.R, d.S, 0, orc.ACT_IDENTITY, 1)
    h0p, _ = orc.conv_valid_fwd(ds, v0, W, b, f64=True)
    h0s = (u < h0p) * 1.0
    v1 = sigmoid(orc.conv_full_bwd(di, h0s, None, None, W, f64=True) + c[None, :, None, None])
    h1p, _ = orc.conv_valid_fwd(ds, v1, W, b, f64=True)
    pos, bp = orc.conv_valid_wgrad(di, v0, h0p, None, None, f64=True)
    neg, bn = orc.conv_valid_wgrad(di, v1, h1p, None, None, f64=True)
    np.testing.assert_array_equal(res.h0_prob, h0p)
    np.testing.assert_array_equal(res.h0_sample, h0s)
    np.testing.assert_allclose(res.v1, v1, rtol=1e-14)
    np.testing.assert_allclose(res.h1_prob, h1p, rtol=1e-13)
    np.testing.assert_allclose(res.dW, (pos - neg) / d.N, atol=1e-13)
    np.testing.assert_allclose(res.db, (bp - bn) / d.N, atol=1e-13)
    np.testing.assert_allclose(res.dc, (v0 - v1).sum(axis=(0, 2, 3)) / d.N, atol=1e-13)
    # supplied samples override the uniforms; lr applies theta += lr * grad
    res2 = orc.crbm_cd1_step(d, v0, W.copy(), b.copy(), c.copy(), None, h0_sample_in=h0s, f64=True)
    np.testing.assert_array_equal(res2.dW, res.dW)
    W2, b2, c2 = W.copy(), b.copy(), c.copy()
    orc.crbm_cd1_step(d, v0, W2, b2, c2, u, lr=0.5, f64=True)
    np.testing.assert_allclose(W2, W + 0.5 * res.dW, rtol=1e-14)
    np.testing.assert_allclose(b2, b + 0.5 * res.db, rtol=1e-14)
    np.testing.assert_allclose(c2, c + 0.5 * res.dc, rtol=1e-14)


# ---------------------------------------------------------------- inference pass

def _np_forward(net, params, x):
    """Independent forward pass: scipy's 2-D cross-correlation per (filter, channel) pair, numpy
    reshapes for the 2x2 max pool, numpy matmul for the dense layers."""
    from scipy.signal import correlate2d
    act = {orc.ACT_IDENTITY: lambda z: z, orc.ACT_SIGMOID: sigmoid, orc.ACT_RELU: lambda z: np.maximum(z, 0)}
    a = np.asarray(x, np.float64)
    L = len(net.conv)
    for l, d in enumerate(net.conv):
        w, b = params[2 * l].astype(np.float64), params[2 * l + 1].astype(np.float64)
        ap = np.pad(a, ((0, 0), (0, 0), (d.pad, d.pad), (d.pad, d.pad)))
        N, K = a.shape[0], w.shape[0]
        Ho, Wo = ap.shape[2] - w.shape[2] + 1, ap.shape[3] - w.shape[3] + 1
        z = np.zeros((N, K, Ho, Wo))
        for n in range(N):
            for k in range(K):
                for c in range(w.shape[1]):
                    z[n, k] += correlate2d(ap[n, c], w[k, c], mode="valid")
                z[n, k] += b[k]
        a = act[d.act](z)
        if d.pool == 2:
            a = a.reshape(N, K, Ho // 2, 2, Wo // 2, 2).max(axis=(3, 5))
    a = a.reshape(a.shape[0], -1)
    for q, (nin, nout, ac) in enumerate(net.dense):
        W, b = params[2 * (L + q)].astype(np.float64), params[2 * (L + q) + 1].astype(np.float64)
        z = a @ W.T + b
        a = z if q == len(net.dense) - 1 else act[ac](z)
    e = np.exp(a - a.max(1, keepdims=True))
    return a, e / e.sum(1, keepdims=True)


def _small_net(act, pad):
    conv = [orc.conv_desc(3, 2, 10, 12, 4, 3, 3, pad, act, 2)]
    h1, w1 = (10 + 2 * pad - 2) // 2, (12 + 2 * pad - 2) // 2
    conv.append(orc.conv_desc(3, 4, h1, w1, 3, 3, 2, 0, act, 1))
    feat = 3 * (h1 - 2) * (w1 - 1)
    return orc.Net(conv, [(feat, 6, act), (6, 5, orc.ACT_IDENTITY)], 5)


@pytest.mark.parametrize("act,pad", [(orc.ACT_SIGMOID, 0), (orc.ACT_RELU, 1)])
def test_cnn_forward_vs_scipy_numpy(act, pad):
    net = _small_net(act, pad)
    r = np.random.default_rng(300 + act)
    params = [r.normal(size=s) * 0.5 for s in net.param_shapes()]
    x = r.normal(size=(3, 2, 10, 12))
    logits, prob = orc.cnn_forward(net, params, x, f64=True)
    ref_logits, ref_prob = _np_forward(net, params, x)
    np.testing.assert_allclose(logits, ref_logits, atol=1e-12)
    np.testing.assert_allclose(prob, ref_prob, atol=1e-13)
    np.testing.assert_allclose(prob.sum(1), 1.0, rtol=1e-14)
    # the float instance rounds once per layer: same values to fp32 accuracy
    l32, p32 = orc.cnn_forward(net, [p.astype(np.float32) for p in params], x.astype(np.float32))
    assert np.abs(l32 - ref_logits).max() <= 2e-5 * max(1.0, np.abs(ref_logits).max())
    assert np.abs(p32 - ref_prob).max() <= 2e-6


def test_cnn_forward_closed_forms():
    net = _small_net(orc.ACT_SIGMOID, 0)
    shapes = net.param_shapes()
    x = np.random.default_rng(310).normal(size=(3, 2, 10, 12))
    # all parameters zero: logits 0, every class equally likely
    logits, prob = orc.cnn_forward(net, [np.zeros(s) for s in shapes], x, f64=True)
    assert not logits.any()
    np.testing.assert_allclose(prob, 0.2, rtol=1e-15)
    # only the output bias set: logits = bias, probabilities = softmax(bias), whatever the image
    params = [np.zeros(s) for s in shapes]
    params[-1][:] = [0.0, np.log(2.0), np.log(3.0), 0.0, np.log(4.0)]
    logits, prob = orc.cnn_forward(net, params, x, f64=True)
    np.testing.assert_allclose(logits, np.tile(params[-1], (3, 1)), atol=1e-15)
    np.testing.assert_allclose(prob, np.tile(np.array([1, 2, 3, 1, 4]) / 11.0, (3, 1)), rtol=1e-14)
    # a constant added to the output bias leaves the probabilities alone, also when huge
    r = np.random.default_rng(311)
    params = [r.normal(size=s) for s in shapes]
    _, p0 = orc.cnn_forward(net, params, x, f64=True)
    params[-1] += 700.0
    _, p1 = orc.cnn_forward(net, params, x, f64=True)
    np.testing.assert_allclose(p1, p0, rtol=1e-9)


def test_cnn_forward_matches_training_pass_logits():
    net = _small_net(orc.ACT_RELU, 1)
    r = np.random.default_rng(320)
    params = [(r.normal(size=s) * 0.5).astype(np.float32) for s in net.param_shapes()]
    x = r.normal(size=(3, 2, 10, 12)).astype(np.float32)
    logits, _ = orc.cnn_forward(net, params, x)
    step = orc.cnn_train_step(net, [p.copy() for p in params], x, np.array([0, 1, 2]), lr=0.0)
    assert np.array_equal(logits, step.logits)


# ---------------------------------------------------------------- momentum and weight decay

def test_sgd_momentum_closed_forms():
    r = np.random.default_rng(400)
    th0, g = r.normal(size=50), r.normal(size=50)
    # no momentum, no decay: exactly the plain update
    a, va = th0.copy(), np.zeros(50)
    orc.sgd_momentum(a, va, g, 0.1, 0.0, 0.0, f64=True)
    b = orc.sgd(th0.copy(), g, 0.1, f64=True)
    assert np.array_equal(a, b) and np.array_equal(va, -0.1 * g)
    # constant gradient, n steps: v_n = -lr g (1 - mu^n)/(1 - mu), theta_n = theta_0 + sum of the v_k
    lr, mu, n = 0.05, 0.9, 7
    th, v = th0.copy(), np.zeros(50)
    for _ in range(n):
        orc.sgd_momentum(th, v, g, lr, mu, 0.0, f64=True)
    geo = lambda k: (1 - mu ** k) / (1 - mu)
    np.testing.assert_allclose(v, -lr * g * geo(n), rtol=1e-13)
    np.testing.assert_allclose(th, th0 - lr * g * sum(geo(k) for k in range(1, n + 1)), rtol=1e-12, atol=1e-14)
    # decay only, zero gradient: theta shrinks geometrically by (1 - lr decay) per step
    th, v = th0.copy(), np.zeros(50)
    for _ in range(5):
        orc.sgd_momentum(th, v, np.zeros(50), 0.1, 0.0, 0.3, f64=True)
    np.testing.assert_allclose(th, th0 * (1 - 0.1 * 0.3) ** 5, rtol=1e-13)
    # one general step against the formula written out with numpy
    th, v = th0.copy(), r.normal(size=50)
    v_ref = 0.8 * v - 0.02 * (g + 0.01 * th)
    th_ref = th + v_ref
    orc.sgd_momentum(th, v, g, 0.02, 0.8, 0.01, f64=True)
    np.testing.assert_allclose(v, v_ref, rtol=1e-14)
    np.testing.assert_allclose(th, th_ref, rtol=1e-14)
