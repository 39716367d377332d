"""GPU-vs-oracle parity of the conv trio, the CRBM CD-1 step and the CNN training step.

Every test calls the HIP path through the C ABI on seeded inputs and compares it element by
element with the CPU oracle.  Tolerances: 1e-4 (forward) and 5e-4 (gradients) on the
per-tensor metric max|got-ref| / max|ref|; pooling indices and Bernoulli samples are
integer decisions taken from fp32 values, so differences are allowed only at (near) ties and
downstream tensors are compared with the oracle re-run on the GPU's decisions.
"""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import oracle as orc
from paper_1804_04512_amd import binding as B
from paper_1804_04512_amd import workloads as wl
from paper_1804_04512_amd.workloads import ConvSpec, DenseSpec

from helpers import (ACT, TOL_FWD, TOL_GRAD, check_idx_bytes, check_idx_flags_against, check_pool_idx,
                     check_relu_activity, max_rel_err, odesc, onet)

pytestmark = pytest.mark.gpu


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


def rand_layer(cs: ConvSpec, seed: int):
    r = np.random.default_rng(seed)
    x = r.standard_normal(cs.x_shape).astype(np.float32)
    w = (r.standard_normal(cs.w_shape) * np.sqrt(2.0 / (cs.C * cs.R * cs.S))).astype(np.float32)
    b = (r.standard_normal((cs.K,)) * 0.1).astype(np.float32)
    dy = r.standard_normal(cs.y_shape).astype(np.float32)
    return x, w, b, dy


def gpu_trio(cs: ConvSpec, x, w, b, dy, y_in=None, idx_in=None, flagged=False):
    """Runs fwd, then bwd and wgrad on (y_in, idx_in) when given, else on the GPU's own.
    flagged: the backward passes get no layer output (pooled ReLU: activity flags in idx).
    The returned idx is the raw byte the library wrote: position in bits 0-1, ReLU flag in bit 2."""
    xd, wd, bd, dyd = dev(x), dev(w), dev(b), dev(dy)
    y = torch.full(cs.y_shape, float("nan"), device="cuda")
    idx = torch.full(cs.y_shape, 255, dtype=torch.uint8, device="cuda") if cs.pool == 2 else None
    B.dll_conv_valid_fwd(cs, xd, wd, bd, y, idx)
    yb = None if flagged else (y if y_in is None else dev(y_in))
    ib = idx if idx_in is None else dev(idx_in)
    dx = torch.full(cs.x_shape, float("nan"), device="cuda")
    B.dll_conv_full_bwd(cs, dyd, yb, ib, wd, dx)
    ws = B.workspace(B.dll_conv_workspace_bytes(cs))
    dw = torch.full(cs.w_shape, float("nan"), device="cuda")
    db = torch.full((cs.K,), float("nan"), device="cuda")
    B.dll_conv_valid_wgrad(cs, xd, dyd, yb, ib, dw, db, ws)
    # the same pass as its two launches, each a call of its own: bit for bit the same gradients
    ws2 = B.workspace(B.dll_conv_workspace_bytes(cs))
    dw2, db2 = torch.full_like(dw, float("nan")), torch.full_like(db, float("nan"))
    B.dll_conv_valid_wgrad_partial(cs, xd, dyd, yb, ib, ws2)
    B.dll_conv_valid_wgrad_finish(cs, dw2, db2, ws2)
    assert torch.equal(dw2, dw) and torch.equal(db2, db), "partial + finish differ from the one call"
    return host(y), (host(idx) if idx is not None else None), host(dx), host(dw), host(db)


def check_trio(cs: ConvSpec, x, w, b, dy):
    d = odesc(cs)
    y_o, idx_o = orc.conv_valid_fwd(d, x, w, b)
    y_g, raw_g, dx_own, dw_own, db_own = gpu_trio(cs, x, w, b, dy)
    assert max_rel_err(y_g, y_o) <= TOL_FWD
    idx_g = None
    if cs.pool == 2:
        pre, _ = orc.conv_valid_fwd(odesc(cs, pool=1), x, w, b)
        idx_g = check_idx_bytes(raw_g, cs.act == "relu", y_g)
        check_pool_idx(idx_g, idx_o, pre, y_o)
        if cs.act == "relu":
            # without the layer output the backward passes take act' from the flags: the very same
            # decisions as y > 0 on the GPU's own y.  Other kernels may take the flagged layers (the
            # minimal-filtering forms of the data and filter gradients), so the results agree with the
            # unflagged route's up to rounding, and they are checked against the oracle on their own:
            # the oracle gets the GPU's decisions (positions, and a 0/1 output standing for the flags)
            _, _, dx_f, dw_f, db_f = gpu_trio(cs, x, w, b, dy, flagged=True)
            assert max_rel_err(dw_f, dw_own) <= 5e-6 and max_rel_err(db_f, db_own) <= 5e-6
            assert max_rel_err(dx_f, dx_own) <= 2e-6
            on = ((raw_g & 4) == 0).astype(np.float32)
            assert max_rel_err(dx_f, orc.conv_full_bwd(d, dy, on, idx_g, w)) <= TOL_GRAD
            dw_o2, db_o2 = orc.conv_valid_wgrad(d, x, dy, on, idx_g)
            assert max_rel_err(dw_f, dw_o2) <= TOL_GRAD and max_rel_err(db_f, db_o2) <= TOL_GRAD
    # backward ops on identical inputs (the oracle's y and the GPU's own index decisions)
    use_idx = idx_g if cs.pool == 2 else None
    _, _, dx_g, dw_g, db_g = gpu_trio(cs, x, w, b, dy, y_in=y_o, idx_in=use_idx)
    dx_o = orc.conv_full_bwd(d, dy, y_o, use_idx, w)
    dw_o, db_o = orc.conv_valid_wgrad(d, x, dy, y_o, use_idx)
    assert max_rel_err(dx_g, dx_o) <= TOL_GRAD
    assert max_rel_err(dw_g, dw_o) <= TOL_GRAD
    assert max_rel_err(db_g, db_o) <= TOL_GRAD


CASES = [
    # N, C, H, W, K, R, S, pad, act, pool
    ConvSpec(1, 1, 3, 3, 1, 2, 2, 0, "identity", 1),          # smallest meaningful layer
    ConvSpec(2, 3, 12, 10, 5, 3, 3, 1, "relu", 2),            # ragged: everything below one tile
    ConvSpec(2, 1, 28, 28, 8, 5, 5, 0, "sigmoid", 1),         # MNIST-like, width 24 overhangs the 32-wide tile
    ConvSpec(3, 8, 12, 12, 8, 5, 5, 0, "relu", 2),            # 8x8 pre-pool map: shallow-tile instance
    ConvSpec(2, 3, 70, 75, 12, 5, 5, 2, "relu", 1),           # several tiles + ragged tail both ways, odd width
    ConvSpec(2, 12, 36, 68, 24, 3, 3, 1, "relu", 2),          # two N-tiles, 3 tiles wide with a tail
    ConvSpec(2, 1, 28, 28, 40, 9, 9, 0, "sigmoid", 1),        # CRBM shape: three N-tiles, single channel
    ConvSpec(1, 20, 20, 34, 50, 3, 3, 1, "sigmoid", 2),       # channel chunks 16+4, filter groups 48+2
    ConvSpec(2, 16, 40, 40, 16, 3, 3, 1, "relu", 2),          # config-5 style block
    ConvSpec(3, 16, 48, 64, 16, 3, 3, 1, "relu", 2),          # whole 16 x 32 tiles: the forward pass takes the minimal-filtering kernel
    ConvSpec(2, 16, 40, 64, 32, 3, 3, 1, "relu", 2),          # 16 -> 32 on whole 8 x 32 tiles: backward-data in two 16-channel chunks
    ConvSpec(25, 16, 64, 128, 16, 3, 3, 1, "relu", 2),        # 800 tiles of the minimal-filtering kernel: one whole round of 768 workgroups + a partial one
    ConvSpec(1, 32, 32, 32, 32, 3, 3, 1, "relu", 2),          # config-5 conv4 shape
    ConvSpec(3, 32, 24, 40, 16, 3, 3, 1, "relu", 2),          # 32 -> 16: two channel tiles, one filter tile; a ragged second column segment
    ConvSpec(5, 16, 36, 72, 32, 3, 3, 1, "relu", 2),          # 16 -> 32 on 18 block rows: row groups with a short last one, three column segments (the last 8 wide)
    ConvSpec(2, 32, 20, 8, 32, 3, 3, 1, "relu", 2),           # 32 -> 32 on a map narrower than one column segment
    # streaming minimal-filtering kernels (16 channels in; forward 16 or 32 filters, backward-data 16 -> 16)
    ConvSpec(12, 16, 256, 256, 16, 3, 3, 1, "relu", 2),       # 768 work items on 512 workgroups: wavefronts pass from one item to the next with rows in flight
    ConvSpec(6, 16, 256, 264, 32, 3, 3, 1, "relu", 2),        # two filter groups, nine column segments: the last group of two has one, a wavefront pair skips items
    ConvSpec(3, 16, 18, 40, 16, 3, 3, 1, "relu", 2),          # nine block rows (a short last row group), a second segment of 8 columns
    # first layers of image networks (one to three channels in, at most 16 filters): the filter gradient forms dz in registers
    ConvSpec(3, 3, 24, 72, 16, 3, 3, 1, "relu", 2),           # RGB, a whole 64-pixel strip and a ragged one of 8 pixels
    ConvSpec(2, 3, 36, 328, 16, 3, 3, 1, "relu", 2),          # six strips: two groups of four, the second with two strips sitting out; 18 window rows
    ConvSpec(2, 1, 20, 64, 8, 3, 3, 1, "relu", 2),            # grey-scale, eight filters: tap columns 9.. and filters 8.. are padding
    ConvSpec(1, 2, 10, 8, 5, 3, 3, 1, "relu", 2),             # far below one strip
    ConvSpec(2, 2, 9, 14, 3, 2, 4, 0, "identity", 1),         # non-square filter
    ConvSpec(2, 4, 11, 9, 6, 1, 1, 0, "relu", 1),             # 1x1 filter, odd map
    ConvSpec(1, 40, 20, 20, 1, 9, 9, 0, "identity", 1),       # single filter, deep contraction
    ConvSpec(2, 24, 24, 40, 10, 3, 3, 1, "sigmoid", 1),       # 24 channels = three 8-channel chunks of the 3x3 instance
    ConvSpec(3, 12, 16, 32, 24, 3, 3, 1, "relu", 2),          # its backward-data pass: 24 -> 12 channels through pooling
    # few input channels: their backward-data pass has few OUTPUT channels and takes the banded-filter kernel
    ConvSpec(3, 3, 20, 22, 6, 7, 7, 0, "sigmoid", 1),         # three channels, 14x16 maps back to 20x22: 2x2 tiles with tails
    ConvSpec(2, 2, 19, 17, 5, 5, 5, 2, "relu", 1),            # two channels, padded, odd sizes
    ConvSpec(2, 1, 16, 33, 20, 3, 5, 1, "identity", 1),       # one channel, non-square filter, 20 source channels = 3 rounds
    # deep padded 3x3 layers: the specialised engine keeps every channel chunk's filter slice in LDS
    ConvSpec(2, 48, 24, 32, 32, 3, 3, 1, "relu", 2),          # three 16-channel chunks: 97 KB of LDS (above the 64 KB default limit)
    ConvSpec(1, 128, 20, 32, 32, 3, 3, 1, "sigmoid", 1),      # eight chunks would need 189 KB: falls through to the generic engine
    ConvSpec(1, 256, 18, 32, 16, 3, 3, 1, "relu", 2),         # 32 8-channel chunks (168 KB): generic engine forward; backward-data 16 -> 256
    ConvSpec(1, 16, 24, 32, 112, 3, 3, 1, "relu", 1),         # 112 filters: the backward-data pass has 112 source channels
]


@pytest.mark.parametrize("cs", CASES, ids=lambda c: f"N{c.N}C{c.C}_{c.H}x{c.W}_K{c.K}_{c.R}x{c.S}p{c.pad}_{c.act}_pool{c.pool}")
def test_trio_matches_oracle(cs):
    x, w, b, dy = rand_layer(cs, 1000 + cs.C * 7 + cs.K)
    check_trio(cs, x, w, b, dy)


FFT_CASES = [
    ConvSpec(2, 1, 28, 28, 40, 9, 9, 0, "sigmoid", 1),        # CRBM shape: 20x20 maps, 9x9 filters, full size 28 -> 32x32
    ConvSpec(3, 5, 40, 36, 7, 15, 11, 0, "identity", 1),      # large non-square filters, 26x26 maps, full 40x36 -> 64x64
    ConvSpec(2, 3, 30, 22, 6, 5, 5, 2, "relu", 2),            # padded layer (the crop starts at 2), pooled ReLU
    ConvSpec(2, 4, 24, 24, 8, 3, 3, 1, "sigmoid", 2),         # pooled sigmoid: act' from the pooled output
    ConvSpec(1, 2, 64, 64, 3, 17, 17, 0, "relu", 1),          # the largest supported full size, 48x48 maps
    ConvSpec(2, 2, 3, 5, 3, 2, 4, 0, "identity", 1),          # tiny: padded sides 4 x 8, fewer butterflies than threads
    ConvSpec(1, 1, 1, 1, 1, 1, 1, 0, "identity", 1),          # degenerate: a single product
    ConvSpec(63, 33, 10, 12, 2, 3, 3, 0, "relu", 1),          # enough (pair, channel) work for the 2 x 2 tiles, both edges ragged
]


def test_trio_on_a_tensor_beyond_2_gib():
    """A first-layer shape whose input holds 553 M elements (2.2 GB): the specialised kernels address
    their tensors through 32-bit byte offsets and must all step aside (forward and filter gradient
    run on the general kernels), while the backward-data pass, whose SOURCE is the 1.1 GB pooled
    gradient, stays on the 3x3 engine and writes a destination beyond 2 GiB."""
    cs = ConvSpec(33, 1, 4096, 4096, 2, 3, 3, 1, "relu", 2)
    assert 4 * cs.N * cs.C * cs.H * cs.W > 2 ** 31 > cs.N * cs.C * cs.H * cs.W
    r = np.random.default_rng(77031)
    x = r.standard_normal(cs.x_shape, dtype=np.float32)
    w = (r.standard_normal(cs.w_shape) * np.sqrt(2.0 / 9.0)).astype(np.float32)
    b = (r.standard_normal((cs.K,)) * 0.1).astype(np.float32)
    dy = r.standard_normal(cs.y_shape, dtype=np.float32)
    check_trio(cs, x, w, b, dy)


@pytest.mark.parametrize("cs", FFT_CASES, ids=lambda c: f"N{c.N}C{c.C}_{c.H}x{c.W}_K{c.K}_{c.R}x{c.S}p{c.pad}_{c.act}_pool{c.pool}")
def test_full_convolution_through_fft_matches_oracle(cs):
    """Backward-data computed through the Fourier transform against the oracle's plain sum, and
    against the direct kernel; with the ReLU flags instead of the layer output as well."""
    x, w, b, dy = rand_layer(cs, 3000 + cs.R * 13 + cs.K)
    d = odesc(cs)
    y_o, idx_o = orc.conv_valid_fwd(d, x, w, b)
    dx_o = orc.conv_full_bwd(d, dy, y_o, idx_o, w)
    idx = dev(idx_o) if cs.pool == 2 else None
    ws = B.workspace(B.dll_conv_full_fft_workspace_bytes(cs))
    assert B.dll_conv_full_fft_workspace_bytes(cs) > 0
    dx_f = torch.full(cs.x_shape, float("nan"), device="cuda")
    B.dll_conv_full_bwd_fft(cs, dev(dy), dev(y_o), idx, dev(w), dx_f, ws)
    assert max_rel_err(host(dx_f), dx_o) <= TOL_GRAD
    if cs.R * cs.S <= 144:   # filters the direct kernels take
        dx_d = torch.full(cs.x_shape, float("nan"), device="cuda")
        B.dll_conv_full_bwd(cs, dev(dy), dev(y_o), idx, dev(w), dx_d)
        assert max_rel_err(host(dx_f), host(dx_d)) <= 1e-5
    if cs.act == "relu" and cs.pool == 2:
        # the library's own forward pass writes the activity flags; without y they decide act'
        yg = torch.empty(cs.y_shape, device="cuda")
        ig = torch.empty(cs.y_shape, dtype=torch.uint8, device="cuda")
        B.dll_conv_valid_fwd(cs, dev(x), dev(w), dev(b), yg, ig)
        a, c = torch.empty(cs.x_shape, device="cuda"), torch.empty(cs.x_shape, device="cuda")
        B.dll_conv_full_bwd_fft(cs, dev(dy), None, ig, dev(w), a, ws)
        B.dll_conv_full_bwd_fft(cs, dev(dy), yg, ig, dev(w), c, ws)
        assert np.array_equal(host(a), host(c))


def test_full_convolution_through_fft_limits():
    big = ConvSpec(1, 1, 66, 20, 2, 3, 3, 0, "identity", 1)   # full size 66 rows: beyond one LDS image
    assert B.dll_conv_full_fft_workspace_bytes(big) == 0
    t = lambda *s: torch.zeros(s, device="cuda")
    with pytest.raises(B.DllError) as e:
        B.dll_conv_full_bwd_fft(big, t(*big.y_shape), None, None, t(*big.w_shape), t(*big.x_shape), B.workspace(1 << 20))
    assert e.value.status == 3
    ok = ConvSpec(1, 2, 12, 12, 3, 5, 5, 0, "identity", 1)
    with pytest.raises(B.DllError) as e:                     # workspace too small
        B.dll_conv_full_bwd_fft(ok, t(*ok.y_shape), None, None, t(*ok.w_shape), t(*ok.x_shape), B.workspace(256))
    assert e.value.status == 4


def test_config1_single_conv_layer():
    w1 = wl.config1()
    check_trio(w1.conv, w1.x, w1.w, w1.bias, w1.dy)


def test_fwd_without_bias_and_shift_identity():
    """A delta filter turns the backward-data pass into a zero-filled shift (exact in fp32)."""
    cs = ConvSpec(1, 1, 12, 37, 1, 3, 3, 0, "identity", 1)
    r = np.random.default_rng(5)
    dz = r.standard_normal(cs.y_shape).astype(np.float32)
    w = np.zeros(cs.w_shape, np.float32)
    w[0, 0, 1, 2] = 1.0
    dx = torch.empty(cs.x_shape, device="cuda")
    B.dll_conv_full_bwd(cs, dev(dz), None, None, dev(w), dx)
    ref = np.zeros(cs.x_shape, np.float32)
    ref[0, 0, 1:11, 2:37] = dz[0, 0]
    np.testing.assert_array_equal(host(dx), ref)
    x = r.standard_normal(cs.x_shape).astype(np.float32)
    y = torch.empty(cs.y_shape, device="cuda")
    B.dll_conv_valid_fwd(cs, dev(x), dev(w), None, y)
    np.testing.assert_array_equal(host(y)[0, 0], x[0, 0, 1:11, 2:37])


def test_wgrad_is_bit_reproducible():
    cs = ConvSpec(4, 16, 40, 40, 16, 3, 3, 1, "relu", 2)
    x, w, b, dy = rand_layer(cs, 77)
    for flagged in (False, True):   # the direct kernel, and the minimal-filtering one that takes the flagged layer
        a = gpu_trio(cs, x, w, b, dy, flagged=flagged)
        c = gpu_trio(cs, x, w, b, dy, flagged=flagged)
        np.testing.assert_array_equal(a[3], c[3])
        np.testing.assert_array_equal(a[4], c[4])


# ---------------------------------------------------------------- CRBM CD-1

def run_crbm_gpu(w3, lr, h0_sample_in=None):
    cs = w3.conv
    W, b, c = dev(w3.W), dev(w3.b), dev(w3.c)
    hs = (cs.N, cs.K, cs.Ho, cs.Wo)
    out = dict(dW=torch.empty(cs.w_shape, device="cuda"), db=torch.empty(cs.K, device="cuda"),
               dc=torch.empty(cs.C, device="cuda"), h0_prob=torch.empty(hs, device="cuda"),
               h0_sample=torch.empty(hs, device="cuda"), v1=torch.empty(cs.x_shape, device="cuda"),
               h1_prob=torch.empty(hs, device="cuda"), recon_mse=torch.empty(1, device="cuda"))
    ws = B.workspace(B.dll_crbm_workspace_bytes(cs))
    B.dll_crbm_cd1_step(cs, dev(w3.v0), W, b, c, dev(w3.u), None if h0_sample_in is None else dev(h0_sample_in),
                        lr, ws=ws, **out)
    res = {k: host(v) for k, v in out.items()}
    res.update(W=host(W), b=host(b), c=host(c))
    return res


@pytest.mark.parametrize("batch", [5, 64])
def test_config3_crbm_cd1(batch):
    w3 = wl.config3(batch)
    cs = w3.conv
    g = run_crbm_gpu(w3, w3.lr)
    d = odesc(cs)
    # (i) hidden probabilities; (ii) sample flips only where u is within rounding of p
    free = orc.crbm_cd1_step(d, w3.v0, w3.W.copy(), w3.b.copy(), w3.c.copy(), w3.u)
    assert max_rel_err(g["h0_prob"], free.h0_prob) <= TOL_FWD
    flips = g["h0_sample"] != free.h0_sample
    assert flips.sum() <= max(2, 1e-5 * flips.size)
    assert np.all(np.abs(w3.u[flips] - free.h0_prob[flips]) <= 1e-6)
    assert set(np.unique(g["h0_sample"])) <= {0.0, 1.0}
    # (iii) everything downstream against the oracle driven by the GPU's samples
    Wn, bn, cn = w3.W.copy(), w3.b.copy(), w3.c.copy()
    o = orc.crbm_cd1_step(d, w3.v0, Wn, bn, cn, None, h0_sample_in=g["h0_sample"], lr=w3.lr)
    assert max_rel_err(g["v1"], o.v1) <= TOL_FWD
    assert max_rel_err(g["h1_prob"], o.h1_prob) <= TOL_FWD
    assert max_rel_err(g["recon_mse"], np.array([o.recon_mse], np.float32)) <= TOL_FWD
    assert max_rel_err(g["dW"], o.dW) <= TOL_GRAD
    assert max_rel_err(g["db"], o.db) <= TOL_GRAD
    assert max_rel_err(g["dc"], o.dc) <= TOL_GRAD
    assert max_rel_err(g["W"] - w3.W, Wn - w3.W) <= TOL_GRAD
    assert max_rel_err(g["b"] - w3.b, bn - w3.b) <= TOL_GRAD
    assert max_rel_err(g["c"] - w3.c, cn - w3.c) <= TOL_GRAD


def test_crbm_sample_override_and_lr_zero():
    w3 = wl.config3(3)
    r = np.random.default_rng(9)
    forced = (r.random((3, 40, 20, 20)) < 0.5).astype(np.float32)
    g = run_crbm_gpu(w3, 0.0, h0_sample_in=forced)
    np.testing.assert_array_equal(g["h0_sample"], forced)
    np.testing.assert_array_equal(g["W"], w3.W)       # lr = 0: parameters untouched
    o = orc.crbm_cd1_step(odesc(w3.conv), w3.v0, w3.W.copy(), w3.b.copy(), w3.c.copy(), None, h0_sample_in=forced)
    assert max_rel_err(g["v1"], o.v1) <= TOL_FWD
    assert max_rel_err(g["dW"], o.dW) <= TOL_GRAD


# ---------------------------------------------------------------- CNN training step

def run_cnn_gpu(w: wl.CnnWorkload, lr, want_grads=True):
    net = B.net_desc(w.conv, w.dense, w.classes, 0 if w.conv else w.batch)
    params = [dev(p) for p in w.params]
    grads = [torch.full_like(p, float("nan")) for p in params] if want_grads else None
    idx = [torch.full(c.y_shape, 255, dtype=torch.uint8, device="cuda") for c in w.conv]
    loss = torch.full((1,), float("nan"), device="cuda")
    logits = torch.full((w.batch, w.classes), float("nan"), device="cuda")
    ws = B.workspace(B.dll_cnn_workspace_bytes(net))
    B.dll_cnn_train_step(net, params, grads, dev(w.x), dev(w.labels), lr, loss, logits, idx, ws)
    # idx: window positions (bits 0-1 of the bytes); raw_idx: the bytes as written
    return dict(loss=host(loss)[0], logits=host(logits), grads=[host(g) for g in grads] if grads else None,
                idx=[host(i) & 3 for i in idx], raw_idx=[host(i) for i in idx], params=[host(p) for p in params])


def gpu_layer_outputs(w: wl.CnnWorkload, upto: int):
    """Outputs of the conv layers 0..upto, one forward call of the library per layer (the calls the
    training step makes, on the same kernels)."""
    a, outs = dev(w.x), []
    for l, c in enumerate(w.conv[:upto + 1]):
        y = torch.empty(c.y_shape, device="cuda")
        idx = torch.empty(c.y_shape, dtype=torch.uint8, device="cuda") if c.pool == 2 else None
        B.dll_conv_valid_fwd(c, a, dev(w.params[2 * l]), dev(w.params[2 * l + 1]), y, idx)
        outs.append(y)
        a = y
    return [host(y) for y in outs]


def check_cnn(w: wl.CnnWorkload):
    """One training step against the oracle.  The integer decisions the GPU took from its own fp32
    values (window positions, and which ReLU units are on) are first checked against the
    oracle's, layer by layer: they may differ only at (near) ties and inside a rounding band
    around zero; then the oracle's backward pass is run on the GPU's decisions and every float
    tensor is compared."""
    g = run_cnn_gpu(w, w.lr)
    net = onet(w)
    unpooled_relu = [l for l, c in enumerate(w.conv) if c.act == "relu" and c.pool == 1]
    y_gpu = gpu_layer_outputs(w, max(unpooled_relu)) if unpooled_relu else []
    # the oracle's own forward, layer by layer, to judge the decisions
    a = w.x
    active = []
    for l, c in enumerate(w.conv):
        pre = None
        if c.pool == 2:
            pre, _ = orc.conv_valid_fwd(odesc(c, pool=1), a, w.params[2 * l], w.params[2 * l + 1])
        a, idx_o = orc.conv_valid_fwd(odesc(c), a, w.params[2 * l], w.params[2 * l + 1])
        rec = None
        if c.pool == 2:
            check_pool_idx(g["idx"][l], idx_o, pre, a)
            check_idx_flags_against(g["raw_idx"][l], c.act == "relu", a)
            if c.act == "relu":
                rec = (g["raw_idx"][l] & 4) == 0
                check_relu_activity(rec, a)
        elif c.act == "relu":
            rec = y_gpu[l] > 0
            check_relu_activity(rec, a)
        active.append(None if rec is None else rec.astype(np.uint8))
        del pre
    new = w.clone_params()
    o = orc.cnn_train_step(net, new, w.x, w.labels, w.lr, pool_idx_in=g["idx"], active_in=active)
    assert max_rel_err(np.array([g["loss"]]), np.array([o.loss])) <= TOL_FWD
    assert max_rel_err(g["logits"], o.logits) <= TOL_FWD
    for p, (gg, og) in enumerate(zip(g["grads"], o.grads)):
        assert max_rel_err(gg, og) <= TOL_GRAD, f"gradient of parameter {p}"
    for p, (gp, op, old) in enumerate(zip(g["params"], new, w.params)):
        assert max_rel_err(gp - old, op - old) <= TOL_GRAD, f"update of parameter {p}"
    return g, o


def test_config2_small_cnn_step():
    check_cnn(wl.config2())


def test_config4_color_cnn_step():
    check_cnn(wl.config4())


def test_config5_architecture_reduced_size():
    """Config 5's architecture at a size the oracle finishes in seconds (64x64 images)."""
    check_cnn(wl.config5(batch=6, image=64, hidden=256, classes=100))


@pytest.mark.timeout(900)
def test_config5_full_size_step():
    """Config 5 exactly as bench.py runs it (batch 128, 3x256x256, dense 2048/1000): the same checks
    as at the reduced size.  Every pooling byte of every layer (33.5 M windows in the first) is
    compared with the oracle's position, a difference being allowed only where the oracle's own
    pre-pool values of the two candidates are (nearly) tied; the activity flags are checked against
    the oracle's output; every float tensor is compared on the GPU's decisions."""
    check_cnn(wl.config5())


def test_cnn_step_layers_that_share_launches():
    """Three padded 3x3 ReLU + pooling layers with 16 -> 16, 16 -> 32 and 32 -> 32 channels: in the
    training step each layer's filter gradient and backward-data pass run as ONE launch (half of
    the workgroups each, the filter gradient with half as many partial blocks as on its own).
    Batch and map sizes give each role a multiple of eight workgroups and several work items per
    workgroup in the first layer."""
    conv = [ConvSpec(24, 16, 64, 128, 16, 3, 3, 1, "relu", 2), ConvSpec(24, 16, 32, 64, 32, 3, 3, 1, "relu", 2),
            ConvSpec(24, 32, 16, 32, 32, 3, 3, 1, "relu", 2)]
    dense = [wl.DenseSpec(32 * 8 * 16, 96, "relu"), wl.DenseSpec(96, 10, "identity")]
    check_cnn(wl._cnn(77, "shared_launch_layers", conv, dense, 10, 0.01, "normal", None))


def test_cnn_step_with_unpooled_and_mixed_layers():
    """Layers without pooling inside a network (sigmoid and identity activations, a 1x1 and a 2x2
    filter, three dense layers): the step's backward passes then read the layer outputs instead
    of pooling bytes."""
    conv = [ConvSpec(5, 3, 20, 24, 8, 3, 3, 1, "relu", 2), ConvSpec(5, 8, 10, 12, 12, 2, 2, 0, "sigmoid", 1),
            ConvSpec(5, 12, 9, 11, 6, 1, 1, 0, "identity", 1), ConvSpec(5, 6, 9, 11, 16, 3, 3, 0, "relu", 1)]
    dense = [DenseSpec(16 * 7 * 9, 64, "sigmoid"), DenseSpec(64, 33, "relu"), DenseSpec(33, 7, "identity")]
    w = wl._cnn(21, "mixed_layers", conv, dense, 7, 0.05, "normal", None)
    check_cnn(w)
    check_forward(w)


def test_step_captured_in_a_hip_graph_replays_bit_identically():
    """The library allocates nothing and synchronises nothing, so a whole training step can be
    captured into a HIP graph (what `bench.py` times by default).  Three replays, with unrelated
    plain launches and synchronisations between them, must leave exactly the parameters, loss and
    logits that three plain steps leave: the kernels are deterministic."""
    w = wl.config5(batch=4, image=64, hidden=128, classes=50)
    net = B.net_desc(w.conv, w.dense, w.classes)
    x, labels = dev(w.x), dev(w.labels)
    ws = B.workspace(B.dll_cnn_workspace_bytes(net))

    def fresh():
        return ([dev(p) for p in w.params], torch.full((1,), float("nan"), device="cuda"),
                torch.full((w.batch, w.classes), float("nan"), device="cuda"))

    pe, le, ge = fresh()
    snaps = []
    for _ in range(3):
        B.dll_cnn_train_step(net, pe, None, x, labels, 0.05, le, ge, None, ws)
        snaps.append(([host(p) for p in pe], host(le).copy(), host(ge).copy()))
    pg, lg, gg = fresh()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        B.dll_cnn_train_step(net, pg, None, x, labels, 0.05, lg, gg, None, ws)
    torch.cuda.synchronize()
    for a, b in zip(pg, w.params):                      # capturing runs nothing
        np.testing.assert_array_equal(host(a), b)
    other = ConvSpec(2, 3, 12, 10, 5, 3, 3, 1, "relu", 2)
    ox, ow, ob, _ = rand_layer(other, 77)
    for r in range(3):
        graph.replay()
        torch.cuda.synchronize()
        params, loss, logits = snaps[r]
        for p, (a, b) in enumerate(zip(pg, params)):
            assert np.array_equal(host(a), b), f"replay {r}: parameter {p}"
        assert np.array_equal(host(lg), loss) and np.array_equal(host(gg), logits), f"replay {r}"
        # the program's own work between replays: another layer through the plain entry point
        oy = torch.empty(other.y_shape, device="cuda")
        B.dll_conv_valid_fwd(other, dev(ox), dev(ow), dev(ob), oy, torch.empty(other.y_shape, dtype=torch.uint8, device="cuda"))
        torch.cuda.synchronize()


def test_cnn_lr_zero_and_no_grads():
    w = wl.config2(batch=10)
    g = run_cnn_gpu(w, 0.0, want_grads=False)
    for a, b in zip(g["params"], w.params):
        np.testing.assert_array_equal(a, b)
    o = orc.cnn_train_step(onet(w), w.clone_params(), w.x, w.labels, 0.0)
    assert max_rel_err(np.array([g["loss"]]), np.array([o.loss])) <= TOL_FWD


# ---------------------------------------------------------------- inference pass

def run_forward_gpu(w: wl.CnnWorkload):
    net = B.net_desc(w.conv, w.dense, w.classes, 0 if w.conv else w.batch)
    params = [dev(p) for p in w.params]
    logits = torch.full((w.batch, w.classes), float("nan"), device="cuda")
    prob = torch.full((w.batch, w.classes), float("nan"), device="cuda")
    ws = B.workspace(B.dll_cnn_forward_workspace_bytes(net))
    B.dll_cnn_forward(net, params, dev(w.x), logits, prob, ws)
    return host(logits), host(prob)


def check_forward(w: wl.CnnWorkload):
    lg, pg = run_forward_gpu(w)
    lo, po = orc.cnn_forward(onet(w), w.params, w.x)
    assert max_rel_err(lg, lo) <= TOL_FWD
    assert max_rel_err(pg, po) <= TOL_FWD
    np.testing.assert_allclose(pg.sum(1), 1.0, rtol=1e-5)


@pytest.mark.parametrize("make", [lambda: wl.paper_mnist_cnn(37), lambda: wl.paper_cifar_cnn(21),
                                  lambda: wl.paper_imagenet_cnn(5, 64, 96, 40),
                                  lambda: wl.config5(batch=3, image=64, hidden=128, classes=50)],
                         ids=["paper_mnist_cnn", "paper_cifar_cnn", "paper_imagenet_cnn_64px", "config5_64px"])
def test_forward_pass_matches_oracle(make):
    """Inference pass of the networks as the paper describes them (full layer shapes for the MNIST
    and CIFAR nets, the ImageNet architecture at 64x64) against the oracle's inference pass."""
    check_forward(make())


def test_forward_pass_full_size_sampled_images():
    """Section VI's network at its full shape (batch 128, 3x256x256, five blocks, dense 2048, dense
    1000), the launch configuration of `bench.py --mode infer`.  An image's logits depend on that
    image alone, so the oracle runs the same network on a sample of the batch (first, last, two in
    between) and those rows are compared one by one."""
    w = wl.paper_imagenet_cnn()
    lg, pg = run_forward_gpu(w)
    rows = [0, 45, 86, w.batch - 1]
    sub = wl.paper_imagenet_cnn(len(rows))
    lo, po = orc.cnn_forward(onet(sub), w.params, np.ascontiguousarray(w.x[rows]))
    assert max_rel_err(lg[rows], lo) <= TOL_FWD
    assert max_rel_err(pg[rows], po) <= TOL_FWD
    assert np.isfinite(lg).all()
    np.testing.assert_allclose(pg.sum(1), 1.0, rtol=1e-5)


def test_forward_pass_logits_equal_training_pass_logits():
    """Same kernels, same order of operations: the inference pass and the training step's forward
    half give bit-identical logits; logits-only and probabilities-only calls work."""
    w = wl.config5(batch=4, image=64, hidden=128, classes=50)
    g = run_cnn_gpu(w, 0.0, want_grads=False)
    lg, pg = run_forward_gpu(w)
    assert np.array_equal(lg, g["logits"])
    net = B.net_desc(w.conv, w.dense, w.classes, 0 if w.conv else w.batch)
    params = [dev(p) for p in w.params]
    ws = B.workspace(B.dll_cnn_forward_workspace_bytes(net))
    only_p = torch.full((w.batch, w.classes), float("nan"), device="cuda")
    B.dll_cnn_forward(net, params, dev(w.x), None, only_p, ws)
    assert np.array_equal(host(only_p), pg)
    with pytest.raises(B.DllError):
        B.dll_cnn_forward(net, params, dev(w.x), None, None, ws)


# ---------------------------------------------------------------- momentum and weight decay

def test_momentum_step_matches_oracle():
    """One step with momentum 0.9, weight decay 1e-3 and a non-zero velocity: gradients, new
    velocities and parameter changes against the oracle's gradients fed through its own
    momentum update (decay on weights only).  Zero momentum/decay/velocity equals the plain step."""
    w = wl.config5(batch=6, image=64, hidden=256, classes=100)
    lr, mu, decay = 0.01, 0.9, 1e-3
    r = np.random.default_rng(77)
    vel0 = [(r.standard_normal(p.shape) * 0.01 * max(float(np.abs(p).max()), 1e-3)).astype(np.float32) for p in w.params]
    net = B.net_desc(w.conv, w.dense, w.classes, 0 if w.conv else w.batch)
    params, vel = [dev(p) for p in w.params], [dev(v) for v in vel0]
    grads = [torch.full_like(p, float("nan")) for p in params]
    idx = [torch.full(c.y_shape, 255, dtype=torch.uint8, device="cuda") for c in w.conv]
    loss = torch.full((1,), float("nan"), device="cuda")
    ws = B.workspace(B.dll_cnn_workspace_bytes(net))
    B.dll_cnn_train_step_momentum(net, params, vel, grads, dev(w.x), dev(w.labels), lr, mu, decay, loss, None, idx, ws)
    o = orc.cnn_train_step(onet(w), w.clone_params(), w.x, w.labels, 0.0, pool_idx_in=[host(i) & 3 for i in idx],
                           active_in=[((host(i) & 4) == 0).astype(np.uint8) for i in idx])
    assert max_rel_err(np.array([host(loss)[0]]), np.array([o.loss])) <= TOL_FWD
    for p, (old, v0, og) in enumerate(zip(w.params, vel0, o.grads)):
        th, v = old.copy(), v0.copy()
        orc.sgd_momentum(th, v, og, lr, mu, decay if p % 2 == 0 else 0.0)
        assert max_rel_err(host(grads[p]), og) <= TOL_GRAD, f"gradient of parameter {p}"
        assert max_rel_err(host(vel[p]), v) <= TOL_GRAD, f"velocity of parameter {p}"
        assert max_rel_err(host(params[p]) - old, th - old) <= TOL_GRAD, f"update of parameter {p}"
    # momentum 0, decay 0, zero velocity: the plain step up to the rounding of one product (the plain
    # update is a single fused multiply-add, the momentum form rounds the velocity first)
    pa, pb = [dev(p) for p in w.params], [dev(p) for p in w.params]
    vz = [torch.zeros_like(p) for p in pa]
    B.dll_cnn_train_step_momentum(net, pa, vz, None, dev(w.x), dev(w.labels), lr, 0.0, 0.0, loss, None, None, ws)
    B.dll_cnn_train_step(net, pb, None, dev(w.x), dev(w.labels), lr, loss, None, None, ws)
    for a_, b_ in zip(pa, pb):
        assert max_rel_err(host(a_), host(b_)) <= 2e-7   # one ulp of the parameter itself
