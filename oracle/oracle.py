"""ctypes front end of the CPU oracle (TEST INFRASTRUCTURE ONLY).

Marshals numpy arrays into `libdll_oracle.so`; holds no arithmetic of the method.
Only tests, the smoke check and the bench's cpu_baseline leg may import this module;
it shares nothing with, and never imports, the GPU package.

The `f64=True` variants call the fp64-storage instantiation of the same C source and
exist for finite-difference pins.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# DLL_ORACLE_LIB points the tests at another build of the same source (the sanitizer build)
_LIB_PATH = os.environ.get("DLL_ORACLE_LIB") or os.path.join(_HERE, "libdll_oracle.so")

ACT_IDENTITY, ACT_SIGMOID, ACT_RELU = 0, 1, 2


def build(force: bool = True) -> str:
    """Compile the oracle with gcc (-O2 -fopenmp).  Returns the library path."""
    if force or not os.path.exists(_LIB_PATH):
        cmd = ["gcc", "-O2", "-fopenmp", "-Wall", "-Wextra", "-shared", "-fPIC",
               os.path.join(_HERE, "dll_oracle.c"), "-o", _LIB_PATH, "-lm"]
        subprocess.run(cmd, check=True, cwd=_HERE)
    return _LIB_PATH


def build_sanitized(out_path: str) -> str:
    """The same source with AddressSanitizer and UndefinedBehaviorSanitizer (host code only).  Run
    the CPU tests on it with
      LD_PRELOAD=$(gcc -print-file-name=libasan.so) ASAN_OPTIONS=detect_leaks=0 \
      UBSAN_OPTIONS=halt_on_error=1 DLL_ORACLE_LIB=<out_path> python -m pytest tests -m 'not gpu'
    """
    cmd = ["gcc", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
           "-fopenmp", "-Wall", "-Wextra", "-shared", "-fPIC", os.path.join(_HERE, "dll_oracle.c"), "-o", out_path, "-lm"]
    subprocess.run(cmd, check=True, cwd=_HERE)
    return out_path


class ConvDesc(C.Structure):
    _fields_ = [(n, C.c_int) for n in ("N", "C", "H", "W", "K", "R", "S", "pad", "act", "pool")]

    @property
    def Ho(self):
        return self.H + 2 * self.pad - self.R + 1

    @property
    def Wo(self):
        return self.W + 2 * self.pad - self.S + 1

    @property
    def out_shape(self):
        return (self.N, self.K, self.Ho // self.pool, self.Wo // self.pool)


class DenseDesc(C.Structure):
    _fields_ = [("in_", C.c_int), ("out", C.c_int), ("act", C.c_int)]


class NetDesc(C.Structure):
    _fields_ = [("n_conv", C.c_int), ("conv", C.POINTER(ConvDesc)), ("n_dense", C.c_int),
                ("dense", C.POINTER(DenseDesc)), ("classes", C.c_int), ("batch", C.c_int)]


def conv_desc(N, C_, H, W, K, R, S, pad=0, act=ACT_IDENTITY, pool=1) -> ConvDesc:
    return ConvDesc(N, C_, H, W, K, R, S, pad, act, pool)


_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            build()
        _lib = C.CDLL(_LIB_PATH)
        _lib.oracle_max_threads.restype = C.c_int
        _lib.oracle_set_threads.argtypes = [C.c_int]
    return _lib


def max_threads() -> int:
    return int(lib().oracle_max_threads())


def set_threads(n: int) -> None:
    lib().oracle_set_threads(int(n))


def _dt(f64):
    return np.float64 if f64 else np.float32


def _pfx(f64):
    return "oracle64_" if f64 else "oracle_"


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _arr(a, f64):
    return None if a is None else np.ascontiguousarray(a, dtype=_dt(f64))


def _check(rc, name):
    if rc != 0:
        raise ValueError(f"oracle {name} rejected its arguments (rc={rc})")


def conv_valid_fwd(d: ConvDesc, x, w, bias=None, f64=False):
    """Returns (y, pool_idx or None)."""
    x, w, bias = _arr(x, f64), _arr(w, f64), _arr(bias, f64)
    assert x.shape == (d.N, d.C, d.H, d.W) and w.shape == (d.K, d.C, d.R, d.S)
    y = np.empty(d.out_shape, dtype=_dt(f64))
    idx = np.empty(d.out_shape, dtype=np.uint8) if d.pool == 2 else None
    fn = getattr(lib(), _pfx(f64) + "conv_valid_fwd")
    fn.argtypes = [C.POINTER(ConvDesc)] + [C.c_void_p] * 5
    _check(fn(C.byref(d), _p(x), _p(w), _p(bias), _p(y), _p(idx)), "conv_valid_fwd")
    return y, idx


def conv_full_bwd(d: ConvDesc, dy, y, pool_idx, w, f64=False):
    dy, y, w = _arr(dy, f64), _arr(y, f64), _arr(w, f64)
    assert dy.shape == d.out_shape
    if pool_idx is not None:
        pool_idx = np.ascontiguousarray(pool_idx, dtype=np.uint8)
    dx = np.empty((d.N, d.C, d.H, d.W), dtype=_dt(f64))
    fn = getattr(lib(), _pfx(f64) + "conv_full_bwd")
    fn.argtypes = [C.POINTER(ConvDesc)] + [C.c_void_p] * 5
    _check(fn(C.byref(d), _p(dy), _p(y), _p(pool_idx), _p(w), _p(dx)), "conv_full_bwd")
    return dx


def conv_valid_wgrad(d: ConvDesc, x, dy, y, pool_idx, f64=False):
    """Returns (dw, db)."""
    x, dy, y = _arr(x, f64), _arr(dy, f64), _arr(y, f64)
    assert dy.shape == d.out_shape and x.shape == (d.N, d.C, d.H, d.W)
    if pool_idx is not None:
        pool_idx = np.ascontiguousarray(pool_idx, dtype=np.uint8)
    dw = np.empty((d.K, d.C, d.R, d.S), dtype=_dt(f64))
    db = np.empty((d.K,), dtype=_dt(f64))
    fn = getattr(lib(), _pfx(f64) + "conv_valid_wgrad")
    fn.argtypes = [C.POINTER(ConvDesc)] + [C.c_void_p] * 6
    _check(fn(C.byref(d), _p(x), _p(dy), _p(y), _p(pool_idx), _p(dw), _p(db)), "conv_valid_wgrad")
    return dw, db


def dense_fwd(a, W, b, act, f64=False):
    a, W, b = _arr(a, f64), _arr(W, f64), _arr(b, f64)
    B, in_ = a.shape
    out = W.shape[0]
    assert W.shape == (out, in_)
    h = np.empty((B, out), dtype=_dt(f64))
    fn = getattr(lib(), _pfx(f64) + "dense_fwd")
    fn.argtypes = [C.c_int] * 4 + [C.c_void_p] * 4
    _check(fn(B, in_, out, act, _p(a), _p(W), _p(b), _p(h)), "dense_fwd")
    return h


def dense_bwd(a, W, h, dh, act, f64=False):
    """Returns (da, dW, db)."""
    a, W, h, dh = _arr(a, f64), _arr(W, f64), _arr(h, f64), _arr(dh, f64)
    B, in_ = a.shape
    out = W.shape[0]
    da = np.empty((B, in_), dtype=_dt(f64))
    dW = np.empty((out, in_), dtype=_dt(f64))
    db = np.empty((out,), dtype=_dt(f64))
    fn = getattr(lib(), _pfx(f64) + "dense_bwd")
    fn.argtypes = [C.c_int] * 4 + [C.c_void_p] * 7
    _check(fn(B, in_, out, act, _p(a), _p(W), _p(h), _p(dh), _p(da), _p(dW), _p(db)), "dense_bwd")
    return da, dW, db


def softmax_ce(logits, labels, f64=False):
    """Returns (loss, prob, dlogits)."""
    logits = _arr(logits, f64)
    labels = np.ascontiguousarray(labels, dtype=np.int32)
    B, classes = logits.shape
    loss = np.empty((1,), dtype=_dt(f64))
    prob = np.empty_like(logits)
    dl = np.empty_like(logits)
    fn = getattr(lib(), _pfx(f64) + "softmax_ce")
    fn.argtypes = [C.c_int, C.c_int] + [C.c_void_p] * 5
    _check(fn(B, classes, _p(logits), _p(labels), _p(loss), _p(prob), _p(dl)), "softmax_ce")
    return loss[0], prob, dl


def sgd(theta, g, lr, f64=False):
    """In place on a contiguous array of the storage dtype; returns it."""
    assert theta.dtype == _dt(f64) and theta.flags.c_contiguous
    g = _arr(g, f64)
    fn = getattr(lib(), _pfx(f64) + "sgd")
    fn.argtypes = [C.c_long, C.c_void_p, C.c_void_p, C.c_double if f64 else C.c_float]
    _check(fn(theta.size, _p(theta), _p(g), lr), "sgd")
    return theta


def sgd_momentum(theta, vel, g, lr, mu, decay, f64=False):
    """In place on contiguous arrays of the storage dtype: v <- mu v - lr (g + decay theta); theta <- theta + v."""
    assert theta.dtype == _dt(f64) and theta.flags.c_contiguous and vel.dtype == _dt(f64) and vel.flags.c_contiguous
    g = _arr(g, f64)
    fn = getattr(lib(), _pfx(f64) + "sgd_momentum")
    real = C.c_double if f64 else C.c_float
    fn.argtypes = [C.c_long, C.c_void_p, C.c_void_p, C.c_void_p, real, real, real]
    _check(fn(theta.size, _p(theta), _p(vel), _p(g), lr, mu, decay), "sgd_momentum")
    return theta, vel


@dataclass
class CrbmResult:
    dW: np.ndarray
    db: np.ndarray
    dc: np.ndarray
    h0_prob: np.ndarray
    h0_sample: np.ndarray
    v1: np.ndarray
    h1_prob: np.ndarray
    recon_mse: float
    pool_prob: Optional[np.ndarray] = None


VIS_BINARY, VIS_GAUSSIAN = 0, 1


def crbm_cd1_step_units(d: ConvDesc, visible, hidden_pool, v0, W, b_hid, c_vis, uniform=None,
                        h0_sample_in=None, lr=0.0, f64=False) -> CrbmResult:
    """CD-1 step with a choice of visible unit (VIS_*) and of hidden layer (hidden_pool 1:
    independent units; 2: probabilistic max pooling, uniform is then one number per 2x2 block).
    W, b_hid, c_vis are updated IN PLACE when lr != 0 (pass arrays of the storage dtype)."""
    dt = _dt(f64)
    for t in (W, b_hid, c_vis):
        assert t.dtype == dt and t.flags.c_contiguous
    v0, uniform, h0_sample_in = _arr(v0, f64), _arr(uniform, f64), _arr(h0_sample_in, f64)
    hs = (d.N, d.K, d.Ho, d.Wo)
    if uniform is not None:
        assert uniform.shape == (hs if hidden_pool == 1 else (d.N, d.K, d.Ho // 2, d.Wo // 2))
    res = CrbmResult(np.empty(W.shape, dt), np.empty((d.K,), dt), np.empty((d.C,), dt),
                     np.empty(hs, dt), np.empty(hs, dt), np.empty(v0.shape, dt), np.empty(hs, dt), 0.0)
    if hidden_pool == 2:
        res.pool_prob = np.empty((d.N, d.K, d.Ho // 2, d.Wo // 2), dt)
    mse = np.empty((1,), dt)
    fn = getattr(lib(), _pfx(f64) + "crbm_cd1_step_units")
    real = C.c_double if f64 else C.c_float
    fn.argtypes = [C.POINTER(ConvDesc), C.c_int, C.c_int] + [C.c_void_p] * 6 + [real] + [C.c_void_p] * 9
    _check(fn(C.byref(d), visible, hidden_pool, _p(v0), _p(W), _p(b_hid), _p(c_vis), _p(uniform),
              _p(h0_sample_in), lr, _p(res.dW), _p(res.db), _p(res.dc), _p(res.h0_prob),
              _p(res.h0_sample), _p(res.pool_prob), _p(res.v1), _p(res.h1_prob), _p(mse)),
           "crbm_cd1_step_units")
    res.recon_mse = float(mse[0])
    return res


def rbm_cd1_step(B, nv, nh, visible, v0, W, b_hid, c_vis, uniform=None, h0_sample_in=None, lr=0.0,
                 f64=False) -> CrbmResult:
    """CD-1 step of a fully-connected RBM: v0 [B, nv], W [nh, nv], uniform [B, nh].
    W, b_hid, c_vis are updated IN PLACE when lr != 0."""
    dt = _dt(f64)
    for t in (W, b_hid, c_vis):
        assert t.dtype == dt and t.flags.c_contiguous
    v0, uniform, h0_sample_in = _arr(v0, f64), _arr(uniform, f64), _arr(h0_sample_in, f64)
    assert v0.shape == (B, nv) and W.shape == (nh, nv) and b_hid.shape == (nh,) and c_vis.shape == (nv,)
    res = CrbmResult(np.empty((nh, nv), dt), np.empty((nh,), dt), np.empty((nv,), dt),
                     np.empty((B, nh), dt), np.empty((B, nh), dt), np.empty((B, nv), dt),
                     np.empty((B, nh), dt), 0.0)
    mse = np.empty((1,), dt)
    fn = getattr(lib(), _pfx(f64) + "rbm_cd1_step")
    real = C.c_double if f64 else C.c_float
    fn.argtypes = [C.c_int] * 4 + [C.c_void_p] * 6 + [real] + [C.c_void_p] * 8
    _check(fn(B, nv, nh, visible, _p(v0), _p(W), _p(b_hid), _p(c_vis), _p(uniform), _p(h0_sample_in),
              lr, _p(res.dW), _p(res.db), _p(res.dc), _p(res.h0_prob), _p(res.h0_sample), _p(res.v1),
              _p(res.h1_prob), _p(mse)), "rbm_cd1_step")
    res.recon_mse = float(mse[0])
    return res


def crbm_cd1_step(d: ConvDesc, v0, W, b_hid, c_vis, uniform=None, h0_sample_in=None, lr=0.0,
                  f64=False) -> CrbmResult:
    """W, b_hid, c_vis are updated IN PLACE when lr != 0 (pass arrays of the storage dtype)."""
    dt = _dt(f64)
    for t in (W, b_hid, c_vis):
        assert t.dtype == dt and t.flags.c_contiguous
    v0, uniform, h0_sample_in = _arr(v0, f64), _arr(uniform, f64), _arr(h0_sample_in, f64)
    hs = (d.N, d.K, d.Ho, d.Wo)
    res = CrbmResult(np.empty(W.shape, dt), np.empty((d.K,), dt), np.empty((d.C,), dt),
                     np.empty(hs, dt), np.empty(hs, dt), np.empty(v0.shape, dt), np.empty(hs, dt), 0.0)
    mse = np.empty((1,), dt)
    fn = getattr(lib(), _pfx(f64) + "crbm_cd1_step")
    real = C.c_double if f64 else C.c_float
    fn.argtypes = [C.POINTER(ConvDesc)] + [C.c_void_p] * 6 + [real] + [C.c_void_p] * 8
    _check(fn(C.byref(d), _p(v0), _p(W), _p(b_hid), _p(c_vis), _p(uniform), _p(h0_sample_in), lr,
              _p(res.dW), _p(res.db), _p(res.dc), _p(res.h0_prob), _p(res.h0_sample), _p(res.v1),
              _p(res.h1_prob), _p(mse)), "crbm_cd1_step")
    res.recon_mse = float(mse[0])
    return res


@dataclass
class Net:
    """A CNN: conv descriptors, then (in, out, act) dense layers, the last one feeding softmax-CE.
    With no conv descriptors it is a fully-connected network on [batch, in] inputs."""
    conv: Sequence[ConvDesc]
    dense: Sequence[tuple]
    classes: int
    batch: int = 0

    @property
    def B(self):
        return self.conv[0].N if len(self.conv) else self.batch

    def param_shapes(self):
        shapes = []
        for d in self.conv:
            shapes += [(d.K, d.C, d.R, d.S), (d.K,)]
        for (i, o, _a) in self.dense:
            shapes += [(o, i), (o,)]
        return shapes


@dataclass
class CnnResult:
    loss: float
    logits: np.ndarray
    grads: list
    pool_idx: list


def cnn_train_step(net: Net, params, x, labels, lr=0.0, pool_idx_in=None, f64=False, active_in=None) -> CnnResult:
    """params: list of arrays (storage dtype, contiguous), updated IN PLACE when lr != 0.
    pool_idx_in / active_in: per conv layer (entries may be None) the pooling positions and, for
    ReLU layers, the activity record (non-zero = unit active) to use in the backward pass instead
    of the oracle's own decisions."""
    dt = _dt(f64)
    shapes = net.param_shapes()
    assert len(params) == len(shapes)
    for p, s in zip(params, shapes):
        assert p.dtype == dt and p.flags.c_contiguous and tuple(p.shape) == tuple(s), (p.shape, s)
    L = len(net.conv)
    convs = (ConvDesc * L)(*net.conv)
    denses = (DenseDesc * len(net.dense))(*[DenseDesc(i, o, a) for (i, o, a) in net.dense])
    nd = NetDesc(L, convs, len(net.dense), denses, net.classes, net.batch)
    x = _arr(x, f64)
    labels = np.ascontiguousarray(labels, dtype=np.int32)
    B = net.B
    grads = [np.empty(s, dt) for s in shapes]
    idx_out = [np.zeros(d.out_shape, np.uint8) for d in net.conv]
    logits = np.empty((B, net.classes), dt)
    loss = np.empty((1,), dt)
    PP = C.c_void_p * len(shapes)
    pp = PP(*[p.ctypes.data for p in params])
    gg = PP(*[g.ctypes.data for g in grads])
    IP = C.c_void_p * L
    io = IP(*[i.ctypes.data for i in idx_out])
    ii = None
    keep = []
    if pool_idx_in is not None:
        keep = [None if i is None else np.ascontiguousarray(i, np.uint8) for i in pool_idx_in]
        ii = IP(*[None if i is None else i.ctypes.data for i in keep])
    aa = None
    keep_a = []
    if active_in is not None:
        keep_a = [None if a is None else np.ascontiguousarray(a, np.uint8) for a in active_in]
        for a, d in zip(keep_a, net.conv):
            assert a is None or a.shape == tuple(d.out_shape), (a.shape, d.out_shape)
        aa = IP(*[None if a is None else a.ctypes.data for a in keep_a])
    fn = getattr(lib(), _pfx(f64) + "cnn_train_step")
    real = C.c_double if f64 else C.c_float
    fn.argtypes = [C.POINTER(NetDesc), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, real,
                   C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    _check(fn(C.byref(nd), pp, gg, _p(x), _p(labels), lr, _p(loss), _p(logits), ii, io, aa), "cnn_train_step")
    return CnnResult(float(loss[0]), logits, grads, idx_out)


def cnn_forward(net: Net, params, x, f64=False):
    """Inference pass: returns (logits, probabilities), both [N, classes]."""
    dt = _dt(f64)
    shapes = net.param_shapes()
    assert len(params) == len(shapes)
    for p, s in zip(params, shapes):
        assert p.dtype == dt and p.flags.c_contiguous and tuple(p.shape) == tuple(s), (p.shape, s)
    L = len(net.conv)
    convs = (ConvDesc * L)(*net.conv)
    denses = (DenseDesc * len(net.dense))(*[DenseDesc(i, o, a) for (i, o, a) in net.dense])
    nd = NetDesc(L, convs, len(net.dense), denses, net.classes, net.batch)
    x = _arr(x, f64)
    B = net.B
    logits = np.empty((B, net.classes), dt)
    prob = np.empty((B, net.classes), dt)
    PP = C.c_void_p * len(shapes)
    pp = PP(*[p.ctypes.data for p in params])
    fn = getattr(lib(), _pfx(f64) + "cnn_forward")
    fn.argtypes = [C.POINTER(NetDesc), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    _check(fn(C.byref(nd), pp, _p(x), _p(logits), _p(prob)), "cnn_forward")
    return logits, prob
