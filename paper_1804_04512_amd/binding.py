"""Thin ctypes binding of libdll_conv.so: argument marshalling only.

Every function has the name of the C entry point it calls (`include/dll_conv.h`) and
does no arithmetic of its own.  PyTorch supplies device memory and the stream.  There is
no CPU fallback: a missing library or a non-OK status raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import List, Optional, Sequence

import torch

from .workloads import ConvSpec, DenseSpec

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdll_conv.so")

ACT = {"identity": 0, "sigmoid": 1, "relu": 2}
SYMBOLS = ["dll_status_string", "dll_conv_workspace_bytes", "dll_conv_valid_fwd", "dll_conv_full_bwd",
           "dll_conv_valid_wgrad", "dll_crbm_workspace_bytes", "dll_crbm_cd1_step",
           "dll_cnn_workspace_bytes", "dll_cnn_train_step", "dll_cnn_forward_workspace_bytes", "dll_cnn_forward",
           "dll_cnn_train_step_momentum", "dll_crbm_cd1_step_units", "dll_rbm_workspace_bytes", "dll_rbm_cd1_step",
           "dll_conv_full_fft_workspace_bytes", "dll_conv_full_bwd_fft", "dll_conv_valid_wgrad_noalloc",
           "dll_conv_valid_wgrad_partial", "dll_conv_valid_wgrad_finish"]
NOALLOC_SCRATCH_BYTES = 8 << 20   # DLL_NOALLOC_SCRATCH_BYTES of include/dll_conv.h
VISIBLE = {"binary": 0, "gaussian": 1}


class DllError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib().dll_status_string(status).decode()
        super().__init__(f"{where}: {msg} (dll_status {status})")


class dll_conv_desc(C.Structure):
    _fields_ = [(n, C.c_int) for n in ("N", "C", "H", "W", "K", "R", "S", "pad", "act", "pool")]


class dll_dense_desc(C.Structure):
    _fields_ = [("in_", C.c_int), ("out", C.c_int), ("act", C.c_int)]


class dll_net_desc(C.Structure):
    _fields_ = [("n_conv", C.c_int), ("conv", C.POINTER(dll_conv_desc)), ("n_dense", C.c_int),
                ("dense", C.POINTER(dll_dense_desc)), ("classes", C.c_int), ("batch", C.c_int)]


_lib = None


def lib() -> C.CDLL:
    """Loads the HIP library; raises if it has not been built (python -m paper_1804_04512_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is missing: build it with `python -m paper_1804_04512_amd.build`")
        L = C.CDLL(LIB_PATH)
        vp, sz = C.c_void_p, C.c_size_t
        pd = C.POINTER(dll_conv_desc)
        L.dll_status_string.restype = C.c_char_p
        L.dll_status_string.argtypes = [C.c_int]
        L.dll_conv_workspace_bytes.restype = sz
        L.dll_conv_workspace_bytes.argtypes = [pd]
        L.dll_conv_valid_fwd.argtypes = [pd, vp, vp, vp, vp, vp, vp, sz, vp]
        L.dll_conv_full_bwd.argtypes = [pd, vp, vp, vp, vp, vp, vp, sz, vp]
        L.dll_conv_valid_wgrad.argtypes = [pd, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.dll_conv_valid_wgrad_noalloc.argtypes = [pd, vp, vp, vp, vp, vp, vp, vp]
        L.dll_conv_valid_wgrad_partial.argtypes = [pd, vp, vp, vp, vp, vp, sz, vp]
        L.dll_conv_valid_wgrad_finish.argtypes = [pd, vp, vp, vp, sz, vp]
        L.dll_conv_full_fft_workspace_bytes.restype = sz
        L.dll_conv_full_fft_workspace_bytes.argtypes = [pd]
        L.dll_conv_full_bwd_fft.argtypes = [pd, vp, vp, vp, vp, vp, vp, sz, vp]
        L.dll_crbm_workspace_bytes.restype = sz
        L.dll_crbm_workspace_bytes.argtypes = [pd]
        L.dll_crbm_cd1_step.argtypes = [pd, vp, vp, vp, vp, vp, vp, C.c_float] + [vp] * 8 + [vp, sz, vp]
        L.dll_crbm_cd1_step_units.argtypes = [pd, C.c_int, C.c_int, vp, vp, vp, vp, vp, vp, C.c_float] + [vp] * 9 + [vp, sz, vp]
        L.dll_rbm_workspace_bytes.restype = sz
        L.dll_rbm_workspace_bytes.argtypes = [C.c_int] * 3
        L.dll_rbm_cd1_step.argtypes = [C.c_int] * 4 + [vp, vp, vp, vp, vp, vp, C.c_float] + [vp] * 8 + [vp, sz, vp]
        L.dll_cnn_workspace_bytes.restype = sz
        L.dll_cnn_workspace_bytes.argtypes = [C.POINTER(dll_net_desc)]
        L.dll_cnn_train_step.argtypes = [C.POINTER(dll_net_desc), vp, vp, vp, vp, C.c_float, vp, vp, vp, vp, sz, vp]
        L.dll_cnn_train_step_momentum.argtypes = [C.POINTER(dll_net_desc), vp, vp, vp, vp, vp, C.c_float, C.c_float, C.c_float,
                                                  vp, vp, vp, vp, sz, vp]
        L.dll_cnn_forward_workspace_bytes.restype = sz
        L.dll_cnn_forward_workspace_bytes.argtypes = [C.POINTER(dll_net_desc)]
        L.dll_cnn_forward.argtypes = [C.POINTER(dll_net_desc), vp, vp, vp, vp, vp, sz, vp]
        _lib = L
    return _lib


def conv_desc(cs: ConvSpec) -> dll_conv_desc:
    return dll_conv_desc(cs.N, cs.C, cs.H, cs.W, cs.K, cs.R, cs.S, cs.pad, ACT[cs.act], cs.pool)


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device-resident contiguous tensors only"
    return C.c_void_p(t.data_ptr())


def _stream(stream=None):
    s = stream if stream is not None else torch.cuda.current_stream()
    return C.c_void_p(s.cuda_stream)


def _ok(status: int, where: str):
    if status != 0:
        raise DllError(status, where)


def workspace(nbytes: int, device="cuda") -> Optional[torch.Tensor]:
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def dll_conv_workspace_bytes(cs: ConvSpec) -> int:
    d = conv_desc(cs)
    return int(lib().dll_conv_workspace_bytes(C.byref(d)))


def dll_conv_valid_fwd(cs: ConvSpec, x, w, bias, y, pool_idx=None, ws=None, stream=None) -> None:
    d = conv_desc(cs)
    _ok(lib().dll_conv_valid_fwd(C.byref(d), _ptr(x), _ptr(w), _ptr(bias), _ptr(y), _ptr(pool_idx), _ptr(ws),
                                 0 if ws is None else ws.numel(), _stream(stream)), "dll_conv_valid_fwd")


def dll_conv_full_bwd(cs: ConvSpec, dy, y, pool_idx, w, dx, ws=None, stream=None) -> None:
    d = conv_desc(cs)
    _ok(lib().dll_conv_full_bwd(C.byref(d), _ptr(dy), _ptr(y), _ptr(pool_idx), _ptr(w), _ptr(dx), _ptr(ws),
                                0 if ws is None else ws.numel(), _stream(stream)), "dll_conv_full_bwd")


def dll_conv_full_fft_workspace_bytes(cs: ConvSpec) -> int:
    d = conv_desc(cs)
    return int(lib().dll_conv_full_fft_workspace_bytes(C.byref(d)))


def dll_conv_full_bwd_fft(cs: ConvSpec, dy, y, pool_idx, w, dx, ws, stream=None) -> None:
    d = conv_desc(cs)
    _ok(lib().dll_conv_full_bwd_fft(C.byref(d), _ptr(dy), _ptr(y), _ptr(pool_idx), _ptr(w), _ptr(dx), _ptr(ws),
                                    0 if ws is None else ws.numel(), _stream(stream)), "dll_conv_full_bwd_fft")


def dll_conv_valid_wgrad(cs: ConvSpec, x, dy, y, pool_idx, dw, dbias, ws, stream=None) -> None:
    d = conv_desc(cs)
    _ok(lib().dll_conv_valid_wgrad(C.byref(d), _ptr(x), _ptr(dy), _ptr(y), _ptr(pool_idx), _ptr(dw), _ptr(dbias),
                                   _ptr(ws), 0 if ws is None else ws.numel(), _stream(stream)), "dll_conv_valid_wgrad")


def dll_conv_valid_wgrad_partial(cs: ConvSpec, x, dy, y, pool_idx, ws, stream=None) -> None:
    d = conv_desc(cs)
    _ok(lib().dll_conv_valid_wgrad_partial(C.byref(d), _ptr(x), _ptr(dy), _ptr(y), _ptr(pool_idx), _ptr(ws),
                                           0 if ws is None else ws.numel(), _stream(stream)), "dll_conv_valid_wgrad_partial")


def dll_conv_valid_wgrad_finish(cs: ConvSpec, dw, dbias, ws, stream=None) -> None:
    d = conv_desc(cs)
    _ok(lib().dll_conv_valid_wgrad_finish(C.byref(d), _ptr(dw), _ptr(dbias), _ptr(ws), 0 if ws is None else ws.numel(),
                                          _stream(stream)), "dll_conv_valid_wgrad_finish")


def dll_conv_valid_wgrad_noalloc(cs: ConvSpec, x, dy, y, pool_idx, dw, dbias, stream=None) -> None:
    d = conv_desc(cs)
    _ok(lib().dll_conv_valid_wgrad_noalloc(C.byref(d), _ptr(x), _ptr(dy), _ptr(y), _ptr(pool_idx), _ptr(dw), _ptr(dbias),
                                           _stream(stream)), "dll_conv_valid_wgrad_noalloc")


def dll_crbm_workspace_bytes(cs: ConvSpec) -> int:
    d = conv_desc(cs)
    return int(lib().dll_crbm_workspace_bytes(C.byref(d)))


def dll_crbm_cd1_step(cs: ConvSpec, v0, W, b_hid, c_vis, uniform, h0_sample_in, lr, dW, db, dc, h0_prob=None,
                      h0_sample=None, v1=None, h1_prob=None, recon_mse=None, ws=None, stream=None) -> None:
    d = conv_desc(cs)
    _ok(lib().dll_crbm_cd1_step(C.byref(d), _ptr(v0), _ptr(W), _ptr(b_hid), _ptr(c_vis), _ptr(uniform),
                                _ptr(h0_sample_in), C.c_float(lr), _ptr(dW), _ptr(db), _ptr(dc), _ptr(h0_prob),
                                _ptr(h0_sample), _ptr(v1), _ptr(h1_prob), _ptr(recon_mse), _ptr(ws),
                                0 if ws is None else ws.numel(), _stream(stream)), "dll_crbm_cd1_step")


def dll_crbm_cd1_step_units(cs: ConvSpec, visible: int, hidden_pool: int, v0, W, b_hid, c_vis, uniform, h0_sample_in, lr,
                            dW, db, dc, h0_prob=None, h0_sample=None, pool_prob=None, v1=None, h1_prob=None,
                            recon_mse=None, ws=None, stream=None) -> None:
    d = conv_desc(cs)
    _ok(lib().dll_crbm_cd1_step_units(C.byref(d), int(visible), int(hidden_pool), _ptr(v0), _ptr(W), _ptr(b_hid),
                                      _ptr(c_vis), _ptr(uniform), _ptr(h0_sample_in), C.c_float(lr), _ptr(dW), _ptr(db),
                                      _ptr(dc), _ptr(h0_prob), _ptr(h0_sample), _ptr(pool_prob), _ptr(v1), _ptr(h1_prob),
                                      _ptr(recon_mse), _ptr(ws), 0 if ws is None else ws.numel(), _stream(stream)),
        "dll_crbm_cd1_step_units")


def dll_rbm_workspace_bytes(batch: int, n_vis: int, n_hid: int) -> int:
    return int(lib().dll_rbm_workspace_bytes(batch, n_vis, n_hid))


def dll_rbm_cd1_step(batch: int, n_vis: int, n_hid: int, visible: int, v0, W, b_hid, c_vis, uniform, h0_sample_in, lr, dW,
                     db, dc, h0_prob=None, h0_sample=None, v1=None, h1_prob=None, recon_mse=None, ws=None,
                     stream=None) -> None:
    _ok(lib().dll_rbm_cd1_step(batch, n_vis, n_hid, int(visible), _ptr(v0), _ptr(W), _ptr(b_hid), _ptr(c_vis),
                               _ptr(uniform), _ptr(h0_sample_in), C.c_float(lr), _ptr(dW), _ptr(db), _ptr(dc),
                               _ptr(h0_prob), _ptr(h0_sample), _ptr(v1), _ptr(h1_prob), _ptr(recon_mse), _ptr(ws),
                               0 if ws is None else ws.numel(), _stream(stream)), "dll_rbm_cd1_step")


@dataclass
class NetHandle:
    """Host-side descriptor arrays kept alive for the duration of the calls."""
    desc: dll_net_desc
    convs: object
    denses: object


def net_desc(conv: Sequence[ConvSpec], dense: Sequence[DenseSpec], classes: int, batch: int = 0) -> NetHandle:
    """`batch` is needed only for a fully-connected network (no conv layers)."""
    convs = (dll_conv_desc * len(conv))(*[conv_desc(c) for c in conv])
    denses = (dll_dense_desc * len(dense))(*[dll_dense_desc(d.in_, d.out, ACT[d.act]) for d in dense])
    return NetHandle(dll_net_desc(len(conv), convs, len(dense), denses, classes, batch), convs, denses)


def dll_cnn_workspace_bytes(net: NetHandle) -> int:
    return int(lib().dll_cnn_workspace_bytes(C.byref(net.desc)))


def _ptr_array(ts: Optional[Sequence[Optional[torch.Tensor]]]):
    if ts is None:
        return None
    arr = (C.c_void_p * len(ts))(*[None if t is None else t.data_ptr() for t in ts])
    for t in ts:
        assert t is None or (t.is_cuda and t.is_contiguous())
    return arr


def dll_cnn_train_step(net: NetHandle, params: List[torch.Tensor], grads, x, labels, lr, loss, logits=None,
                       pool_idx=None, ws=None, stream=None) -> None:
    pa, ga, ia = _ptr_array(params), _ptr_array(grads), _ptr_array(pool_idx)
    _ok(lib().dll_cnn_train_step(C.byref(net.desc), pa, ga, _ptr(x), _ptr(labels), C.c_float(lr), _ptr(loss),
                                 _ptr(logits), ia, _ptr(ws), 0 if ws is None else ws.numel(), _stream(stream)),
        "dll_cnn_train_step")


def dll_cnn_forward_workspace_bytes(net: NetHandle) -> int:
    return int(lib().dll_cnn_forward_workspace_bytes(C.byref(net.desc)))


def dll_cnn_forward(net: NetHandle, params: List[torch.Tensor], x, logits=None, prob=None, ws=None, stream=None) -> None:
    pa = _ptr_array(params)
    _ok(lib().dll_cnn_forward(C.byref(net.desc), pa, _ptr(x), _ptr(logits), _ptr(prob), _ptr(ws),
                              0 if ws is None else ws.numel(), _stream(stream)), "dll_cnn_forward")


def dll_cnn_train_step_momentum(net: NetHandle, params: List[torch.Tensor], velocity: List[torch.Tensor], grads, x, labels, lr,
                                momentum, weight_decay, loss, logits=None, pool_idx=None, ws=None, stream=None) -> None:
    pa, va, ga, ia = _ptr_array(params), _ptr_array(velocity), _ptr_array(grads), _ptr_array(pool_idx)
    _ok(lib().dll_cnn_train_step_momentum(C.byref(net.desc), pa, va, ga, _ptr(x), _ptr(labels), C.c_float(lr),
                                          C.c_float(momentum), C.c_float(weight_decay), _ptr(loss), _ptr(logits), ia, _ptr(ws),
                                          0 if ws is None else ws.numel(), _stream(stream)), "dll_cnn_train_step_momentum")
