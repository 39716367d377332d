"""The C-ABI library loads, exports every symbol the header declares, and rejects bad
arguments on the host before anything is launched (no GPU needed)."""
import ctypes as C
import os
import re

import pytest

from paper_1804_04512_amd import binding
from paper_1804_04512_amd.workloads import ConvSpec, DenseSpec

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "dll_conv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dll_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_are_exported():
    L = binding.lib()
    names = declared_symbols()
    assert set(names) == set(binding.SYMBOLS)
    for n in names:
        assert getattr(L, n) is not None


def test_status_strings():
    L = binding.lib()
    seen = {L.dll_status_string(i).decode() for i in range(7)}
    assert len(seen) == 7 and "ok" in seen


def test_workspace_queries_are_host_side():
    cs = ConvSpec(8, 1, 28, 28, 8, 5, 5, 0, "sigmoid", 1)
    assert binding.dll_conv_workspace_bytes(cs) > 0
    assert binding.dll_conv_workspace_bytes(cs) % 256 == 0
    assert binding.dll_crbm_workspace_bytes(ConvSpec(64, 1, 28, 28, 40, 9, 9)) > 0
    net = binding.net_desc([ConvSpec(4, 1, 28, 28, 8, 5, 5, 0, "relu", 2), ConvSpec(4, 8, 12, 12, 8, 5, 5, 0, "relu", 2)],
                           [DenseSpec(128, 150, "relu"), DenseSpec(150, 10)], 10)
    assert binding.dll_cnn_workspace_bytes(net) > 0
    bad = binding.net_desc([ConvSpec(4, 1, 28, 28, 8, 5, 5, 0, "relu", 2)], [DenseSpec(77, 10)], 10)
    assert binding.dll_cnn_workspace_bytes(bad) == 0          # flatten size mismatch
    assert binding.dll_conv_workspace_bytes(ConvSpec(1, 1, 5, 5, 1, 3, 3, 0, "relu", 2)) == 0   # odd map + pool
    # fully-connected networks: the batch size comes from the descriptor
    dense = [DenseSpec(784, 500, "sigmoid"), DenseSpec(500, 250, "sigmoid"), DenseSpec(250, 10)]
    assert binding.dll_cnn_workspace_bytes(binding.net_desc([], dense, 10, 100)) > 0
    assert binding.dll_cnn_forward_workspace_bytes(binding.net_desc([], dense, 10, 100)) > 0
    assert binding.dll_cnn_workspace_bytes(binding.net_desc([], dense, 10, 0)) == 0
    assert binding.dll_cnn_workspace_bytes(binding.net_desc([], dense, 11, 100)) == 0        # classes != last layer
    assert binding.dll_rbm_workspace_bytes(100, 784, 500) > 0
    assert binding.dll_rbm_workspace_bytes(100, 784, 500) % 256 == 0
    assert binding.dll_rbm_workspace_bytes(0, 784, 500) == 0


def test_argument_errors_are_reported_before_any_launch():
    L = binding.lib()
    d = binding.conv_desc(ConvSpec(2, 1, 8, 8, 4, 3, 3))
    one = C.c_void_p(0x1000)   # never dereferenced: validation fails first
    assert L.dll_conv_valid_fwd(None, one, one, None, one, None, None, 0, None) == 1           # NULL desc
    assert L.dll_conv_valid_fwd(C.byref(d), None, one, None, one, None, None, 0, None) == 1     # NULL x
    assert L.dll_conv_valid_fwd(C.byref(d), one, one, None, one, None, None, 0, None) == 2      # y aliases x
    bad = binding.conv_desc(ConvSpec(2, 1, 8, 8, 4, 3, 3, 3))
    assert L.dll_conv_valid_fwd(C.byref(bad), one, one, None, one, None, None, 0, None) == 2    # pad > R-1
    bad = binding.conv_desc(ConvSpec(2, 1, 2, 2, 4, 3, 3))
    assert L.dll_conv_valid_fwd(C.byref(bad), one, one, None, one, None, None, 0, None) == 2    # filter > input
    bad = binding.conv_desc(ConvSpec(2, 1, 9, 9, 4, 3, 3, 0, "relu", 2))
    assert L.dll_conv_valid_fwd(C.byref(bad), one, one, None, one, one, None, 0, None) == 2     # odd map + pool
    bad = binding.dll_conv_desc(2, 1, 8, 8, 4, 3, 3, 0, 9, 1)
    assert L.dll_conv_valid_fwd(C.byref(bad), one, one, None, one, None, None, 0, None) == 3    # unknown act
    bad = binding.conv_desc(ConvSpec(2, 1, 32, 32, 4, 13, 13))
    assert L.dll_conv_valid_fwd(C.byref(bad), one, one, None, one, None, None, 0, None) == 3    # 13x13 > 144 taps
    a, b, c, e = (C.c_void_p(0x1000 * i) for i in (1, 2, 3, 4))
    assert L.dll_conv_valid_wgrad(C.byref(d), a, b, None, None, c, None, None, 0, None) == 4    # no workspace
    assert L.dll_conv_valid_wgrad(C.byref(d), a, b, None, None, c, None, e, 16, None) == 4      # too small
    assert L.dll_conv_valid_wgrad_partial(C.byref(d), a, None, None, None, e, 1 << 30, None) == 1   # NULL dy
    assert L.dll_conv_valid_wgrad_partial(C.byref(d), a, b, None, None, e, 16, None) == 4           # too small
    assert L.dll_conv_valid_wgrad_finish(C.byref(d), None, None, e, 1 << 30, None) == 1             # NULL dw
    assert L.dll_conv_valid_wgrad_finish(C.byref(d), c, None, e, 16, None) == 4                     # too small
    assert L.dll_conv_valid_wgrad_finish(C.byref(d), e, None, e, 1 << 30, None) == 2                # dw is the workspace
    assert L.dll_conv_full_bwd(C.byref(d), a, None, None, None, c, None, 0, None) == 1          # NULL w
    pooled = binding.conv_desc(ConvSpec(2, 1, 8, 8, 4, 3, 3, 0, "relu", 2))
    assert L.dll_conv_full_bwd(C.byref(pooled), a, b, None, c, e, None, 0, None) == 1           # pool needs idx
    assert L.dll_crbm_cd1_step(C.byref(d), a, b, c, e, None, None, 0.0, *([a] * 8), None, 0, None) == 1   # no uniforms
    assert L.dll_crbm_cd1_step_units(C.byref(d), 0, 1, a, b, c, e, None, None, 0.0, *([a] * 9), None, 0, None) == 1  # no uniforms
    assert L.dll_crbm_cd1_step_units(C.byref(d), 7, 1, a, b, c, e, a, None, 0.0, b, c, e, *([None] * 6), None, 0, None) == 2
    odd = binding.conv_desc(ConvSpec(2, 1, 9, 8, 4, 3, 3))
    assert L.dll_crbm_cd1_step_units(C.byref(odd), 0, 2, a, b, c, e, a, None, 0.0, b, c, e, *([None] * 6), None, 0, None) == 2
    assert L.dll_rbm_cd1_step(4, 8, 6, 0, a, b, c, e, None, None, 0.0, *([a] * 8), None, 0, None) == 1    # no uniforms
    assert L.dll_rbm_cd1_step(4, 0, 6, 0, a, b, c, e, a, None, 0.0, *([a] * 8), None, 0, None) == 2       # no visible units
    assert L.dll_rbm_cd1_step(4, 8, 6, 0, a, b, c, e, a, None, 0.0, b, a, a, *([None] * 5), None, 0, None) == 2  # dW aliases W
    assert L.dll_rbm_cd1_step(4, 8, 6, 0, a, b, c, e, a, None, 0.0, a, b, c, *([None] * 5), None, 0, None) == 4  # no workspace
    assert L.dll_cnn_train_step(None, None, None, None, None, 0.0, None, None, None, None, 0, None) == 1
    assert L.dll_cnn_forward(None, None, None, None, None, None, 0, None) == 1
    assert L.dll_cnn_train_step_momentum(None, None, None, None, None, None, 0.0, 0.0, 0.0, None, None, None, None, 0, None) == 1
    assert L.dll_cnn_forward_workspace_bytes(None) == 0


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", "/nonexistent/libdll_conv.so")
    with pytest.raises(FileNotFoundError):
        binding.lib()
