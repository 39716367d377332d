"""Shared helpers of the parity tests: error metric and descriptor conversion."""
import numpy as np

from oracle import oracle as orc
from paper_1804_04512_amd import workloads as wl

ACT = {"identity": orc.ACT_IDENTITY, "sigmoid": orc.ACT_SIGMOID, "relu": orc.ACT_RELU}
TOL_FWD = 1e-4    # forward outputs, loss, logits, probabilities
TOL_GRAD = 5e-4   # gradients and parameter deltas


# (worst per-tensor error, worst element-wise relative error, number of tensors) of the test that is
# running; conftest.py prints the table at the end of the session
REPORT = {}
_current = [None]


def begin_report(test_name):
    _current[0] = test_name


def max_rel_err(got, ref) -> float:
    """Per-tensor error: max |got - ref| / max(max |ref|, 1e-30).  Also records, for the session's
    report, the element-wise relative error max |got - ref| / |ref| over the elements with
    |ref| > 1e-3 max |ref| (small elements excluded: ReLU zeros and cancelling sums make the
    ratio meaningless there)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if ref.size == 0:
        return 0.0
    assert np.all(np.isfinite(got)), "non-finite values in the GPU result"
    diff = np.abs(got - ref)
    top = max(np.abs(ref).max(), 1e-30)
    err = float(diff.max() / top)
    big = np.abs(ref) > 1e-3 * top
    elem = float((diff[big] / np.abs(ref[big])).max()) if big.any() else 0.0
    if _current[0] is not None:
        e0, l0, n0 = REPORT.get(_current[0], (0.0, 0.0, 0))
        REPORT[_current[0]] = (max(e0, err), max(l0, elem), n0 + 1)
    return err


def odesc(cs: wl.ConvSpec, pool=None, act=None):
    return orc.conv_desc(cs.N, cs.C, cs.H, cs.W, cs.K, cs.R, cs.S, cs.pad,
                         ACT[cs.act] if act is None else act, cs.pool if pool is None else pool)


def onet(w: wl.CnnWorkload) -> orc.Net:
    return orc.Net([odesc(c) for c in w.conv], [(d.in_, d.out, ACT[d.act]) for d in w.dense], w.classes,
                   batch=0 if w.conv else w.batch)


def check_idx_bytes(raw, relu, y_gpu):
    """Splits the library's pooling-index bytes: bits 0-1 are the window position; bit 2 is set
    exactly where a ReLU layer's pooled output (the library's own y) is zero; nothing else is set.
    Returns the positions."""
    flags = raw & ~np.uint8(3)
    if relu:
        assert np.array_equal(flags, np.where(y_gpu > 0, 0, 4).astype(np.uint8))
    else:
        assert not flags.any()
    return raw & np.uint8(3)


def check_idx_flags_against(raw, relu, y_ref, tol=2e-5):
    """Flag bits against a reference output: clear where y_ref is clearly positive; where y_ref
    is zero they may only be clear if the GPU's y rounded to a tiny positive value, which must
    stay rare."""
    flags = raw & ~np.uint8(3)
    if not relu:
        assert not flags.any()
        return
    assert not (flags & ~np.uint8(4)).any()
    scale = max(float(np.abs(y_ref).max()), 1e-30)
    assert not (flags[y_ref > tol * scale] != 0).any(), "inactive flag on a clearly active unit"
    stray = int((flags[y_ref == 0] == 0).sum())
    assert stray <= max(4, int(1e-4 * raw.size)), f"{stray} units flagged active where the reference output is zero"


def check_relu_activity(active_gpu, y_ref, tol=2e-5):
    """Activity decisions (unit output > 0) of a ReLU layer taken from the GPU's fp32 output against
    a reference output: they may differ only inside a rounding band around zero, and rarely."""
    active_ref = y_ref > 0
    differ = active_gpu != active_ref
    n = int(differ.sum())
    if n:
        scale = max(float(np.abs(y_ref).max()), 1e-30)
        assert not (differ & (np.abs(y_ref) > tol * scale)).any(), "activity differs on a unit that is clearly on"
        assert n <= max(4, int(1e-4 * differ.size)), f"{n} activity decisions differ"
    return n


def check_pool_idx(gpu_idx, ora_idx, prepool_act, y, tol=2e-5):
    """GPU and oracle may pick different window positions only where the two candidates are
    (nearly) tied or where the pooled output is 0 (ReLU: no gradient flows either way).
    prepool_act: oracle activations before pooling [N,K,Ho,Wo]; y: pooled oracle output."""
    diff = gpu_idx != ora_idx
    ndiff = int(diff.sum())
    if ndiff == 0:
        return 0
    N, K, Ho, Wo = prepool_act.shape
    win = prepool_act.reshape(N, K, Ho // 2, 2, Wo // 2, 2).transpose(0, 1, 2, 4, 3, 5).reshape(N, K, Ho // 2, Wo // 2, 4)
    picked = np.take_along_axis(win, gpu_idx[..., None].astype(np.int64), axis=-1)[..., 0]
    scale = max(float(np.abs(prepool_act).max()), 1e-30)
    gap = np.abs(picked.astype(np.float64) - y.astype(np.float64))
    bad = diff & (gap > tol * scale)
    assert not bad.any(), f"{int(bad.sum())} pooling indices differ at non-ties (max gap {gap[diff].max():.3e}, scale {scale:.3e})"
    # exact ties (e.g. a window of ReLU zeros) may go either way; near-ties must stay rare
    near = int((diff & (gap > 0)).sum())
    assert near <= max(4, int(1e-4 * diff.size)), f"too many near-tie pooling differences: {near} of {diff.size}"
    return ndiff
