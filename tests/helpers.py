"""Shared helpers of the GPU parity tests: host <-> device moves and tolerance checks."""
import numpy as np
import torch


def dev(a):
    """numpy -> contiguous cuda tensor (uint64 travels as int64 bits)."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint64:
        a = a.view(np.int64)
    return torch.from_numpy(a).cuda()


def host(t, dtype=None):
    a = t.detach().cpu().numpy()
    if dtype is not None:
        a = a.view(dtype)
    return a


def codes_host(t):
    return host(t).view(np.uint64)


def assert_close(got, ref, rtol, atol, what=""):
    """|got - ref| <= atol + rtol * |ref| elementwise; ref is the fp64 oracle value."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    err = np.abs(got - ref)
    lim = atol + rtol * np.abs(ref)
    bad = err > lim
    if bad.any():
        i = np.unravel_index(np.argmax(err - lim), err.shape)
        raise AssertionError("%s: %d of %d outside tolerance; worst at %s got %r ref %r"
                             % (what, int(bad.sum()), bad.size, i, got[i], ref[i]))


# Spec tolerance of the floating-point attention outputs.
ATTN_RTOL, ATTN_ATOL = 1e-4, 1e-5


def kv_tolerance(ref):
    """Unscaled K^T V partial sums grow like sqrt(N): the absolute term scales with their rms."""
    rms = float(np.sqrt(np.mean(np.square(ref)))) if ref.size else 1.0
    return 1e-4, 1e-5 * max(1.0, rms)
