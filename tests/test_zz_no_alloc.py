"""sa_moe_dispatch_static, the dispatch entry point that allocates nothing (its scratch is an array built into the
library), against sa_moe_dispatch on the same inputs: the two share every kernel, so all four outputs must be identical,
call after call, also when a smaller input follows a larger one in the same scratch."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
from helpers import assert_close, dev, host

pytestmark = pytest.mark.gpu


def logits_for(T, E, seed, tie_every):
    g = np.random.default_rng([77, seed, T, E])
    logits = g.standard_normal((T, E), dtype=np.float32)
    if tie_every:
        logits[::tie_every] = logits[::tie_every, :1]
    return logits


def both(sa, logits):
    d = dev(logits)
    ref = [host(t) for t in sa.sa_moe_dispatch(d)]
    T, E = logits.shape
    # the caller's outputs exist before the call; the call itself goes straight to the C ABI and allocates nothing
    out = (torch.full((T,), -7, dtype=torch.int32, device="cuda"), torch.full((T,), -7, dtype=torch.int32, device="cuda"),
           torch.full((max(E, 4),), -7, dtype=torch.int32, device="cuda")[:E], torch.full((T,), -7.0, dtype=torch.float32, device="cuda"))
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    lib = sa.load_library()
    rc = lib.sa_moe_dispatch_static(ctypes.c_void_p(d.data_ptr()), ctypes.c_long(T), E, ctypes.c_void_p(out[0].data_ptr()),
                                    ctypes.c_void_p(out[1].data_ptr()), ctypes.c_void_p(out[2].data_ptr()),
                                    ctypes.c_void_p(out[3].data_ptr()), ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert rc == 0, lib.sa_last_error()
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    return ref, [host(t) for t in out]


@pytest.mark.parametrize("sizes,E,tie_every", [
    ((100000, 40000), 2, 7),          # histograms summed by the scatter pass; the second call is smaller
    ((200001, 50001, 200001), 8, 5),  # the separate scan kernel, then a smaller input, then the large one again
    ((40000, 197), 4, 0),             # the second call takes the one-launch path and leaves the scratch alone
])
def test_static_dispatch_equals_the_workspace_one_call_after_call(sa, sizes, E, tie_every):
    for i, T in enumerate(sizes):
        logits = logits_for(T, E, i, tie_every)
        (perm_r, eo_r, cnt_r, gate_r), (perm, eo, cnt, gate) = both(sa, logits)
        assert np.array_equal(cnt, cnt_r), (T, cnt, cnt_r)
        assert np.array_equal(eo, eo_r) and np.array_equal(perm, perm_r), T
        assert np.array_equal(gate, gate_r), T
        # and both are the oracle's result
        perm_o, eo_o, cnt_o, gate_o = oracle.moe_dispatch(logits)
        assert np.array_equal(cnt, cnt_o) and np.array_equal(eo, eo_o) and np.array_equal(perm, perm_o)
        assert_close(gate, gate_o, 1e-6, 0.0, "gate")


def test_static_dispatch_rejects_what_its_scratch_cannot_hold(sa):
    lib = sa.load_library()
    limit = lib.sa_moe_dispatch_static_max_tokens()
    assert limit == 1 << 20
    fake = ctypes.c_void_p(0x1000)
    rc = lib.sa_moe_dispatch_static(fake, ctypes.c_long(limit + 1), 2, fake, fake, fake, fake, ctypes.c_void_p(None))
    assert rc == -6 and b"exceed" in lib.sa_last_error()
    # no tokens: counts are zeroed, nothing else is touched
    cnt = torch.full((4,), 5, dtype=torch.int32, device="cuda")
    rc = lib.sa_moe_dispatch_static(ctypes.c_void_p(None), ctypes.c_long(0), 2, ctypes.c_void_p(None), ctypes.c_void_p(None),
                                    ctypes.c_void_p(cnt.data_ptr()), ctypes.c_void_p(None),
                                    ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert rc == 0
    torch.cuda.synchronize()
    assert cnt.tolist() == [0, 0, 5, 5]
