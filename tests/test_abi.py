"""Host-only checks of the C ABI: the library loads, exports what the header declares and
rejects bad arguments before touching a GPU."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "shiftadd.h")
LIB = os.path.join(ROOT, "paper_2306_06446_amd", "libshiftadd.so")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sa_[a-z0-9_]+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        import sys
        sys.path.insert(0, ROOT)
        from paper_2306_06446_amd import build
        build.build_library(verbose=False)
    lib = ctypes.CDLL(LIB)
    lib.sa_last_error.restype = ctypes.c_char_p
    return lib


def test_header_declares_the_north_star_calls():
    names = declared_functions()
    for n in ("sa_binarize", "sa_additive_attention", "sa_hamming_attention", "sa_shift_linear",
              "sa_moe_dispatch", "sa_block_forward"):
        assert n in names


def test_library_exports_every_declared_symbol(lib):
    from paper_2306_06446_amd import binding
    names = declared_functions()
    assert len(names) >= 19
    for n in names:
        assert hasattr(lib, n), "libshiftadd.so does not export %s" % n
    assert sorted(binding.EXPORTS) == names


def test_version(lib):
    assert lib.sa_version() >= 100


def test_argument_errors_are_reported_without_a_gpu(lib):
    null = ctypes.c_void_p(None)
    fake = ctypes.c_void_p(0x1000)
    odd = ctypes.c_void_p(0x1004)
    # nbits not a multiple of 64
    assert lib.sa_binarize(fake, 1, 1, 1, 64, fake, 65, fake, null) == -2
    assert b"nbits" in lib.sa_last_error()
    # without proj nbits must equal d
    assert lib.sa_binarize(fake, 1, 1, 1, 64, null, 128, fake, null) == -2
    # misaligned pointer
    assert lib.sa_binarize(odd, 1, 1, 1, 64, fake, 64, fake, null) == -3
    # unsupported head dim
    assert lib.sa_binarize(fake, 1, 1, 1, 48, fake, 64, fake, null) == -6
    # empty problem is fine and launches nothing
    assert lib.sa_binarize(null, 0, 5, 1, 64, null, 64, null, null) == 0
    assert lib.sa_last_error() == b""
    # additive attention: bad phases, bad dv, missing workspace
    f = ctypes.c_float(1.0)
    assert lib.sa_additive_attention(fake, fake, fake, fake, 1, 1, 4, 4, 64, 64, f, fake, 0, null,
                                     ctypes.c_size_t(0), null) == -1
    assert lib.sa_additive_attention(fake, fake, fake, fake, 1, 1, 4, 4, 64, 48, f, fake, 3, null,
                                     ctypes.c_size_t(0), null) == -6
    lib.sa_additive_attention_workspace_bytes.restype = ctypes.c_size_t
    need = lib.sa_additive_attention_workspace_bytes(8, 4, 16384, 256, 64)
    assert need > 0 and need % (8 * 4 * 256 * 64 * 4) == 0
    assert lib.sa_additive_attention(fake, fake, fake, fake, 8, 4, 16384, 16384, 256, 64, f, fake, 3, null,
                                     ctypes.c_size_t(0), null) == -4
    # hamming: zero keys, non-finite scale
    assert lib.sa_hamming_attention(fake, fake, fake, fake, 1, 1, 4, 0, 64, 64, f, null, null) == -2
    assert lib.sa_hamming_attention(fake, fake, fake, fake, 1, 1, 4, 4, 64, 64, ctypes.c_float(float("nan")),
                                    null, null) == -1
    # shift linear: odd K, K that is not a multiple of 32 (any variant), unknown variant
    M = ctypes.c_long(4)
    z0 = ctypes.c_size_t(0)
    assert lib.sa_shift_linear(fake, fake, null, fake, M, 33, 8, 0, null, z0, null) == -2
    assert lib.sa_shift_linear(fake, fake, null, fake, M, 64, 8, 7, null, z0, null) == -1
    assert lib.sa_shift_linear(fake, fake, null, fake, M, 48, 8, 1, null, z0, null) == -2
    assert lib.sa_shift_linear(fake, fake, null, fake, M, 96, 8, 1, null, z0, null) == -4   # planes workspace (96 -> 128 per row)
    assert lib.sa_shift_planes_bytes(96, 8) == 2 * 8 * 128 and lib.sa_shift_planes_bytes(48, 8) == 0
    assert lib.sa_shift_linear(null, fake, null, fake, M, 64, 8, 0, null, z0, null) == -1
    assert lib.sa_shift_linear(fake, fake, null, fake, M, 64, 8, 1, null, z0, null) == -4   # planes workspace
    # dispatch: E out of range, missing workspace
    T = ctypes.c_long(100)
    assert lib.sa_moe_dispatch(fake, T, 1, fake, fake, fake, fake, null, ctypes.c_size_t(0), null) == -2
    # (up to 32768 tokens the dispatch is one launch without scratch; longer inputs need the workspace)
    lib.sa_moe_dispatch_workspace_bytes.restype = ctypes.c_size_t
    assert lib.sa_moe_dispatch_workspace_bytes(T, 2) == 0
    T = ctypes.c_long(100000)
    assert lib.sa_moe_dispatch_workspace_bytes(T, 2) >= 2 * 391 * 2 * 4
    assert lib.sa_moe_dispatch(fake, T, 2, fake, fake, fake, fake, null, ctypes.c_size_t(0), null) == -4
    # block: NULL descriptor
    lib.sa_block_workspace_bytes.restype = ctypes.c_size_t
    assert lib.sa_block_workspace_bytes(null) == 0
    assert lib.sa_block_forward(null, null) == -1


def test_argument_errors_of_the_layer_entry_points_without_a_gpu(lib):
    null = ctypes.c_void_p(None)
    fake = ctypes.c_void_p(0x1000)
    odd = ctypes.c_void_p(0x1008)
    f = ctypes.c_float(1.0)
    T = ctypes.c_long(10)
    z0 = ctypes.c_size_t(0)
    # LayerNorm: E not a multiple of 4, too wide, no output, logits without weights, misaligned
    ln = lib.sa_layernorm_quant
    assert ln(fake, T, 66, fake, fake, f, f, fake, null, null, null, null, 0, null, null) == -2
    assert ln(fake, T, 16384, fake, fake, f, f, fake, null, null, null, null, 0, null, null) == -6
    assert ln(fake, T, 64, fake, fake, f, f, null, null, null, null, null, 0, null, null) == -1
    assert ln(fake, T, 64, fake, fake, f, f, null, null, null, null, null, 2, fake, null) == -1
    assert ln(fake, T, 64, fake, fake, f, f, null, null, null, fake, fake, 9, fake, null) == -2
    assert ln(odd, T, 64, fake, fake, f, f, fake, null, null, null, null, 0, null, null) == -3
    assert ln(null, ctypes.c_long(0), 64, null, null, f, f, null, null, null, null, null, 0, null, null) == 0
    # fp32 shift Linear: parts out of range, N not divisible, residual with parts > 1, missing part pointer
    lin = lib.sa_shift_linear_f32
    assert lin(fake, fake, T, 64, 24, 0, f, null, 4, fake, fake, fake, null, z0, null) == -1
    assert lin(fake, fake, T, 64, 20, 0, f, null, 3, fake, fake, fake, null, z0, null) == -2
    assert lin(fake, fake, T, 64, 24, 0, f, fake, 2, fake, fake, null, null, z0, null) == -1
    assert lin(fake, fake, T, 64, 24, 0, f, null, 2, fake, null, null, null, z0, null) == -1
    assert lin(fake, fake, T, 64, 24, 1, f, null, 1, fake, null, null, null, z0, null) == -4
    # weight conversion, {0,1} attention, depthwise convolution, balancing loss
    assert lib.sa_shift_weights_from_float(fake, 4, 12, fake, null) == -2
    assert lib.sa_shift_weights_from_float(null, 4, 16, fake, null) == -1
    la = lib.sa_linear_attention_01
    assert la(fake, fake, fake, fake, 1, 1, 4, 4, 64, 64, ctypes.c_float(0.0), fake, fake, 3, fake, ctypes.c_size_t(1 << 20), null) == -1
    assert la(fake, fake, fake, fake, 1, 1, 4, 4, 65, 64, f, fake, fake, 3, fake, ctypes.c_size_t(1 << 20), null) == -2
    assert la(fake, fake, fake, fake, 1, 1, 4, 4, 64, 64, f, fake, fake, 3, null, z0, null) == -4
    assert lib.sa_dwconv3x3(fake, fake, null, fake, 0, 1, 4, 4, 6, null) == -2
    assert lib.sa_dwconv3x3(fake, fake, null, fake, 0, 1, 4, 4, 8, null) == -1     # out == v
    assert lib.sa_dwconv3x3(fake, fake, null, ctypes.c_void_p(0x2000), 0, 0, 4, 4, 8, null) == 0
    bl = lib.sa_moe_balance_loss
    assert bl(fake, T, 9, fake, f, fake, null, fake, ctypes.c_size_t(1 << 20), null) == -2
    assert bl(fake, T, 2, fake, ctypes.c_float(0.0), fake, null, fake, ctypes.c_size_t(1 << 20), null) == -1
    assert bl(fake, T, 2, fake, f, fake, null, null, z0, null) == -4
    # stages flag of the experts
    lib.sa_layer_workspace_bytes.restype = ctypes.c_size_t
    assert lib.sa_layer_workspace_bytes(null) == 0
    assert lib.sa_layer_forward(null, null) == -1


def test_bench_refuses_more_than_one_gpu():
    """The bench measures one GPU: asked for more, it exits with a message and code 2 before touching a device."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode == 2
    assert "one GPU" in (r.stdout + r.stderr)
