"""ctypes binding of libshiftadd.so: same names as the C ABI, argument marshalling only.

Tensors are torch tensors on the GPU (torch supplies device memory and the
stream, nothing else); every step of the path runs in the library's kernels.
A missing library is an error: there is no fallback of any kind.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libshiftadd.so")
_lib = None

SA_VARIANT_VALU, SA_VARIANT_MFMA, SA_VARIANT_AUTO, SA_VARIANT_MFMA_PREPARED = 0, 1, 2, 3
SA_MLP_ACCUMULATE = 4

EXPORTS = [
    "sa_version", "sa_last_error", "sa_binarize", "sa_binarize_ex", "sa_binarize_pair", "sa_additive_attention_workspace_bytes",
    "sa_additive_attention", "sa_linear_attention_01_workspace_bytes", "sa_linear_attention_01", "sa_dwconv3x3",
    "sa_hamming_attention", "sa_hamming_attention_fused", "sa_shift_planes_bytes", "sa_shift_planes_prepare",
    "sa_shift_linear_workspace_bytes", "sa_shift_linear", "sa_shift_linear_f32", "sa_layernorm_quant",
    "sa_shift_weights_from_float", "sa_shift_linear_qkv_codes",
    "sa_moe_dispatch_workspace_bytes", "sa_moe_dispatch", "sa_moe_dispatch_static_max_tokens", "sa_moe_dispatch_static",
    "sa_moe_balance_loss_workspace_bytes", "sa_moe_balance_loss", "sa_quantize_act", "sa_quantize_act_half", "sa_requant_lut",
    "sa_shift_mlp_workspace_bytes", "sa_shift_mlp", "sa_mult_mlp_workspace_bytes",
    "sa_mult_mlp_f16", "sa_mult_mlp_f16_half", "sa_gather_rows", "sa_combine_rows", "sa_block_workspace_bytes",
    "sa_block_forward", "sa_moe_linear_workspace_bytes", "sa_moe_linear", "sa_probe_mfma", "sa_layer_workspace_bytes", "sa_layer_forward",
]


class SAError(RuntimeError):
    def __init__(self, code, text):
        super().__init__("libshiftadd error %d: %s" % (code, text))
        self.code = code


class SaRows(ctypes.Structure):
    _fields_ = [("rows_or_null", ctypes.c_void_p), ("counts_or_null", ctypes.c_void_p),
                ("expert", ctypes.c_int), ("max_rows", ctypes.c_long)]


class SaBlockDesc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int) for n in
                ("B", "N", "H", "d", "nbits", "dv", "attention", "hid", "moe", "shift_variant")] + \
               [(n, ctypes.c_float) for n in
                ("attn_scale", "act_inv_scale", "requant_scale", "out_scale")] + \
               [(n, ctypes.c_void_p) for n in
                ("q", "k", "v", "proj", "logits", "w1", "w2", "lut", "mw1", "mw2", "o", "y",
                 "workspace")] + \
               [("workspace_bytes", ctypes.c_size_t)]


class SaLayerDesc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int) for n in
                ("B", "N", "H", "nbits", "E", "hid", "attention", "moe", "shift_variant")] + \
               [(n, ctypes.c_float) for n in
                ("eps", "ln_inv_scale", "qkv_scale", "attn_scale", "act_inv_scale", "o_scale", "requant_scale",
                 "out_scale")] + \
               [(n, ctypes.c_void_p) for n in
                ("x", "gamma1", "beta1", "gamma2", "beta2", "wqkv", "wo", "proj", "wg", "bg", "w1", "w2", "lut",
                 "mw1", "mw2", "y", "workspace")] + \
               [("workspace_bytes", ctypes.c_size_t)]


def load_library():
    """Load the in-tree library; raises if it has not been built."""
    global _lib, LIB_PATH
    if _lib is None:
        LIB_PATH = os.environ.get("SHIFTADD_LIB", LIB_PATH)    # another build of the same library
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                "libshiftadd.so is not built (%s): run `python -c 'import __graft_entry__ as g; "
                "g.build()'` first; there is no fallback path" % LIB_PATH)
        lib = ctypes.CDLL(LIB_PATH)
        lib.sa_last_error.restype = ctypes.c_char_p
        lib.sa_moe_dispatch_static_max_tokens.restype = ctypes.c_long
        for name in ("sa_moe_balance_loss_workspace_bytes", "sa_additive_attention_workspace_bytes", "sa_linear_attention_01_workspace_bytes", "sa_moe_dispatch_workspace_bytes",
                     "sa_shift_linear_workspace_bytes", "sa_shift_planes_bytes",
                     "sa_shift_mlp_workspace_bytes", "sa_mult_mlp_workspace_bytes",
                     "sa_block_workspace_bytes", "sa_layer_workspace_bytes", "sa_moe_linear_workspace_bytes"):
            getattr(lib, name).restype = ctypes.c_size_t
        _lib = lib
    return _lib


def _check(code):
    if code != 0:
        raise SAError(code, load_library().sa_last_error().decode())


def _ptr(t):
    if t is None:
        return ctypes.c_void_p(None)
    assert t.is_cuda and t.is_contiguous(), "device-resident contiguous tensors only"
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _f(x):
    return ctypes.c_float(x)


def _l(x):
    return ctypes.c_long(x)


def _z(x):
    return ctypes.c_size_t(x)


def _rows(rows=None, counts=None, expert=0, max_rows=0):
    return SaRows(None if rows is None else rows.data_ptr(),
                  None if counts is None else counts.data_ptr(), expert, max_rows)


def _workspace(nbytes, device):
    return torch.empty(max(int(nbytes), 16), dtype=torch.uint8, device=device)


def sa_probe_mfma(kind, operands, workgroups, iters, out=None):
    """Register-only matrix-instruction loop (measurement helper): returns the 3 x uint64 device tensor
    [shader cycles, 100 MHz wall ticks, scratch] of workgroup 0."""
    if out is None:
        out = torch.zeros(4, dtype=torch.int64, device="cuda")
    _check(load_library().sa_probe_mfma(kind, operands, workgroups, iters, _ptr(out), _stream()))
    return out


def sa_version():
    return load_library().sa_version()


def sa_binarize(x, proj, nbits, codes=None, variant=None):
    B, N, H, d = x.shape
    if codes is None:
        codes = torch.empty((B, H, N, nbits // 64), dtype=torch.int64, device=x.device)
    lib = load_library()
    if variant is None:
        _check(lib.sa_binarize(_ptr(x), B, N, H, d, _ptr(proj), nbits, _ptr(codes), _stream()))
    else:
        _check(lib.sa_binarize_ex(_ptr(x), B, N, H, d, _ptr(proj), nbits, _ptr(codes), variant, _stream()))
    return codes


def sa_binarize_pair(q, k, proj, nbits, q_codes=None, k_codes=None):
    """Q and K of one block through the same hash, one launch where the matrix-core kernel takes the shape."""
    B, N, H, d = q.shape
    if q_codes is None:
        q_codes = torch.empty((B, H, N, nbits // 64), dtype=torch.int64, device=q.device)
    if k_codes is None:
        k_codes = torch.empty((B, H, N, nbits // 64), dtype=torch.int64, device=q.device)
    _check(load_library().sa_binarize_pair(_ptr(q), _ptr(k), B, N, H, d, _ptr(proj), nbits, _ptr(q_codes),
                                           _ptr(k_codes), _stream()))
    return q_codes, k_codes


def sa_additive_attention(q_codes, k_codes, v, scale, nbits, phases=3, kv=None, out=None,
                          workspace=None):
    lib = load_library()
    B, H, Nq, W = q_codes.shape if q_codes is not None else k_codes.shape
    Nk = k_codes.shape[2] if k_codes is not None else 0
    dv = v.shape[3] if v is not None else kv.shape[3]
    dev = (v if v is not None else kv).device
    if kv is None:
        kv = torch.empty((B, H, nbits, dv), dtype=torch.float32, device=dev)
    if out is None and (phases & 2):
        out = torch.empty((B, Nq, H, dv), dtype=torch.float32, device=dev)
    if workspace is None:
        workspace = _workspace(lib.sa_additive_attention_workspace_bytes(B, H, Nk, nbits, dv), dev)
    _check(lib.sa_additive_attention(_ptr(q_codes), _ptr(k_codes), _ptr(v), _ptr(out), B, H, Nq, Nk,
                                     nbits, dv, _f(scale), _ptr(kv), phases, _ptr(workspace),
                                     _z(workspace.numel()), _stream()))
    return out, kv


def sa_linear_attention_01(q_codes, k_codes, v, eps, nbits, phases=3, kv=None, ksum=None, out=None, workspace=None):
    """Normalised linear attention on {0,1} codes; returns (out, kv, ksum)."""
    lib = load_library()
    B, H, Nq, W = q_codes.shape if q_codes is not None else k_codes.shape
    if q_codes is None:
        Nq = 0
    Nk = k_codes.shape[2] if k_codes is not None else 0
    dv = v.shape[3] if v is not None else kv.shape[3]
    dev = (v if v is not None else kv).device
    if kv is None:
        kv = torch.empty((B, H, nbits, dv), dtype=torch.float32, device=dev)
    if ksum is None:
        ksum = torch.empty((B, H, nbits), dtype=torch.int32, device=dev)
    if out is None and (phases & 2):
        out = torch.empty((B, Nq, H, dv), dtype=torch.float32, device=dev)
    if workspace is None:
        workspace = _workspace(lib.sa_linear_attention_01_workspace_bytes(B, H, Nq, Nk, nbits, dv), dev)
    _check(lib.sa_linear_attention_01(_ptr(q_codes), _ptr(k_codes), _ptr(v), _ptr(out), B, H, Nq, Nk, nbits, dv,
                                      _f(eps), _ptr(kv), _ptr(ksum), phases, _ptr(workspace), _z(workspace.numel()),
                                      _stream()))
    return out, kv, ksum


def sa_dwconv3x3(v, w, bias=None, out=None, accumulate=False):
    """Depthwise 3x3 over the token grid: v [B, gh, gw, E], w [E, 3, 3]; adds to `out` when accumulate."""
    B, gh, gw, E = v.shape
    if out is None:
        assert not accumulate
        out = torch.empty_like(v)
    _check(load_library().sa_dwconv3x3(_ptr(v), _ptr(w), _ptr(bias), _ptr(out), int(bool(accumulate)), B, gh, gw, E,
                                       _stream()))
    return out


def sa_hamming_attention(q_codes, k_codes, v, scale, nbits, want_scores=False, out=None):
    B, H, Nq, W = q_codes.shape
    Nk = k_codes.shape[2]
    dv = v.shape[3]
    if out is None:
        out = torch.empty((B, Nq, H, dv), dtype=torch.float32, device=v.device)
    scores = torch.empty((B, H, Nq, Nk), dtype=torch.int16, device=v.device) if want_scores else None
    _check(load_library().sa_hamming_attention(_ptr(q_codes), _ptr(k_codes), _ptr(v), _ptr(out), B, H,
                                               Nq, Nk, nbits, dv, _f(scale), _ptr(scores), _stream()))
    return (out, scores) if want_scores else out


def sa_hamming_attention_fused(q_codes, k_codes, v, scale, nbits, act_inv_scale, out=None, xq=None, xh=None,
                               want_xq=True, want_xh=True, variant=SA_VARIANT_AUTO, want_out=True):
    """Hamming attention that also leaves its output as int8 codes (xq) and in fp16 (xh), both [B*Nq, H*dv]."""
    B, H, Nq, W = q_codes.shape
    Nk = k_codes.shape[2]
    dv = v.shape[3]
    dev = v.device
    if out is None and want_out:
        out = torch.empty((B, Nq, H, dv), dtype=torch.float32, device=dev)
    if xq is None and want_xq:
        xq = torch.empty((B * Nq, H * dv), dtype=torch.int8, device=dev)
    if xh is None and want_xh:
        xh = torch.empty((B * Nq, H * dv), dtype=torch.float16, device=dev)
    _check(load_library().sa_hamming_attention_fused(_ptr(q_codes), _ptr(k_codes), _ptr(v), _ptr(out), B, H, Nq, Nk,
                                                     nbits, dv, _f(scale), _ptr(None), _ptr(xq), _ptr(xh),
                                                     _f(act_inv_scale), variant, _stream()))
    return out, xq, xh


def sa_shift_weights_from_float(w):
    """fp32 weights [N, K] -> packed 4-bit shift weights [N, K/2] (sign, rounded log2 magnitude)."""
    N, K = w.shape
    w4 = torch.empty((N, K // 2), dtype=torch.uint8, device=w.device)
    _check(load_library().sa_shift_weights_from_float(_ptr(w), N, K, _ptr(w4), _stream()))
    return w4


def sa_shift_planes_prepare(w4):
    """Packed 4-bit weights [N, K/2] -> the two int8 operand planes [2, N, Kp] of the prepared MFMA variant
    (Kp = K rounded up to a multiple of 64, zero padded)."""
    lib = load_library()
    N, K = w4.shape[0], 2 * w4.shape[1]
    nbytes = lib.sa_shift_planes_bytes(K, N)
    if nbytes == 0:
        raise SAError(-2, "sa_shift_planes_prepare: K must be a multiple of 32")
    flat = torch.empty(nbytes, dtype=torch.int8, device=w4.device)
    _check(lib.sa_shift_planes_prepare(_ptr(w4), K, N, _ptr(flat), _z(nbytes), _stream()))
    Kp = (K + 63) // 64 * 64
    return flat[:2 * N * Kp].view(2, N, Kp)


def _out_width(w, variant):
    """Rows of a shift weight: packed [N, K/2], or prepared planes [2, N, K]."""
    return w.shape[1] if variant == SA_VARIANT_MFMA_PREPARED else w.shape[0]


def sa_shift_linear(x, w4, bias=None, variant=SA_VARIANT_AUTO, y=None, workspace=None):
    lib = load_library()
    M, K = x.shape
    N = _out_width(w4, variant)
    if y is None:
        y = torch.empty((M, N), dtype=torch.int32, device=x.device)
    if workspace is None:
        workspace = _workspace(lib.sa_shift_linear_workspace_bytes(_l(M), K, N, variant), x.device)
    _check(lib.sa_shift_linear(_ptr(x), _ptr(w4), _ptr(bias), _ptr(y), _l(M), K, N, variant,
                               _ptr(workspace), _z(workspace.numel()), _stream()))
    return y


def sa_shift_linear_f32(x, w4, scale, residual=None, parts=1, variant=SA_VARIANT_AUTO, ys=None, workspace=None):
    """fp32 outputs y_p = fma(float(acc), scale, residual): a tuple of `parts` [M, N / parts] tensors."""
    lib = load_library()
    M, K = x.shape
    N = _out_width(w4, variant)
    if ys is None:
        ys = tuple(torch.empty((M, N // parts), dtype=torch.float32, device=x.device) for _ in range(parts))
    if workspace is None:
        workspace = _workspace(lib.sa_shift_linear_workspace_bytes(_l(M), K, N, variant), x.device)
    y = list(ys) + [None] * (3 - len(ys))
    _check(lib.sa_shift_linear_f32(_ptr(x), _ptr(w4), _l(M), K, N, variant, _f(scale), _ptr(residual), parts,
                                   _ptr(y[0]), _ptr(y[1]), _ptr(y[2]), _ptr(workspace), _z(workspace.numel()),
                                   _stream()))
    return tuple(ys)


def sa_shift_linear_qkv_codes(x, wqkv, B, N, H, scale, variant=SA_VARIANT_MFMA, workspace=None, q_codes=None,
                              k_codes=None, v=None):
    """Fused Q/K/V projection with the sign hash in its epilogue: returns (q_codes, k_codes, v)."""
    lib = load_library()
    M, E = x.shape
    d = E // H
    if q_codes is None:
        q_codes = torch.empty((B, H, N, d // 64), dtype=torch.int64, device=x.device)
    if k_codes is None:
        k_codes = torch.empty((B, H, N, d // 64), dtype=torch.int64, device=x.device)
    if v is None:
        v = torch.empty((M, E), dtype=torch.float32, device=x.device)
    if workspace is None:
        workspace = _workspace(lib.sa_shift_linear_workspace_bytes(_l(M), E, 3 * E, variant), x.device)
    _check(lib.sa_shift_linear_qkv_codes(_ptr(x), _ptr(wqkv), B, N, H, E, variant, _f(scale), _ptr(q_codes),
                                         _ptr(k_codes), _ptr(v), _ptr(workspace), _z(workspace.numel()), _stream()))
    return q_codes, k_codes, v


def sa_layernorm_quant(x, gamma, beta, eps, inv_scale=1.0, want_ln=True, want_q=False, want_half=False,
                       wg=None, bg=None, ln=None, q=None, xh=None, logits=None):
    """Returns (ln, q, xh, logits); entries not asked for (want_* false and no buffer given) are None."""
    T, E = x.shape
    dev = x.device
    if ln is None and want_ln:
        ln = torch.empty((T, E), dtype=torch.float32, device=dev)
    if q is None and want_q:
        q = torch.empty((T, E), dtype=torch.int8, device=dev)
    if xh is None and want_half:
        xh = torch.empty((T, E), dtype=torch.float16, device=dev)
    n_exp = 0 if wg is None else wg.shape[1]
    if logits is None and wg is not None:
        logits = torch.empty((T, n_exp), dtype=torch.float32, device=dev)
    _check(load_library().sa_layernorm_quant(_ptr(x), _l(T), E, _ptr(gamma), _ptr(beta), _f(eps), _f(inv_scale),
                                             _ptr(ln), _ptr(q), _ptr(xh), _ptr(wg), _ptr(bg), n_exp, _ptr(logits),
                                             _stream()))
    return ln, q, xh, logits


def sa_moe_dispatch(logits, out=None, workspace=None):
    lib = load_library()
    T, E = logits.shape
    dev = logits.device
    if out is None:
        perm = torch.empty(T, dtype=torch.int32, device=dev)
        expert_of = torch.empty(T, dtype=torch.int32, device=dev)
        counts = torch.empty(max(E, 4), dtype=torch.int32, device=dev)[:E]
        gate = torch.empty(T, dtype=torch.float32, device=dev)
    else:
        perm, expert_of, counts, gate = out
    ws = workspace
    if ws is None:
        ws = _workspace(lib.sa_moe_dispatch_workspace_bytes(_l(T), E), dev)
    _check(lib.sa_moe_dispatch(_ptr(logits), _l(T), E, _ptr(perm), _ptr(expert_of), _ptr(counts),
                               _ptr(gate), _ptr(ws), _z(ws.numel()), _stream()))
    return perm, expert_of, counts, gate


def sa_moe_dispatch_static(logits, out=None):
    """sa_moe_dispatch without a workspace: the library's built-in scratch array is used (nothing is allocated by the call;
    the four output tensors are the caller's, made here only when `out` is not given)."""
    lib = load_library()
    T, E = logits.shape
    dev = logits.device
    if out is None:
        out = (torch.empty(T, dtype=torch.int32, device=dev), torch.empty(T, dtype=torch.int32, device=dev),
               torch.empty(max(E, 4), dtype=torch.int32, device=dev)[:E], torch.empty(T, dtype=torch.float32, device=dev))
    perm, expert_of, counts, gate = out
    _check(lib.sa_moe_dispatch_static(_ptr(logits), _l(T), E, _ptr(perm), _ptr(expert_of), _ptr(counts), _ptr(gate),
                                      _stream()))
    return perm, expert_of, counts, gate


def sa_moe_linear(xq, xh, logits, w4, w_half, out_scale, variant=SA_VARIANT_AUTO, y=None, want_routing=False,
                  workspace=None):
    """MoE form of one Linear layer: y [T, N] fp32 (and, on request, expert_of [T] int32 and gate [T] fp32)."""
    lib = load_library()
    T, K = xq.shape
    N = w_half.shape[0]
    if y is None:
        y = torch.empty((T, N), dtype=torch.float32, device=xq.device)
    expert_of = torch.empty(T, dtype=torch.int32, device=xq.device) if want_routing else None
    gate = torch.empty(T, dtype=torch.float32, device=xq.device) if want_routing else None
    if workspace is None:
        workspace = _workspace(lib.sa_moe_linear_workspace_bytes(_l(T), K, N, variant), xq.device)
    _check(lib.sa_moe_linear(_ptr(xq), _ptr(xh), _ptr(logits), _l(T), K, N, _ptr(w4), _ptr(w_half), _f(out_scale), _ptr(y),
                             _ptr(expert_of), _ptr(gate), variant, _ptr(workspace), _z(workspace.numel()), _stream()))
    return (y, expert_of, gate) if want_routing else y


def sa_moe_balance_loss(logits, alpha, noise_std):
    """Eq. 4 forward: returns (losses [2], sums [2, E]) as device tensors."""
    lib = load_library()
    T, E = logits.shape
    losses = torch.empty(4, dtype=torch.float32, device=logits.device)[:2]
    sums = torch.empty((2, E), dtype=torch.float32, device=logits.device)
    ws = _workspace(lib.sa_moe_balance_loss_workspace_bytes(_l(T), E), logits.device)
    _check(lib.sa_moe_balance_loss(_ptr(logits), _l(T), E, _ptr(alpha), _f(noise_std), _ptr(losses), _ptr(sums),
                                   _ptr(ws), _z(ws.numel()), _stream()))
    return losses, sums


def sa_quantize_act(x, inv_scale, q=None):
    if q is None:
        q = torch.empty(x.shape, dtype=torch.int8, device=x.device)
    _check(load_library().sa_quantize_act(_ptr(x), _l(x.numel()), _f(inv_scale), _ptr(q), _stream()))
    return q


def sa_quantize_act_half(x, inv_scale, q=None, xh=None):
    if q is None:
        q = torch.empty(x.shape, dtype=torch.int8, device=x.device)
    if xh is None:
        xh = torch.empty(x.shape, dtype=torch.float16, device=x.device)
    _check(load_library().sa_quantize_act_half(_ptr(x), _l(x.numel()), _f(inv_scale), _ptr(q), _ptr(xh), _stream()))
    return q, xh


def sa_requant_lut(y, s, lut, h=None):
    if h is None:
        h = torch.empty(y.shape, dtype=torch.int8, device=y.device)
    _check(load_library().sa_requant_lut(_ptr(y), _l(y.numel()), _f(s), _ptr(lut), _ptr(h), _stream()))
    return h


def sa_shift_mlp(xq, w1, w2, requant_scale, lut, rows=None, counts=None, expert=0, max_rows=None,
                 want_y2=True, y=None, gate=None, out_scale=1.0, variant=SA_VARIANT_AUTO, stages=3,
                 workspace=None):
    lib = load_library()
    T, E = xq.shape
    hid = _out_width(w1, variant)
    if max_rows is None:
        max_rows = T if rows is None or counts is not None else rows.numel()
    r = _rows(rows, counts, expert, max_rows)
    y2 = torch.empty((max_rows, E), dtype=torch.int32, device=xq.device) if want_y2 else None
    ws = workspace
    if ws is None:
        ws = _workspace(lib.sa_shift_mlp_workspace_bytes(_l(max_rows), E, hid), xq.device)
    _check(lib.sa_shift_mlp(_ptr(xq), ctypes.byref(r), E, hid, _ptr(w1), _ptr(w2), _f(requant_scale),
                            _ptr(lut), _ptr(y2), _ptr(y), _ptr(gate), _f(out_scale), variant, stages,
                            _ptr(ws), _z(ws.numel()), _stream()))
    return y2


def sa_mult_mlp_f16(x, w1, w2, rows=None, counts=None, expert=0, max_rows=None, want_out=True,
                    y=None, gate=None, stages=3, workspace=None):
    lib = load_library()
    T, E = x.shape
    hid = w1.shape[0]
    if max_rows is None:
        max_rows = T if rows is None or counts is not None else rows.numel()
    r = _rows(rows, counts, expert, max_rows)
    out = torch.empty((max_rows, E), dtype=torch.float32, device=x.device) if want_out else None
    ws = workspace
    if ws is None:
        ws = _workspace(lib.sa_mult_mlp_workspace_bytes(_l(max_rows), E, hid), x.device)
    _check(lib.sa_mult_mlp_f16(_ptr(x), ctypes.byref(r), E, hid, _ptr(w1), _ptr(w2), _ptr(out), _ptr(y),
                               _ptr(gate), stages, _ptr(ws), _z(ws.numel()), _stream()))
    return out


def sa_mult_mlp_f16_half(xh_all, w1, w2, rows=None, counts=None, expert=0, max_rows=None, want_out=True,
                         y=None, gate=None, stages=3, workspace=None):
    """The Mult expert on fp16 rows of all tokens [T, E]; `rows` are picked inside the first layer."""
    lib = load_library()
    T, E = xh_all.shape
    hid = w1.shape[0]
    if max_rows is None:
        max_rows = T if rows is None or counts is not None else rows.numel()
    r = _rows(rows, counts, expert, max_rows)
    out = torch.empty((max_rows, E), dtype=torch.float32, device=xh_all.device) if want_out else None
    ws = workspace
    if ws is None:
        ws = _workspace(lib.sa_mult_mlp_workspace_bytes(_l(max_rows), E, hid), xh_all.device)
    _check(lib.sa_mult_mlp_f16_half(_ptr(xh_all), ctypes.byref(r), E, hid, _ptr(w1), _ptr(w2), _ptr(out), _ptr(y),
                                    _ptr(gate), stages, _ptr(ws), _z(ws.numel()), _stream()))
    return out


def sa_gather_rows(src, rows=None, counts=None, expert=0, max_rows=None):
    if max_rows is None:
        max_rows = rows.numel()
    r = _rows(rows, counts, expert, max_rows)
    dst = torch.zeros((max_rows,) + tuple(src.shape[1:]), dtype=src.dtype, device=src.device)
    row_bytes = src[0].numel() * src.element_size()
    _check(load_library().sa_gather_rows(_ptr(src), _z(row_bytes), ctypes.byref(r), _ptr(dst), _stream()))
    return dst


def sa_combine_rows(src, y, rows=None, counts=None, expert=0, max_rows=None, gate=None):
    if max_rows is None:
        max_rows = src.shape[0]
    r = _rows(rows, counts, expert, max_rows)
    _check(load_library().sa_combine_rows(_ptr(src), ctypes.byref(r), _ptr(gate), src.shape[1], _ptr(y),
                                          _stream()))
    return y


class Block:
    """Holds the descriptor and the workspace of one block configuration; forward() enqueues it."""

    def __init__(self, *, B, N, H, d, nbits, dv, attention, hid, moe, attn_scale, act_inv_scale=1.0,
                 requant_scale=1.0, out_scale=1.0, q, k, v, proj, logits=None, w1=None, w2=None,
                 lut=None, mw1=None, mw2=None, shift_variant=SA_VARIANT_AUTO):
        lib = load_library()
        dev = q.device
        T, E = B * N, H * dv
        self.o = torch.empty((B, N, H, dv), dtype=torch.float32, device=dev)
        self.y = torch.empty((T, E), dtype=torch.float32, device=dev) if hid else None
        self._keep = (q, k, v, proj, logits, w1, w2, lut, mw1, mw2)
        d_ = SaBlockDesc()
        d_.B, d_.N, d_.H, d_.d, d_.nbits, d_.dv = B, N, H, d, nbits, dv
        d_.attention, d_.hid, d_.moe, d_.shift_variant = attention, hid, int(moe), shift_variant
        d_.attn_scale, d_.act_inv_scale = attn_scale, act_inv_scale
        d_.requant_scale, d_.out_scale = requant_scale, out_scale
        for name, t in (("q", q), ("k", k), ("v", v), ("proj", proj), ("logits", logits), ("w1", w1),
                        ("w2", w2), ("lut", lut), ("mw1", mw1), ("mw2", mw2), ("o", self.o),
                        ("y", self.y)):
            setattr(d_, name, None if t is None else t.data_ptr())
        nbytes = lib.sa_block_workspace_bytes(ctypes.byref(d_))
        self.ws = _workspace(nbytes, dev)
        d_.workspace = self.ws.data_ptr()
        d_.workspace_bytes = self.ws.numel()
        self.desc = d_

    def forward(self):
        _check(load_library().sa_block_forward(ctypes.byref(self.desc), _stream()))
        return self.o, self.y


class Layer:
    """Descriptor and workspace of one complete block (Eq. 2); forward() enqueues it and returns y."""

    _INTS = ("B", "N", "H", "nbits", "E", "hid", "attention", "moe", "shift_variant")
    _FLOATS = ("eps", "ln_inv_scale", "qkv_scale", "attn_scale", "act_inv_scale", "o_scale", "requant_scale",
               "out_scale")
    _TENSORS = ("x", "gamma1", "beta1", "gamma2", "beta2", "wqkv", "wo", "proj", "wg", "bg", "w1", "w2", "lut",
                "mw1", "mw2")

    def __init__(self, **kw):
        lib = load_library()
        d_ = SaLayerDesc()
        for n in self._INTS:
            setattr(d_, n, int(kw.get(n, 0)))
        for n in self._FLOATS:
            setattr(d_, n, float(kw.get(n, 1.0)))
        self._keep = [kw.get(n) for n in self._TENSORS]
        for n in self._TENSORS:
            t = kw.get(n)
            setattr(d_, n, None if t is None else t.data_ptr())
        x = kw["x"]
        self.y = torch.empty_like(x)
        d_.y = self.y.data_ptr()
        nbytes = lib.sa_layer_workspace_bytes(ctypes.byref(d_))
        if nbytes == 0:
            _check(lib.sa_layer_forward(ctypes.byref(d_), _stream()))    # raises with the reason
        self.ws = _workspace(nbytes, x.device)
        d_.workspace = self.ws.data_ptr()
        d_.workspace_bytes = self.ws.numel()
        self.desc = d_

    def forward(self):
        _check(load_library().sa_layer_forward(ctypes.byref(self.desc), _stream()))
        return self.y
