"""CPU oracle of the ShiftAddViT block path: ctypes front end of shiftadd_oracle.c.

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  The GPU library never imports or calls it and
it never imports the GPU library.  The arithmetic lives in the C file (plain
loops, fp64 / int64); this module only marshals numpy arrays and chains the
stages in the order of the block (Eq. 2 restricted to attention + MLP/MoE).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "shiftadd_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2 -fopenmp, no fast-math, no contraction)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-ffp-contract=off", "-fno-fast-math", "-std=c11",
             "-shared", "-fPIC", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.oracle_shift_linear.restype = ctypes.c_long
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def num_threads() -> int:
    """Threads the OpenMP loops use (what cpu_baseline reports as cores)."""
    env = os.environ.get("OMP_NUM_THREADS")
    if env:
        return int(env.split(",")[0])
    return len(os.sched_getaffinity(0))


# ------------------------------------------------------------------ stages --

def binarize(x, proj, nbits):
    x = _c(x, np.float32)
    B, N, H, d = x.shape
    if proj is not None:
        proj = _c(proj, np.float32)
        assert proj.shape == (d, nbits)
    else:
        assert nbits == d
    assert nbits % 64 == 0
    codes = np.zeros((B, H, N, nbits // 64), dtype=np.uint64)
    _load().oracle_binarize(_p(x), B, N, H, d, _p(proj), nbits, _p(codes))
    return codes


def ktv(k_codes, v, nbits):
    k_codes = _c(k_codes, np.uint64)
    v = _c(v, np.float32)
    B, H, Nk, W = k_codes.shape
    assert W * 64 == nbits and v.shape[:3] == (B, Nk, H)
    dv = v.shape[3]
    kv = np.zeros((B, H, nbits, dv), dtype=np.float64)
    _load().oracle_ktv(_p(k_codes), _p(v), B, H, Nk, nbits, dv, _p(kv))
    return kv


def qkv(q_codes, kv, scale):
    q_codes = _c(q_codes, np.uint64)
    kv = _c(kv, np.float64)
    B, H, Nq, W = q_codes.shape
    nbits, dv = kv.shape[2], kv.shape[3]
    assert W * 64 == nbits
    out = np.zeros((B, Nq, H, dv), dtype=np.float64)
    _load().oracle_qkv(_p(q_codes), _p(kv), B, H, Nq, nbits, dv, ctypes.c_float(scale), _p(out))
    return out


def additive_attention(q_codes, k_codes, v, nbits, scale):
    kv = ktv(k_codes, v, nbits)
    return qkv(q_codes, kv, scale), kv


def ktv01(k_codes, v, nbits):
    """{0,1}-code K^T V and the per-bit counts of set key bits: (kv fp64 [B,H,nbits,dv], ksum int64 [B,H,nbits])."""
    k_codes = _c(k_codes, np.uint64)
    v = _c(v, np.float32)
    B, H, Nk, W = k_codes.shape
    assert W * 64 == nbits and v.shape[:3] == (B, Nk, H)
    dv = v.shape[3]
    kv = np.zeros((B, H, nbits, dv), dtype=np.float64)
    ksum = np.zeros((B, H, nbits), dtype=np.int64)
    _load().oracle_ktv01(_p(k_codes), _p(v), B, H, Nk, nbits, dv, _p(kv), _p(ksum))
    return kv, ksum


def qkv01(q_codes, kv, ksum, eps):
    """Normalised {0,1}-code Q(K^T V): (out fp64 [B,Nq,H,dv], den int64 [B,H,Nq])."""
    q_codes = _c(q_codes, np.uint64)
    kv = _c(kv, np.float64)
    ksum = _c(ksum, np.int64)
    B, H, Nq, W = q_codes.shape
    nbits, dv = kv.shape[2], kv.shape[3]
    out = np.zeros((B, Nq, H, dv), dtype=np.float64)
    den = np.zeros((B, H, Nq), dtype=np.int64)
    _load().oracle_qkv01(_p(q_codes), _p(kv), _p(ksum), B, H, Nq, nbits, dv, ctypes.c_double(eps), _p(out), _p(den))
    return out, den


def linear_attention_01(q_codes, k_codes, v, nbits, eps):
    kv, ksum = ktv01(k_codes, v, nbits)
    out, den = qkv01(q_codes, kv, ksum, eps)
    return out, kv, ksum, den


def dwconv3x3(v, w, bias=None):
    """v [B,gh,gw,E] fp32, w [E,3,3] fp32, bias [E] or None -> fp64 [B,gh,gw,E]."""
    v = _c(v, np.float32)
    w = _c(w, np.float32)
    B, gh, gw, E = v.shape
    assert w.shape == (E, 3, 3)
    if bias is not None:
        bias = _c(bias, np.float32)
    out = np.zeros((B, gh, gw, E), dtype=np.float64)
    _load().oracle_dwconv3x3(_p(v), _p(w), _p(bias), B, gh, gw, E, _p(out))
    return out


def hamming_scores(q_codes, k_codes, nbits):
    q_codes = _c(q_codes, np.uint64)
    k_codes = _c(k_codes, np.uint64)
    B, H, Nq, W = q_codes.shape
    Nk = k_codes.shape[2]
    s = np.zeros((B, H, Nq, Nk), dtype=np.int16)
    _load().oracle_hamming_scores(_p(q_codes), _p(k_codes), B, H, Nq, Nk, nbits, _p(s))
    return s


def hamming_attention(q_codes, k_codes, v, nbits, scale):
    q_codes = _c(q_codes, np.uint64)
    k_codes = _c(k_codes, np.uint64)
    v = _c(v, np.float32)
    B, H, Nq, W = q_codes.shape
    Nk = k_codes.shape[2]
    dv = v.shape[3]
    out = np.zeros((B, Nq, H, dv), dtype=np.float64)
    _load().oracle_hamming_attention(_p(q_codes), _p(k_codes), _p(v), B, H, Nq, Nk, nbits, dv,
                                     ctypes.c_float(scale), _p(out))
    return out


def shift_linear(x, w4, bias=None):
    x = _c(x, np.int8)
    w4 = _c(w4, np.uint8)
    M, K = x.shape
    N = w4.shape[0]
    assert w4.shape[1] * 2 == K
    if bias is not None:
        bias = _c(bias, np.int32)
    y = np.zeros((M, N), dtype=np.int32)
    ovf = _load().oracle_shift_linear(_p(x), _p(w4), _p(bias), _p(y), ctypes.c_long(M), K, N)
    if ovf:
        raise OverflowError("%d shift-linear outputs do not fit int32" % ovf)
    return y


def shift_weights_from_float(w):
    w = _c(w, np.float32)
    N, K = w.shape
    assert K % 2 == 0
    w4 = np.zeros((N, K // 2), dtype=np.uint8)
    _load().oracle_shift_weights_from_float(_p(w), ctypes.c_long(N), K, _p(w4))
    return w4


def quantize_act(x, inv_scale):
    x = _c(x, np.float32)
    q = np.zeros(x.shape, dtype=np.int8)
    _load().oracle_quantize_act(_p(x), ctypes.c_long(x.size), ctypes.c_float(inv_scale), _p(q))
    return q


def requant_lut(y, s, lut):
    y = _c(y, np.int32)
    lut = _c(lut, np.int8)
    assert lut.size == 256
    h = np.zeros(y.shape, dtype=np.int8)
    _load().oracle_requant_lut(_p(y), ctypes.c_long(y.size), ctypes.c_float(s), _p(lut), _p(h))
    return h


def moe_dispatch(logits):
    logits = _c(logits, np.float32)
    T, E = logits.shape
    perm = np.zeros(T, dtype=np.int32)
    expert_of = np.zeros(T, dtype=np.int32)
    counts = np.zeros(E, dtype=np.int32)
    gate = np.zeros(T, dtype=np.float64)
    _load().oracle_moe_dispatch(_p(logits), ctypes.c_long(T), E, _p(perm), _p(expert_of),
                                _p(counts), _p(gate))
    return perm, expert_of, counts, gate


def moe_balance_loss(logits, alpha, noise_std):
    """Eq. 4 forward: (losses [2] = (L_IMP, L_LOAD), sums [2, E] = alpha-weighted importance and load)."""
    logits = _c(logits, np.float32)
    alpha = _c(alpha, np.float32)
    T, E = logits.shape
    assert alpha.shape == (E,) and E <= 64
    losses = np.zeros(2, dtype=np.float64)
    sums = np.zeros((2, E), dtype=np.float64)
    _load().oracle_moe_balance_loss(_p(logits), ctypes.c_long(T), E, _p(alpha), ctypes.c_double(noise_std),
                                    _p(losses), _p(sums))
    return losses, sums


def mult_mlp(x, rows, w1_half, w2_half):
    x = _c(x, np.float32)
    E = x.shape[1]
    w1 = _c(w1_half, np.float16)
    w2 = _c(w2_half, np.float16)
    hid = w1.shape[0]
    assert w1.shape == (hid, E) and w2.shape == (E, hid)
    if rows is not None:
        rows = _c(rows, np.int32)
        n = rows.size
    else:
        n = x.shape[0]
    y = np.zeros((n, E), dtype=np.float64)
    _load().oracle_mult_mlp(_p(x), _p(rows), ctypes.c_long(n), E, hid,
                            _p(w1.view(np.uint16)), _p(w2.view(np.uint16)), _p(y))
    return y


def round_to_half(x):
    x = _c(x, np.float64)
    r = np.zeros(x.shape, dtype=np.float64)
    _load().oracle_round_to_half(_p(x), ctypes.c_long(x.size), _p(r))
    return r


def combine(expert_out, perm, gate):
    expert_out = _c(expert_out, np.float64)
    perm = _c(perm, np.int32)
    gate = _c(gate, np.float64)
    T, E = expert_out.shape
    y = np.zeros((T, E), dtype=np.float64)
    _load().oracle_combine(_p(expert_out), _p(perm), _p(gate), ctypes.c_long(T), E, _p(y))
    return y


def layernorm(x, gamma, beta, eps):
    x = _c(x, np.float32)
    T, E = x.shape
    gamma = _c(gamma, np.float32)
    beta = _c(beta, np.float32)
    assert gamma.shape == (E,) and beta.shape == (E,)
    y = np.zeros((T, E), dtype=np.float64)
    _load().oracle_layernorm(_p(x), ctypes.c_long(T), E, _p(gamma), _p(beta), ctypes.c_double(eps), _p(y))
    return y


def dequant_residual(acc, scale, residual=None):
    acc = _c(acc, np.int32)
    if residual is not None:
        residual = _c(residual, np.float32)
        assert residual.shape == acc.shape
    y = np.zeros(acc.shape, dtype=np.float32)
    _load().oracle_dequant_residual(_p(acc), ctypes.c_long(acc.size), ctypes.c_float(scale), _p(residual), _p(y))
    return y


def router_logits(z, wg, bg):
    z = _c(z, np.float64)
    wg = _c(wg, np.float32)
    bg = _c(bg, np.float32)
    T, E = z.shape
    n_exp = wg.shape[1]
    assert wg.shape == (E, n_exp) and bg.shape == (n_exp,)
    logits = np.zeros((T, n_exp), dtype=np.float64)
    _load().oracle_router_logits(_p(z), ctypes.c_long(T), E, _p(wg), _p(bg), n_exp, _p(logits))
    return logits


# ------------------------------------------------------------- compositions --

def shift_mlp(xq, w1, w2, requant_scale, lut):
    """Shift expert: shift linear -> requantise + table -> shift linear (int32 out)."""
    y1 = shift_linear(xq, w1)
    h = requant_lut(y1, requant_scale, lut)
    return shift_linear(h, w2)


def mlp_stage(x, logits, p):
    """MLP / MoE half of the block on fp32 rows x [T, E].

    logits None: every token goes through the Shift expert with gate 1.
    Otherwise top-1 dispatch between the Mult expert (0) and the Shift expert (1).
    Returns y [T, E] fp64.
    """
    x = _c(x, np.float32)
    T, E = x.shape
    xq = quantize_act(x, p.act_inv_scale)
    if logits is None:
        y2 = shift_mlp(xq, p.w1, p.w2, p.requant_scale, p.lut)
        return np.float64(np.float32(p.out_scale)) * y2.astype(np.float64)
    perm, expert_of, counts, gate = moe_dispatch(logits)
    c0 = int(counts[0])
    out0 = mult_mlp(x, perm[:c0], p.mw1, p.mw2)
    y2 = shift_mlp(xq[perm[c0:]], p.w1, p.w2, p.requant_scale, p.lut)
    out1 = np.float64(np.float32(p.out_scale)) * y2.astype(np.float64)
    return combine(np.concatenate([out0, out1], axis=0), perm, gate)


def moe_linear(x, logits, w4, w_half, act_inv_scale, out_scale):
    """MoE form of one Linear layer (Sec. 4.1: the Linears of the attention module become Shift layers or MoEs;
    Sec. 4.2: y = sum_i G(x) E_i(x) with one non-zero term).  x [T, K] fp32, logits [T, 2].  Expert 0 multiplies
    (fp16 weights w_half [N, K] times the fp16 rounding of x, exact sums), expert 1 shifts (the int8 codes of
    x * act_inv_scale times the shift weights w4, times out_scale).  Both experts are evaluated for every token and
    the routed one is kept: the definition, not a schedule.  Returns y [T, N] fp64."""
    x = _c(x, np.float32)
    _, expert_of, _, gate = moe_dispatch(logits)
    w = np.asarray(w_half, dtype=np.float16).astype(np.float64)
    y_mult = round_to_half(x.astype(np.float64)) @ w.T
    y_shift = np.float64(np.float32(out_scale)) * shift_linear(quantize_act(x, act_inv_scale), w4).astype(np.float64)
    return gate[:, None] * np.where(expert_of[:, None] == 0, y_mult, y_shift)


def block_forward(cfg, q, k, v, proj, scale, logits, p):
    """binarize -> (additive | Hamming) attention -> MLP / MoE.  Returns (O, y) in fp64."""
    qc = binarize(q, proj, cfg.nbits)
    kc = binarize(k, proj, cfg.nbits)
    if cfg.attention == "linear":
        o, _ = additive_attention(qc, kc, v, cfg.nbits, scale)
    else:
        o = hamming_attention(qc, kc, v, cfg.nbits, scale)
    if cfg.E == 0:
        return o, None
    x = o.reshape(cfg.T, cfg.E).astype(np.float32)
    return o, mlp_stage(x, logits, p)


def layer_forward(cfg, x, lp, p, proj, scale):
    """The whole block of Eq. 2 on tokens x [T, E] fp32.

    LayerNorm -> int8 -> shift Linears Wq, Wk, Wv -> fp32 Q, K, V -> hash -> attention ->
    int8 -> shift Linear Wo + residual -> LayerNorm -> router + MLP / MoE + residual.
    lp holds the attention-side parameters (see workloads.LayerParams), p the MLP's.
    Returns a dict of every intermediate; floats are fp64 except where the definition
    rounds to fp32 (the dequantised Linears), integers are exact.
    """
    x = _c(x, np.float32)
    T, E = x.shape
    B, N, H = cfg.B, cfg.N, cfg.H
    r = {}
    r["ln1"] = layernorm(x, lp.gamma1, lp.beta1, lp.eps)
    r["z1q"] = quantize_act(r["ln1"].astype(np.float32), lp.ln_inv_scale)
    for name, w in (("q", lp.wq), ("k", lp.wk), ("v", lp.wv)):
        r[name] = dequant_residual(shift_linear(r["z1q"], w), lp.qkv_scale)
    q4, k4, v4 = (r[n].reshape(B, N, H, E // H) for n in ("q", "k", "v"))
    r["qc"] = binarize(q4, proj, cfg.nbits)
    r["kc"] = binarize(k4, proj, cfg.nbits)
    if cfg.attention == "linear":
        o, _ = additive_attention(r["qc"], r["kc"], v4, cfg.nbits, scale)
    else:
        o = hamming_attention(r["qc"], r["kc"], v4, cfg.nbits, scale)
    r["o"] = o.reshape(T, E)
    r["oq"] = quantize_act(r["o"].astype(np.float32), p.act_inv_scale)
    r["x1"] = dequant_residual(shift_linear(r["oq"], lp.wo), lp.o_scale, x)
    r["ln2"] = layernorm(r["x1"], lp.gamma2, lp.beta2, lp.eps)
    z2 = r["ln2"].astype(np.float32)
    logits = None
    if lp.wg is not None:
        r["logits"] = router_logits(r["ln2"], lp.wg, lp.bg)
        logits = r["logits"].astype(np.float32)
    p2 = _replace_inv_scale(p, lp.ln_inv_scale)
    r["mlp"] = mlp_stage(z2, logits, p2)
    r["y"] = r["x1"].astype(np.float64) + r["mlp"]
    return r


def _replace_inv_scale(p, inv_scale):
    import dataclasses
    return dataclasses.replace(p, act_inv_scale=inv_scale)
