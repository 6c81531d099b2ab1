"""Pins of the CPU oracle's shift-layer, quantisation, routing and expert functions (no GPU)."""
import math

import numpy as np
import pytest
import torch

import oracle
from paper_2306_06446_amd import workloads as wl


def decode_raw(neg, e):
    """Test-local decode from the UNPACKED draws: W = s * 2^e as int64."""
    return np.where(neg == 1, -1, 1).astype(np.int64) * (np.int64(1) << e.astype(np.int64))


# ------------------------------------------------------------- shift layer ---

@pytest.mark.parametrize("M,K,N", [(5, 16, 7), (33, 384, 40), (12, 1536, 9)])
def test_shift_linear_equals_integer_matmul_with_decoded_weights(M, K, N):
    neg, e = wl.shift_weight_raw(3, 4, N, K)
    w4 = wl.pack_w4(neg, e)
    assert w4.shape == (N, K // 2)
    x = wl.int8_activations(3, M, K)
    y = oracle.shift_linear(x, w4)
    ref = x.astype(np.int64) @ decode_raw(neg, e).T
    assert np.array_equal(y.astype(np.int64), ref)


def test_shift_linear_nibble_order_by_one_hot_rows():
    """x = unit vectors: row k of Y is column k of the decoded weights, so the
    low nibble must be the even k."""
    K, N = 8, 3
    nib = np.array([[0x0, 0x9, 0x2, 0xB, 0x4, 0xD, 0x6, 0xF],
                    [0x7, 0x8, 0x1, 0xA, 0x3, 0xC, 0x5, 0xE],
                    [0xF, 0x0, 0xF, 0x0, 0x8, 0x7, 0x8, 0x7]], dtype=np.uint8)
    w4 = (nib[:, 0::2] | (nib[:, 1::2] << 4)).astype(np.uint8)
    x = np.eye(K, dtype=np.int8)
    y = oracle.shift_linear(x, w4)
    expect = np.where(nib & 8, -1, 1) * (1 << (nib & 7).astype(np.int64))
    assert np.array_equal(y, expect.T)
    assert y[1, 0] == -2 and y[7, 0] == -128 and y[0, 1] == 128 and y[0, 0] == 1


def test_shift_linear_special_cases():
    M, K, N = 6, 64, 5
    x = wl.int8_activations(3, M, K, extra=1)
    rows = x.astype(np.int64).sum(axis=1, keepdims=True)
    w_plus0 = np.zeros((N, K // 2), dtype=np.uint8)                 # s=+1, e=0
    assert np.array_equal(oracle.shift_linear(x, w_plus0), np.tile(rows, (1, N)))
    w_plus7 = np.full((N, K // 2), 0x77, dtype=np.uint8)            # s=+1, e=7
    assert np.array_equal(oracle.shift_linear(x, w_plus7), np.tile(128 * rows, (1, N)))
    w = wl.shift_weights(3, 5, N, K)
    y = oracle.shift_linear(x, w)
    assert np.array_equal(oracle.shift_linear(x, w ^ np.uint8(0x88)), -y)      # flip every sign
    x2 = wl.int8_activations(3, M, K, extra=2) // 2
    x1 = x // 2
    assert np.array_equal(oracle.shift_linear((x1 + x2).astype(np.int8), w),
                          oracle.shift_linear(x1.astype(np.int8), w) + oracle.shift_linear(x2.astype(np.int8), w))
    bias = np.arange(N, dtype=np.int32) * 1000 - 7
    assert np.array_equal(oracle.shift_linear(x, w, bias), y + bias[None, :])
    # worst case stays inside int32: |Y| <= 127 * 128 * K
    xmax = np.full((1, 3072), 127, dtype=np.int8)
    wmax = np.full((2, 1536), 0x77, dtype=np.uint8)
    assert oracle.shift_linear(xmax, wmax)[0, 0] == 127 * 128 * 3072


# ------------------------------------------------------------ quantisation ---

def test_quantize_act_rounding_and_clamp():
    x = np.array([0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 126.5, 127.5, 300.0, -127.5, -1e9, 3.0, -0.0,
                  np.nan, np.inf, -np.inf], dtype=np.float32)
    q = oracle.quantize_act(x, 1.0)
    assert q.tolist() == [0, 2, 2, 0, -2, -2, 126, 127, 127, -127, -127, 3, 0, 0, 127, -127]
    ints = np.arange(-127, 128, dtype=np.float32)
    assert np.array_equal(oracle.quantize_act(ints, 1.0), ints.astype(np.int8))
    g = np.random.default_rng(1).standard_normal(4096).astype(np.float32)
    s = np.float32(31.75)
    ref = np.clip(np.rint(g * s), -127, 127).astype(np.int8)     # numpy rint = half to even
    assert np.array_equal(oracle.quantize_act(g, float(s)), ref)


def test_requant_lut():
    lut = wl.activation_lut()
    assert lut.shape == (256,) and lut.dtype == np.int8
    y = np.array([0, 1, -1, 1000, -1000, 2**31 - 1, -2**31, 48, 80, 16777217], dtype=np.int32)
    s = np.float32(1 / 32)
    t = np.clip(np.rint(y.astype(np.float32) * s), -127, 127).astype(np.int64)
    assert np.array_equal(oracle.requant_lut(y, float(s), lut), lut[t + 128])
    ident = np.arange(-128, 128).astype(np.int8)
    assert oracle.requant_lut(np.array([48, 80], np.int32), float(s), ident).tolist() == [2, 2]
    # table shape: ~identity for large positive codes, ~0 for large negative, 0 at 0
    assert lut[128] == 0 and lut[128 + 127] == 127 and lut[128 - 127] == 0 and lut[128 + 32] == 27


# ----------------------------------------------------------------- routing ---

def test_moe_dispatch_invariants_and_ties():
    T = 1000
    logits = wl.random_logits(1, T, tie_every=7)
    perm, expert_of, counts, gate = oracle.moe_dispatch(logits)
    assert np.array_equal(np.sort(perm), np.arange(T))
    assert counts.sum() == T
    assert counts[1] == int((logits[:, 1] > logits[:, 0]).sum())
    assert np.array_equal(expert_of, (logits[:, 1] > logits[:, 0]).astype(np.int32))
    assert np.all(expert_of[::7] == 0)                         # ties go to the Mult expert
    c0 = counts[0]
    assert np.all(np.diff(perm[:c0]) > 0) and np.all(np.diff(perm[c0:]) > 0)
    assert np.all(expert_of[perm[:c0]] == 0) and np.all(expert_of[perm[c0:]] == 1)
    ref = torch.softmax(torch.from_numpy(logits.astype(np.float64)), dim=1).max(dim=1).values.numpy()
    np.testing.assert_allclose(gate, ref, rtol=1e-14)
    assert np.all(gate >= 0.5) and np.all(gate < 1.0)
    _, _, _, gate_swapped = oracle.moe_dispatch(np.ascontiguousarray(logits[:, ::-1]))
    np.testing.assert_allclose(gate_swapped, gate, rtol=1e-15)


@pytest.mark.parametrize("cfg", [wl.C1, wl.C4])
def test_router_recipe_gives_the_stated_split(cfg):
    logits = wl.router_logits(cfg)
    _, expert_of, counts, _ = oracle.moe_dispatch(logits)
    n_shift = int(math.floor(cfg.shift_frac * cfg.T + 0.5))
    assert counts.tolist() == [cfg.T - n_shift, n_shift]
    assert np.all(logits[:, 0] != logits[:, 1])
    assert {1: (98, 99), 4: (3782, 8826)}[cfg.cfg_id] == tuple(counts.tolist())


# ------------------------------------------------------------ Mult expert ----

def test_round_to_half_matches_ieee_binary16():
    g = np.random.default_rng(2)
    x = np.concatenate([g.standard_normal(20000) * 10.0 ** g.uniform(-9, 5, 20000),
                        [0.0, 65504.0, 65519.9, 65520.0, 1e6, -1e6, 2.0 ** -24, 2.0 ** -25,
                         1.5 * 2.0 ** -25, 2.0 ** -14, 1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11]])
    with np.errstate(over="ignore"):
        ref = x.astype(np.float16).astype(np.float64)
    assert np.array_equal(oracle.round_to_half(x), ref)


def test_mult_mlp_equals_dense_fp64_mlp_on_half_rounded_operands():
    E, hid, T = 24, 40, 9
    g = np.random.default_rng(3)
    x = g.standard_normal((T, E)).astype(np.float32)
    w1 = (g.standard_normal((hid, E)) / math.sqrt(E)).astype(np.float16)
    w2 = (g.standard_normal((E, hid)) / math.sqrt(hid)).astype(np.float16)
    rows = np.array([8, 0, 3], dtype=np.int32)
    y = oracle.mult_mlp(x, rows, w1, w2)
    tx = torch.from_numpy(x[rows].astype(np.float16).astype(np.float64))
    h = torch.nn.functional.gelu(tx @ torch.from_numpy(w1.astype(np.float64)).T)     # erf GELU
    h = h.numpy().astype(np.float16).astype(np.float64)
    ref = h @ w2.astype(np.float64).T
    np.testing.assert_allclose(y, ref, rtol=1e-12, atol=1e-13)
    assert y.shape == (3, E)
    np.testing.assert_allclose(oracle.mult_mlp(x, None, w1, w2)[rows], y, rtol=1e-15)


def test_combine_scatters_gated_rows():
    T, E = 7, 3
    g = np.random.default_rng(4)
    out = g.standard_normal((T, E))
    perm = np.array([1, 4, 6, 0, 2, 3, 5], dtype=np.int32)
    gate = g.uniform(0.5, 1.0, T)
    y = oracle.combine(out, perm, gate)
    ref = np.zeros((T, E))
    ref[perm] = gate[perm, None] * out
    np.testing.assert_allclose(y, ref, rtol=1e-15)


def test_mlp_stage_composition_all_shift_and_moe():
    """The composed MLP stage equals its parts chained by hand in numpy index arithmetic."""
    cfg = wl.scaled_down(wl.C1, N=23)
    p = wl.mlp_params(cfg)
    x = wl.float_activations(1, cfg.T, cfg.E)
    logits = wl.router_logits(cfg)
    y = oracle.mlp_stage(x, logits, p)
    perm, expert_of, counts, gate = oracle.moe_dispatch(logits)
    xq = oracle.quantize_act(x, p.act_inv_scale)
    for t in range(cfg.T):
        if expert_of[t] == 1:
            y2 = oracle.shift_mlp(xq[t:t + 1], p.w1, p.w2, p.requant_scale, p.lut)
            ref = gate[t] * float(np.float32(p.out_scale)) * y2[0].astype(np.float64)
        else:
            ref = gate[t] * oracle.mult_mlp(x[t:t + 1], None, p.mw1, p.mw2)[0]
        np.testing.assert_allclose(y[t], ref, rtol=1e-13, atol=1e-15)
    y_all = oracle.mlp_stage(x, None, p)
    y2 = oracle.shift_mlp(xq, p.w1, p.w2, p.requant_scale, p.lut)
    np.testing.assert_allclose(y_all, float(np.float32(p.out_scale)) * y2, rtol=1e-15)


# ------------------------------------------ dense weights -> shift weights ---

def unpack_nibbles(w4):
    nib = np.empty((w4.shape[0], w4.shape[1] * 2), dtype=np.uint8)
    nib[:, 0::2] = w4 & 15
    nib[:, 1::2] = w4 >> 4
    return nib


def test_shift_weights_from_float_powers_of_two_round_trip():
    """W = +-2^p, p in [-7, 0], converts to exactly (sign, p) and decodes back to W * 2^7."""
    p = np.arange(-7, 1)
    w = np.concatenate([np.exp2(p), -np.exp2(p)]).astype(np.float32)[None]
    nib = unpack_nibbles(oracle.shift_weights_from_float(w))[0]
    assert np.array_equal(nib & 7, np.concatenate([p + 7, p + 7]))
    assert np.array_equal(nib >> 3, np.concatenate([np.zeros(8), np.ones(8)]))
    x = np.eye(16, dtype=np.int8)
    y = oracle.shift_linear(x, oracle.shift_weights_from_float(w))
    assert np.array_equal(y[:, 0], (w[0] * 128).astype(np.int32))


def test_shift_weights_from_float_rounds_log2_at_sqrt2_and_clamps():
    lo, hi = np.float32(1.41421354), np.float32(1.41421366)        # the fp32 neighbours of sqrt(2)
    assert float(lo) ** 2 < 2.0 < float(hi) ** 2
    w = np.array([[0.25 * lo, 0.25 * hi, 0.3, 0.4, 0.7, 0.71, 1.0, 1.5, 3.0, 1e-3, 0.0, -0.0,
                   -0.25 * lo, -0.25 * hi, 2.0**-7.6, np.inf]], dtype=np.float32)
    nib = unpack_nibbles(oracle.shift_weights_from_float(w))[0]
    expect_p = np.array([-2, -1, -2, -1, -1, 0, 0, 0, 0, -7, -7, -7, -2, -1, -7, 0])
    assert np.array_equal((nib & 7).astype(int) - 7, expect_p)
    assert np.array_equal(nib >> 3, np.array([0] * 12 + [1, 1, 0, 0]))


def test_shift_weights_from_float_equals_library_log2_rounding():
    g = np.random.default_rng(61)
    w = (g.standard_normal((64, 256)) * 0.2).astype(np.float32)
    nib = unpack_nibbles(oracle.shift_weights_from_float(w))
    p_ref = np.clip(np.rint(np.log2(np.abs(w.astype(np.float64)))), -7, 0).astype(int)
    assert np.array_equal((nib & 7).astype(int) - 7, p_ref)
    assert np.array_equal(nib >> 3, (w < 0).astype(np.uint8))
    inside = (np.abs(w) > 2.0**-7) & (np.abs(w) < 1.0)
    assert np.all(np.abs(np.log2(np.abs(w[inside])) - p_ref[inside]) <= 0.5)


# ---------------------------------------- latency-aware balancing loss (Eq. 4) ---

def test_balance_loss_closed_forms():
    # equal logits, equal alpha: every expert gets T/2 of both sums -> both losses 0
    logits = np.zeros((100, 2), dtype=np.float32)
    losses, sums = oracle.moe_balance_loss(logits, np.array([0.5, 0.5], np.float32), 0.1)
    assert np.allclose(sums, 25.0) and np.allclose(losses, 0.0, atol=1e-30)
    # everything on expert 0 with certainty: the vector is (a T, 0): mean a T / 2, variance (a T / 2)^2 -> SCV 1
    logits = np.tile(np.array([[40.0, -40.0]], np.float32), (64, 1))
    losses, sums = oracle.moe_balance_loss(logits, np.array([0.3, 0.7], np.float32), 0.01)
    assert np.allclose(sums[:, 0], 0.3 * 64, rtol=1e-6) and np.allclose(sums[:, 1], 0.0, atol=1e-12)
    assert np.allclose(losses, 1.0, rtol=1e-6)
    # latency-aware optimum: loads inversely proportional to alpha make the weighted vector flat -> loss 0
    # 70 tokens certain for expert 1 (alpha 0.3), 30 certain for expert 0 (alpha 0.7)
    logits = np.concatenate([np.tile([[-40.0, 40.0]], (70, 1)), np.tile([[40.0, -40.0]], (30, 1))]).astype(np.float32)
    losses, sums = oracle.moe_balance_loss(logits, np.array([0.7, 0.3], np.float32), 0.01)
    assert np.allclose(sums, 21.0, rtol=1e-6) and np.allclose(losses, 0.0, atol=1e-10)


def test_balance_loss_equals_direct_formulas():
    g = np.random.default_rng(63)
    T, E = 500, 4
    logits = g.standard_normal((T, E)).astype(np.float32)
    alpha = np.array([0.4, 0.3, 0.2, 0.1], np.float32)
    sigma = 0.05
    losses, sums = oracle.moe_balance_loss(logits, alpha, sigma)
    p = torch.softmax(torch.from_numpy(logits).double(), dim=1).numpy()
    other = np.stack([np.delete(p, e, axis=1).max(axis=1) for e in range(E)], axis=1)
    q = np.array([[0.5 * (1.0 + math.erf((p[t, e] - other[t, e]) / sigma / math.sqrt(2.0))) for e in range(E)]
                  for t in range(T)])
    imp, load = alpha.astype(np.float64) * p.sum(axis=0), alpha.astype(np.float64) * q.sum(axis=0)
    assert np.allclose(sums[0], imp, rtol=1e-12) and np.allclose(sums[1], load, rtol=1e-10)
    assert np.allclose(losses, [np.var(imp) / np.mean(imp) ** 2, np.var(load) / np.mean(load) ** 2], rtol=1e-10)
    # with tiny noise the load is the top-1 count
    _, sums0 = oracle.moe_balance_loss(logits, np.ones(E, np.float32), 1e-9)
    assert np.allclose(sums0[1], np.bincount(p.argmax(axis=1), minlength=E), atol=1e-6)
