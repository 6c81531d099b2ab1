"""Pins of oracle.moe_linear, the MoE form of a Linear layer (Sec. 4.1 and 4.2), against things it does not
compute itself: a token-by-token evaluation in plain Python integers and fractions, and the two degenerate
routings, where the layer is a plain dense layer or a plain shift layer times the gate."""
from fractions import Fraction

import numpy as np

import oracle
from paper_2306_06446_amd import workloads as wl


def _case(seed, T, K, N):
    g = np.random.default_rng([91, seed])
    x = (g.standard_normal((T, K)) * 3).astype(np.float32)
    logits = g.standard_normal((T, 2)).astype(np.float32)
    neg = g.integers(0, 2, size=(N, K), dtype=np.uint8)
    e = g.integers(0, 8, size=(N, K), dtype=np.uint8)
    w4 = wl.pack_w4(neg, e)
    w_half = (g.standard_normal((N, K)) / 8).astype(np.float16)
    return x, logits, neg, e, w4, w_half


def test_moe_linear_token_by_token_in_exact_arithmetic():
    T, K, N = 9, 32, 5
    x, logits, neg, e, w4, w_half = _case(0, T, K, N)
    logits[3] = [0.25, 0.25]                      # a tie goes to expert 0
    inv, out_scale = np.float32(7.5), np.float32(0.013)
    got = oracle.moe_linear(x, logits, w4, w_half, inv, out_scale)
    for t in range(T):
        l0, l1 = float(logits[t, 0]), float(logits[t, 1])
        expert = 1 if l1 > l0 else 0
        p = np.exp(np.array([l0, l1]) - max(l0, l1))
        gate = p[expert] / p.sum()
        for n in range(N):
            if expert == 0:
                acc = sum(Fraction(float(np.float16(x[t, k]))) * Fraction(float(w_half[n, k])) for k in range(K))
            else:
                total = 0
                for k in range(K):
                    v = float(np.float32(x[t, k]) * inv)
                    code = int(max(-127, min(127, np.rint(v))))
                    total += (-1 if neg[n, k] else 1) * (code << int(e[n, k]))
                acc = Fraction(float(out_scale)) * total
            want = gate * float(acc)
            assert abs(got[t, n] - want) <= 1e-12 * max(1.0, abs(want)), (t, n, got[t, n], want)


def test_moe_linear_degenerate_routings_are_the_plain_layers():
    T, K, N = 40, 64, 24
    x, logits, _, _, w4, w_half = _case(1, T, K, N)
    inv, out_scale = 9.0, 0.02
    to_mult = np.tile(np.array([[30.0, -30.0]], dtype=np.float32), (T, 1))     # gate = 1 / (1 + e^-60) = 1 in fp64
    y = oracle.moe_linear(x, to_mult, w4, w_half, inv, out_scale)
    dense = x.astype(np.float16).astype(np.float64) @ w_half.astype(np.float64).T
    assert np.allclose(y, dense, rtol=1e-13, atol=1e-13)
    to_shift = to_mult[:, ::-1].copy()
    y = oracle.moe_linear(x, to_shift, w4, w_half, inv, out_scale)
    shift = np.float64(np.float32(out_scale)) * oracle.shift_linear(oracle.quantize_act(x, inv), w4).astype(np.float64)
    assert np.allclose(y, shift, rtol=1e-13, atol=0)
    # mixed routing: every row is one of the two, scaled by a gate in (0.5, 1]
    y = oracle.moe_linear(x, logits, w4, w_half, inv, out_scale)
    _, expert_of, counts, gate = oracle.moe_dispatch(logits)
    assert counts.sum() == T and 0 < counts[0] < T
    assert np.all((gate > 0.5 - 1e-12) & (gate <= 1.0))
    assert np.allclose(y[expert_of == 0], gate[expert_of == 0, None] * dense[expert_of == 0], rtol=1e-13, atol=1e-13)
    assert np.allclose(y[expert_of == 1], gate[expert_of == 1, None] * shift[expert_of == 1], rtol=1e-13, atol=0)
