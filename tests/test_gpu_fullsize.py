"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times.

The oracle cannot run the whole of configs 2-5 in seconds, so it recomputes sampled outputs:
whole batch elements for attention (batch elements are independent), sampled token rows for
the MLP (rows are independent once the routing decision is known), plus properties that hold
at any size.
"""
import dataclasses

import numpy as np
import pytest

import oracle
from helpers import ATTN_ATOL, ATTN_RTOL, assert_close, dev, host
from paper_2306_06446_amd import workloads as wl
from test_gpu_parity import _block_inputs, check_block_output, run_block

pytestmark = pytest.mark.gpu


def _attention_oracle_for_batches(cfg, inputs, batches):
    q, k, v, pr, scale, _, _ = inputs
    out = {}
    for b in batches:
        sub = dataclasses.replace(cfg, B=1, E=0, hid=0, shift_frac=None)      # attention only
        o, _ = oracle.block_forward(sub, q[b:b + 1], k[b:b + 1], v[b:b + 1], pr, scale, None, None)
        out[b] = o[0]
    return out


def _mlp_oracle_for_tokens(cfg, o_rows, tokens, logits, p):
    """y rows for the sampled tokens from the oracle's own attention rows."""
    x = o_rows.astype(np.float32)
    xq = oracle.quantize_act(x, p.act_inv_scale)
    ref = np.zeros((len(tokens), cfg.E))
    if logits is None:
        y2 = oracle.shift_mlp(xq, p.w1, p.w2, p.requant_scale, p.lut)
        return np.float64(np.float32(p.out_scale)) * y2
    _, expert_of, _, gate = oracle.moe_dispatch(logits[tokens])
    for i in range(len(tokens)):
        if expert_of[i] == 1:
            y2 = oracle.shift_mlp(xq[i:i + 1], p.w1, p.w2, p.requant_scale, p.lut)
            ref[i] = gate[i] * np.float64(np.float32(p.out_scale)) * y2[0]
        else:
            ref[i] = gate[i] * oracle.mult_mlp(x[i:i + 1], None, p.mw1, p.mw2)[0]
    return ref


@pytest.mark.parametrize("cfg,batches", [(wl.C2, [0, 31]), (wl.C4, [0, 17, 63]), (wl.C5, [5])],
                         ids=lambda c: getattr(c, "name", str(c)))
def test_full_size_block_on_sampled_batches(sa, cfg, batches):
    inputs = _block_inputs(cfg)
    q, k, v, pr, scale, p, logits = inputs
    o, y = run_block(sa, cfg, inputs, prepared=cfg.E > 0)
    assert np.isfinite(o).all()
    o_ref = _attention_oracle_for_batches(cfg, inputs, batches)
    for b in batches:
        assert_close(o[b], o_ref[b], ATTN_RTOL, ATTN_ATOL, "attention output, batch %d" % b)
    if cfg.E == 0:
        return
    assert np.isfinite(y).all()
    g = np.random.default_rng([7, cfg.cfg_id])
    for b in batches:
        toks_in_b = np.sort(g.choice(cfg.N, size=48, replace=False))
        tokens = b * cfg.N + toks_in_b
        o_rows = o_ref[b].reshape(cfg.N, cfg.E)[toks_in_b]
        y_ref = _mlp_oracle_for_tokens(cfg, o_rows, tokens, logits, p)
        check_block_output(y[tokens], y_ref)


def test_full_size_codes_bit_exact_on_sampled_batches(sa):
    for cfg, batches in ((wl.C4, [3, 60]), (wl.C5, [7]), (wl.C2, [11])):
        q, k, _ = wl.qkv(cfg)
        pr = wl.proj(cfg)
        codes = host(sa.sa_binarize(dev(k), dev(pr), cfg.nbits)).view(np.uint64)
        for b in batches:
            ref = oracle.binarize(k[b:b + 1], pr, cfg.nbits)
            assert np.array_equal(codes[b:b + 1], ref), (cfg.name, b)


@pytest.mark.parametrize("variant", [0, 1])
@pytest.mark.parametrize("K,N", wl.C3_SHAPES)
def test_config3_shift_linear_full_size_sampled_rows(sa, variant, K, N):
    M = wl.C3_M
    w4 = wl.shift_weights(3, 4 if K == 384 else 5, N, K)
    x = wl.int8_activations(3, M, K, extra=K)
    y = host(sa.sa_shift_linear(dev(x), dev(w4), variant=variant))
    rows = np.unique(np.concatenate([[0, 1, 127, 128, 255, 256, M - 1],
                                     np.random.default_rng(9).choice(M, 96, replace=False)]))
    assert np.array_equal(y[rows], oracle.shift_linear(x[rows], w4))
    # a property that holds for every row: flipping all weight signs negates the output
    y_neg = host(sa.sa_shift_linear(dev(x), dev(w4 ^ np.uint8(0x88)), variant=1))
    assert np.array_equal(y_neg, -y)


def test_config4_dispatch_full_size_properties(sa):
    cfg = wl.C4
    logits = wl.router_logits(cfg)
    perm, eo, cnt, gate = [host(t) for t in sa.sa_moe_dispatch(dev(logits))]
    assert cnt.tolist() == [3782, 8826]
    assert np.array_equal(np.sort(perm), np.arange(cfg.T))
    assert np.all(np.diff(perm[:cnt[0]]) > 0) and np.all(np.diff(perm[cnt[0]:]) > 0)
    assert np.array_equal(eo, (logits[:, 1] > logits[:, 0]).astype(np.int32))
    assert np.all(gate >= 0.5) and np.all(gate < 1.0)


@pytest.mark.parametrize("cfg,batches", [(wl.C4, [0, 41]), (wl.C5, [3])], ids=lambda c: getattr(c, "name", str(c)))
def test_full_size_layer_on_sampled_batches(sa, cfg, batches):
    """The complete block of Eq. 2 at the benchmark shapes, prepared planes as bench.py --layer runs it.
    Batch elements are independent in every step of the layer, so the oracle recomputes whole sampled
    batch elements; the bounds are those of the small-size test (see there for why they are statistical)."""
    from test_gpu_layer import layer_kwargs
    x = wl.layer_input(cfg)
    lp, p, proj, scale = wl.layer_params(cfg), wl.mlp_params(cfg), wl.proj(cfg), wl.attention_scale(cfg)
    y = host(sa.binding.Layer(**layer_kwargs(sa, cfg, x, lp, p, proj, scale, prepared=True)).forward())
    assert np.isfinite(y).all()
    one = dataclasses.replace(cfg, B=1)
    for b in batches:
        rows = slice(b * cfg.N, (b + 1) * cfg.N)
        r = oracle.layer_forward(one, x[rows], lp, p, proj, scale)
        err = float(np.linalg.norm(y[rows] - r["y"]) / np.linalg.norm(r["y"]))
        err_branches = float(np.linalg.norm((y[rows] - x[rows]) - (r["y"] - x[rows])) / np.linalg.norm(r["y"] - x[rows]))
        print("layer %s batch %d: output error %.3g, both branches %.3g" % (cfg.name, b, err, err_branches))
        assert err < 1e-2 and err_branches < 3e-2
