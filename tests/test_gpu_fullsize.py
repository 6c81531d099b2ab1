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


def test_full_size_hamming_pipeline_equals_the_one_unit_kernel(sa):
    """Config-4 attention as bench.py launches it (768 units on 512 workgroups: half of them walk over two units):
    all three output forms bit-identical to the one-unit-per-workgroup kernel, and sampled batch elements
    against the oracle."""
    import torch
    cfg = wl.C4
    q, k, v = wl.qkv(cfg)
    pr, scale, p = wl.proj(cfg), wl.attention_scale(cfg), wl.mlp_params(cfg)
    qc, kc = sa.sa_binarize_pair(dev(q), dev(k), dev(pr), cfg.nbits)
    dv_ = dev(v)
    o2, xq2, xh2 = sa.sa_hamming_attention_fused(qc, kc, dv_, scale, cfg.nbits, p.act_inv_scale, variant=2)
    o0, xq0, xh0 = sa.sa_hamming_attention_fused(qc, kc, dv_, scale, cfg.nbits, p.act_inv_scale, variant=0)
    assert torch.equal(o2, o0) and torch.equal(xq2, xq0) and torch.equal(xh2, xh0)
    got, hq, hk = host(o2), host(qc), host(kc)
    for b in (0, 40, 63):
        ref = oracle.hamming_attention(hq[b:b + 1], hk[b:b + 1], v[b:b + 1], cfg.nbits, scale)
        assert_close(got[b:b + 1], ref, ATTN_RTOL, ATTN_ATOL, "Hamming attention, batch %d" % b)


def test_full_size_moe_linear_on_sampled_tokens(sa):
    """The MoE form of a DeiT-Base attention Linear on all 12608 tokens of config 4 (70 % to the Shift expert):
    the routing of every token, and the outputs of sampled tokens, against the oracle (a token's row depends on
    its own activations and logits only)."""
    T, K, N = wl.C4.T, 768, 768
    g = np.random.default_rng([19, T])
    x = (g.standard_normal((T, K)) * 1.5).astype(np.float32)
    logits = wl.router_logits(wl.C4)
    neg = g.integers(0, 2, size=(N, K), dtype=np.uint8)
    e = g.integers(0, 8, size=(N, K), dtype=np.uint8)
    w4 = wl.pack_w4(neg, e)
    w_half = (g.standard_normal((N, K)) / np.sqrt(K)).astype(np.float16)
    inv, out_scale = 25.0, 1.0 / (128.0 * K)
    y, expert_of, gate = sa.sa_moe_linear(dev(oracle.quantize_act(x, inv)), dev(x.astype(np.float16)), dev(logits), dev(w4),
                                          dev(w_half), out_scale, variant=1, want_routing=True)
    _, expert_ref, counts_ref, gate_ref = oracle.moe_dispatch(logits)
    assert np.array_equal(host(expert_of), expert_ref)
    assert np.allclose(host(gate), gate_ref, rtol=1e-6, atol=0)
    tokens = np.sort(g.choice(T, size=400, replace=False))
    ref = oracle.moe_linear(x[tokens], logits[tokens], w4, w_half, inv, out_scale)
    got = host(y).astype(np.float64)[tokens]
    shift_rows = expert_ref[tokens] == 1
    err = np.abs(got - ref)
    assert shift_rows.any() and (~shift_rows).any()
    assert np.all(err[shift_rows] <= 3e-7 * np.abs(ref[shift_rows]) + 1e-30), "Shift rows: %g" % err[shift_rows].max()
    rms = float(np.sqrt(np.mean(ref[~shift_rows] ** 2)))
    assert np.all(err[~shift_rows] <= 2e-3 * np.abs(ref[~shift_rows]) + 1e-3 * rms), "Mult rows: %g" % err[~shift_rows].max()


def test_full_size_narrow_shift_layer_on_sampled_rows(sa):
    """A stage-1 layer of a pyramid ViT at batch 32 (100352 rows, K = 32: half a 64-byte stage, the padded last
    stage of the matrix-core variants): sampled rows, the first and the last ones included, bit-exact."""
    M, K, N = 100352, 32, 256
    w4 = wl.shift_weights(3, 8, N, K)
    x = wl.int8_activations(3, M, K, extra=8)
    rows = np.unique(np.concatenate([np.arange(300), np.arange(M - 300, M), np.random.default_rng(4).choice(M, 2000, replace=False)]))
    ref = oracle.shift_linear(x[rows], w4)
    for variant, w in ((1, dev(w4)), (3, sa.sa_shift_planes_prepare(dev(w4)))):
        got = host(sa.sa_shift_linear(dev(x), w, variant=variant))
        assert np.array_equal(got[rows], ref), variant
