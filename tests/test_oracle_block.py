"""Pins of oracle.block_forward, the composition every block-level GPU test and the smoke check compare against
(hash Q and K -> additive or Hamming attention -> activation quantiser -> Shift MLP or top-1 MoE; Sec. 4.1, 4.2,
Eq. 1-3), against an independent dense reconstruction written with fp64 library operations only (no GPU)."""
import dataclasses
import math

import numpy as np
import pytest
import torch

import oracle
from paper_2306_06446_amd import workloads as wl
from test_oracle_layer import dense_weight, quant


def dense_block(cfg, q, k, v, proj, scale, logits, p):
    """The block with decoded +-1 code matrices, decoded weight matrices, torch softmax / erf: shares no code with
    the oracle.  Layouts as at the boundary: q, k [B,N,H,d], v [B,N,H,dv], output rows are [T, H*dv]."""
    B, N, H, dv = cfg.B, cfg.N, cfg.H, cfg.dv
    T = B * N
    pj = None if proj is None else proj.astype(np.float64)

    def signs(x):
        z = x.astype(np.float64) if pj is None else x.astype(np.float64) @ pj
        return torch.from_numpy(np.ascontiguousarray(np.where(z >= 0, 1.0, -1.0).transpose(0, 2, 1, 3)))   # [B,H,N,nbits]

    sq, sk = signs(q), signs(k)
    vv = torch.from_numpy(np.ascontiguousarray(v.transpose(0, 2, 1, 3))).double()                          # [B,H,N,dv]
    s = np.float64(np.float32(scale))
    if cfg.attention == "linear":
        o = s * (sq @ (sk.transpose(-1, -2) @ vv))
    else:
        o = torch.softmax(s * (sq @ sk.transpose(-1, -2)), dim=-1) @ vv
    o = o.permute(0, 2, 1, 3).contiguous().numpy()                                                         # [B,N,H,dv]
    if cfg.E == 0:
        return o, None
    x32 = o.reshape(T, H * dv).astype(np.float32)

    def shift_expert(rows):
        h1 = quant(x32[rows], p.act_inv_scale) @ dense_weight(p.w1).T
        hq = np.clip(np.rint((h1.astype(np.float32) * np.float32(p.requant_scale)).astype(np.float32)), -127, 127)
        h = p.lut.astype(np.float64)[hq.astype(np.int64) + 128]
        return np.float64(np.float32(p.out_scale)) * (h @ dense_weight(p.w2).T)

    def mult_expert(rows):
        xh = torch.from_numpy(x32[rows]).half().double()
        hpre = xh @ torch.from_numpy(p.mw1).double().T
        hact = (0.5 * hpre * (1.0 + torch.erf(hpre / math.sqrt(2.0)))).half().double()
        return (hact @ torch.from_numpy(p.mw2).double().T).numpy()

    if logits is None:
        return o, shift_expert(np.arange(T))
    to_shift = logits[:, 1] > logits[:, 0]
    gate = torch.softmax(torch.from_numpy(logits).double(), dim=1).numpy().max(axis=1)
    y = np.zeros((T, H * dv))
    y[to_shift] = shift_expert(np.nonzero(to_shift)[0])
    y[~to_shift] = mult_expert(np.nonzero(~to_shift)[0])
    return o, y * gate[:, None]


def tiny(attention, moe, nbits, H=2, E=128, hid=256, B=2, N=24):
    return wl.BlockConfig(8, "tiny-block", B, N, H, 64, nbits, E // H, attention, E, hid, 0.6 if moe else None)


def inputs(cfg, use_proj=True):
    q, k, v = wl.qkv(cfg)
    pr = wl.proj(cfg) if use_proj else None
    p = wl.mlp_params(cfg) if cfg.E else None
    logits = wl.router_logits(cfg) if (cfg.E and cfg.shift_frac is not None) else None
    return q, k, v, pr, wl.attention_scale(cfg), logits, p


@pytest.mark.parametrize("attention,moe,nbits,use_proj", [
    ("hamming", True, 128, True),      # the DeiT-Base block in small: projection hash, Hamming attention, MoE
    ("linear", True, 64, True),        # the DeiT-Tiny block in small
    ("linear", False, 256, True),      # the long-sequence block in small: Shift MLP for every token
    ("hamming", False, 64, False),     # sign hash without a projection
])
def test_block_equals_an_independent_dense_reconstruction(attention, moe, nbits, use_proj):
    cfg = tiny(attention, moe, nbits)
    q, k, v, pr, scale, logits, p = inputs(cfg, use_proj)
    o, y = oracle.block_forward(cfg, q, k, v, pr, scale, logits, p)
    o_ref, y_ref = dense_block(cfg, q, k, v, pr, scale, logits, p)
    assert o.shape == (cfg.B, cfg.N, cfg.H, cfg.dv) and y.shape == (cfg.T, cfg.E)
    assert np.allclose(o, o_ref, rtol=1e-9, atol=1e-12)
    assert np.allclose(y, y_ref, rtol=1e-9, atol=1e-12)
    # the comparison has teeth: heads and tokens differ, both stages contribute, both experts are used
    assert np.abs(o[:, :, 0] - o[:, :, 1]).std() > 1e-3 and np.abs(o[0] - o[1]).std() > 1e-3
    assert y.std() > 1e-2
    if moe:
        n_shift = int((logits[:, 1] > logits[:, 0]).sum())
        assert 0 < n_shift < cfg.T


def test_attention_only_block_returns_no_mlp_output():
    cfg = dataclasses.replace(tiny("linear", False, 64, H=1, E=32), E=0, hid=0, d=32, dv=32)
    q, k, v = wl.qkv(cfg)
    pr = wl.proj(cfg)
    o, y = oracle.block_forward(cfg, q, k, v, pr, wl.attention_scale(cfg), None, None)
    o_ref, _ = dense_block(cfg, q, k, v, pr, wl.attention_scale(cfg), None, None)
    assert y is None and np.allclose(o, o_ref, rtol=1e-9, atol=1e-12)


def test_block_output_rows_follow_the_token_major_head_inner_layout():
    """Only head 1 of token (b=1, n=5) has a non-zero V row and all codes are equal (Q = K = all-positive rows), so
    the linear attention output of every token of batch 1 is scale * nbits * that row in head 1's columns, zero
    elsewhere; the MLP input row t = b*N + n, columns h*dv .. h*dv+dv-1, must carry exactly that."""
    cfg = tiny("linear", False, 64, B=2, N=8)
    q = np.ones((cfg.B, cfg.N, cfg.H, cfg.d), np.float32)
    k = np.ones_like(q)
    v = np.zeros((cfg.B, cfg.N, cfg.H, cfg.dv), np.float32)
    row = np.linspace(-2.0, 2.0, cfg.dv).astype(np.float32)
    v[1, 5, 1] = row
    p = wl.mlp_params(cfg)
    scale = 0.01
    o, y = oracle.block_forward(cfg, q, k, v, None, scale, None, p)
    expect = np.zeros_like(o)
    expect[1, :, 1, :] = np.float64(np.float32(scale)) * cfg.nbits * row.astype(np.float64)
    assert np.allclose(o, expect, rtol=1e-12, atol=0)
    x = expect.reshape(cfg.T, cfg.E).astype(np.float32)
    assert np.array_equal(y, oracle.mlp_stage(x, None, p))
    assert np.all(y[: cfg.N] == y[0]) and np.abs(y[cfg.N] - y[0]).max() > 0      # batch 0 saw zeros, batch 1 did not
