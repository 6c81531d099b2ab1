"""Pins of the CPU oracle's whole-layer functions (Eq. 2: LayerNorm, attention Linears as shift
layers, residuals, router) against library routines, closed forms and an independent dense
reconstruction of the layer in fp64 torch (no GPU)."""
import dataclasses
import math
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
from paper_2306_06446_amd import workloads as wl


# ---------------------------------------------------------------- LayerNorm ---

@pytest.mark.parametrize("T,E", [(7, 64), (3, 192), (5, 768)])
def test_layernorm_equals_library_layer_norm_in_fp64(T, E):
    g = np.random.default_rng([41, T, E])
    x = (g.standard_normal((T, E)) * 3.0 + 1.5).astype(np.float32)
    gamma = g.standard_normal(E).astype(np.float32)
    beta = g.standard_normal(E).astype(np.float32)
    y = oracle.layernorm(x, gamma, beta, 1e-6)
    ref = torch.nn.functional.layer_norm(torch.from_numpy(x).double(), (E,), torch.from_numpy(gamma).double(),
                                         torch.from_numpy(beta).double(), 1e-6).numpy()
    assert np.allclose(y, ref, rtol=1e-12, atol=1e-12)


def test_layernorm_rows_have_zero_mean_and_unit_variance():
    g = np.random.default_rng(42)
    x = (g.standard_normal((9, 256)) * 7.0 - 2.0).astype(np.float32)
    y = oracle.layernorm(x, np.ones(256, np.float32), np.zeros(256, np.float32), 0.0)
    assert np.allclose(y.mean(axis=1), 0.0, atol=1e-12)
    assert np.allclose((y * y).mean(axis=1), 1.0, rtol=1e-12)


def test_layernorm_is_invariant_to_shift_and_positive_power_of_two_scale():
    g = np.random.default_rng(43)
    x = g.standard_normal((4, 128)).astype(np.float32)
    gamma = g.standard_normal(128).astype(np.float32)
    beta = g.standard_normal(128).astype(np.float32)
    a = oracle.layernorm(x, gamma, beta, 0.0)
    b = oracle.layernorm(x * np.float32(8.0), gamma, beta, 0.0)        # exact in fp32
    assert np.allclose(a, b, rtol=1e-12, atol=1e-12)
    c = oracle.layernorm(-x, gamma, np.zeros(128, np.float32), 0.0)
    a0 = oracle.layernorm(x, gamma, np.zeros(128, np.float32), 0.0)
    assert np.allclose(c, -a0, rtol=1e-12, atol=1e-12)


def test_layernorm_constant_row_gives_beta_and_eps_enters_under_the_root():
    beta = np.arange(64, dtype=np.float32)
    y = oracle.layernorm(np.full((1, 64), 3.25, np.float32), np.ones(64, np.float32), beta, 1e-6)
    assert np.array_equal(y[0], beta.astype(np.float64))
    # two-valued row +-1: mean 0, var 1 -> y = x / sqrt(1 + eps)
    x = np.tile(np.array([1.0, -1.0], np.float32), 32)[None]
    y = oracle.layernorm(x, np.ones(64, np.float32), np.zeros(64, np.float32), 3.0)
    assert np.allclose(y, x / 2.0, rtol=1e-15)


# --------------------------------------------- dequantised shift Linear output ---

def test_dequant_is_one_fused_multiply_add():
    """A case where multiply-then-add and the fused form differ: the product
    (2^24 - 1)(1 + 2^-23) = 2^24 + 1 - 2^-23 rounds to 2^24 on its own."""
    acc = np.array([16777215], dtype=np.int32)
    scale = np.float32(1.0 + 2.0**-23)
    res = np.array([-16777216.0], dtype=np.float32)
    y = oracle.dequant_residual(acc, scale, res)
    assert y[0] == np.float32(1.0 - 2.0**-23)
    assert np.float32(np.float32(acc[0]) * scale) + res[0] == 0.0      # what the unfused form gives


def test_dequant_rounds_the_exact_value_once():
    g = np.random.default_rng(44)
    acc = g.integers(-(2**24) + 1, 2**24, size=400, dtype=np.int64).astype(np.int32)   # exactly fp32
    scale = np.float32(3.1e-5)
    res = g.standard_normal(400).astype(np.float32)
    y = oracle.dequant_residual(acc, scale, res)
    for i in range(400):
        exact = Fraction(int(acc[i])) * Fraction(float(scale)) + Fraction(float(res[i]))
        lo, hi = np.nextafter(y[i], np.float32(-np.inf)), np.nextafter(y[i], np.float32(np.inf))
        assert abs(Fraction(float(y[i])) - exact) <= abs(Fraction(float(lo)) - exact)
        assert abs(Fraction(float(y[i])) - exact) <= abs(Fraction(float(hi)) - exact)


def test_dequant_large_accumulators_are_rounded_to_fp32_first_and_no_residual_means_zero():
    acc = np.array([2**24 + 1, -(2**24) - 3, 2**30 + 64], dtype=np.int32)
    y = oracle.dequant_residual(acc, np.float32(1.0))
    assert np.array_equal(y, acc.astype(np.float32))                   # numpy converts round-to-nearest-even
    assert y[0] == 2.0**24 and y[1] == -(2.0**24) - 4.0


# ------------------------------------------------------------------- router ---

def test_router_logits_equal_a_dense_matmul():
    g = np.random.default_rng(45)
    z = g.standard_normal((33, 192))
    wg = g.standard_normal((192, 2)).astype(np.float32)
    bg = np.array([0.25, -1.5], dtype=np.float32)
    got = oracle.router_logits(z, wg, bg)
    assert np.allclose(got, z @ wg.astype(np.float64) + bg.astype(np.float64), rtol=1e-13, atol=1e-13)
    e = np.zeros((1, 192)); e[0, 5] = 1.0
    assert np.array_equal(oracle.router_logits(e, wg, np.zeros(2, np.float32))[0], wg[5].astype(np.float64))


# -------------------------------------------------- the layer, reconstructed ---

def dense_weight(w4):
    """Test-local decode of packed 4-bit rows to fp64 [N, K]."""
    nib = np.empty((w4.shape[0], w4.shape[1] * 2), dtype=np.uint8)
    nib[:, 0::2] = w4 & 15
    nib[:, 1::2] = w4 >> 4
    return np.where(nib & 8, -1.0, 1.0) * np.exp2((nib & 7).astype(np.float64))


def unpack_pm1(codes, nbits):
    """[B,H,N,W] uint64 -> [B,H,N,nbits] of +-1.0."""
    bits = ((codes[..., :, None] >> np.arange(64, dtype=np.uint64)) & np.uint64(1)).reshape(codes.shape[:-1] + (nbits,))
    return bits.astype(np.float64) * 2.0 - 1.0


def quant(x32, inv):
    t = (x32.astype(np.float32) * np.float32(inv)).astype(np.float32)
    return np.clip(np.rint(t), -127, 127)


def dense_layer(cfg, x, lp, p, proj, scale):
    """The layer of Eq. 2 written with dense fp64 library ops only (torch / numpy), sharing no
    code with the oracle: decoded weight matrices, +-1 code matrices, softmax, layer_norm."""
    T, E = x.shape
    B, N, H, d = cfg.B, cfg.N, cfg.H, cfg.E // cfg.H
    tx = torch.from_numpy(x).double()

    def ln(t, gamma, beta):
        return torch.nn.functional.layer_norm(t, (E,), torch.from_numpy(gamma).double(),
                                              torch.from_numpy(beta).double(), lp.eps).numpy()

    def lin(xq, w4, s, res=None):
        acc = xq @ dense_weight(w4).T                                  # exact integers in fp64
        y = acc.astype(np.float32).astype(np.float64) * np.float64(np.float32(s))
        if res is not None:
            y = y + res.astype(np.float64)
        return y.astype(np.float32)

    z1q = quant(ln(tx, lp.gamma1, lp.beta1), lp.ln_inv_scale)
    q, k, v = (lin(z1q, w, lp.qkv_scale).reshape(B, N, H, d) for w in (lp.wq, lp.wk, lp.wv))
    if proj is None:
        sq, sk = np.where(q >= 0, 1.0, -1.0), np.where(k >= 0, 1.0, -1.0)
    else:
        sq = np.where(q.astype(np.float64) @ proj.astype(np.float64) >= 0, 1.0, -1.0)
        sk = np.where(k.astype(np.float64) @ proj.astype(np.float64) >= 0, 1.0, -1.0)
    sq, sk, vv = (torch.from_numpy(np.ascontiguousarray(a.transpose(0, 2, 1, 3))).double() for a in (sq, sk, v))
    s = np.float64(np.float32(scale))
    if cfg.attention == "linear":
        o = s * (sq @ (sk.transpose(-1, -2) @ vv))
    else:
        o = torch.softmax(s * (sq @ sk.transpose(-1, -2)), dim=-1) @ vv
    o = o.permute(0, 2, 1, 3).reshape(T, E).numpy()
    x1 = lin(quant(o, p.act_inv_scale), lp.wo, lp.o_scale, x)
    z2 = ln(torch.from_numpy(x1).double(), lp.gamma2, lp.beta2)
    z2_32 = z2.astype(np.float32)

    def shift_expert(rows):
        h1 = quant(z2_32[rows], lp.ln_inv_scale) @ dense_weight(p.w1).T
        hq = np.clip(np.rint((h1.astype(np.float32) * np.float32(p.requant_scale)).astype(np.float32)), -127, 127)
        h = p.lut.astype(np.float64)[hq.astype(np.int64) + 128]
        return np.float64(np.float32(p.out_scale)) * (h @ dense_weight(p.w2).T)

    def mult_expert(rows):
        xh = torch.from_numpy(z2_32[rows]).half().double()
        hpre = xh @ torch.from_numpy(p.mw1).double().T
        hact = (0.5 * hpre * (1.0 + torch.erf(hpre / math.sqrt(2.0)))).half().double()
        return (hact @ torch.from_numpy(p.mw2).double().T).numpy()

    if lp.wg is None:
        mlp = shift_expert(np.arange(T))
    else:
        logits = (z2 @ lp.wg.astype(np.float64) + lp.bg.astype(np.float64)).astype(np.float32)
        to_shift = logits[:, 1] > logits[:, 0]
        gate = torch.softmax(torch.from_numpy(logits).double(), dim=1).numpy().max(axis=1)
        mlp = np.zeros((T, E))
        mlp[to_shift] = shift_expert(np.nonzero(to_shift)[0])
        mlp[~to_shift] = mult_expert(np.nonzero(~to_shift)[0])
        mlp *= gate[:, None]
    return x1, x1.astype(np.float64) + mlp


@pytest.mark.parametrize("attention,moe,use_proj", [("hamming", True, True), ("linear", False, True),
                                                      ("hamming", False, False)])
def test_layer_equals_an_independent_dense_reconstruction(attention, moe, use_proj):
    nbits = 128 if use_proj else 64
    cfg = wl.BlockConfig(7, "tiny-layer", 2, 24, 2, 64, nbits, 64, attention, 128, 256, 0.6 if moe else None)
    x = wl.layer_input(cfg)
    lp = wl.layer_params(cfg)
    p = wl.mlp_params(cfg)
    proj = wl.proj(cfg) if use_proj else None
    scale = wl.attention_scale(cfg)
    r = oracle.layer_forward(cfg, x, lp, p, proj, scale)
    x1, y = dense_layer(cfg, x, lp, p, proj, scale)
    assert np.allclose(r["x1"], x1, rtol=1e-6, atol=1e-6)
    assert np.allclose(r["y"], y, rtol=1e-6, atol=1e-6)
    # the pieces are not trivial: residuals, attention and MLP all contribute
    assert np.abs(r["x1"] - x).std() > 0.1 and np.abs(r["mlp"]).std() > 0.05
    if moe:
        n_shift = int((r["logits"][:, 1] > r["logits"][:, 0]).sum())
        assert 0 < n_shift < cfg.T


def test_layer_reduces_to_the_input_when_both_branches_are_scaled_to_zero():
    cfg = wl.BlockConfig(7, "tiny-layer", 1, 16, 2, 64, 64, 64, "linear", 128, 256, None)
    x = wl.layer_input(cfg)
    lp = dataclasses.replace(wl.layer_params(cfg), o_scale=0.0)
    p = dataclasses.replace(wl.mlp_params(cfg), out_scale=0.0)
    r = oracle.layer_forward(cfg, x, lp, p, None, wl.attention_scale(cfg))
    assert np.array_equal(r["x1"], x) and np.array_equal(r["y"], x.astype(np.float64))
