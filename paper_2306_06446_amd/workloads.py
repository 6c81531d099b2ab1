"""Seeded synthetic inputs for the five benchmark configurations.

This module draws random tensors and lays them out in the boundary's storage
formats.  It holds none of the method's arithmetic (no hashing, no attention,
no shift accumulation, no routing decision): it serves the HIP path, the CPU
oracle and the tests alike and imports neither of the first two.

The shapes stand in for the paper's workloads, whose data sets and trained
weights are not available: 197 = 14*14 + 1 tokens of a 224x224 DeiT, 3136 =
56*56 tokens of a pyramid-ViT first stage (Sec. 5.1, models and data sets),
16384 tokens = the upper end of the long-range benchmark the appendix on NLP
tasks quotes.

Storage formats (identical on both sides of every comparison because they are
the interface, not an implementation detail):

* activations  x, Q, K   fp32  [B, N, H, d]      (token-major, heads inner)
* values       V         fp32  [B, N, H, dv]
* hash matrix  proj      fp32  [d, nbits]        row-major, shared by heads
* shift weight W = s*2^p, p in [-7, 0], stored as nibble (neg << 3) | e with
  e = p + 7; w4[n, k // 2] holds k even in the low nibble, k odd in the high
  nibble; shape [N_out, K // 2] uint8.
* router logits          fp32  [T, 2]            column 0 = Mult, 1 = Shift
* router weight Wg       fp32  [E, 2], bias bg [2]   (whole-layer path: logits = LN2(x) Wg + bg)
"""
from __future__ import annotations

import dataclasses
import math

import numpy as np


@dataclasses.dataclass(frozen=True)
class BlockConfig:
    cfg_id: int
    name: str
    B: int
    N: int
    H: int
    d: int            # head dim of Q/K (input of the hash)
    nbits: int        # code length
    dv: int           # head dim of V
    attention: str    # "linear" | "hamming" | "none"
    E: int = 0        # embed width (= H * dv in every block config)
    hid: int = 0      # MLP hidden width
    shift_frac: float | None = None   # None: no MoE, every token -> shift MLP

    @property
    def T(self) -> int:
        return self.B * self.N

    @property
    def W(self) -> int:
        return self.nbits // 64


C1 = BlockConfig(1, "c1-deit-tiny-block", 1, 197, 3, 64, 64, 64, "linear", 192, 768, 0.5)
C2 = BlockConfig(2, "c2-pvt-stage1-linear-attn", 32, 3136, 1, 32, 64, 32, "linear")
C4 = BlockConfig(4, "c4-deit-base-block", 64, 197, 12, 64, 128, 64, "hamming", 768, 3072, 0.7)
C5 = BlockConfig(5, "c5-long-seq-block", 8, 16384, 4, 64, 256, 64, "linear", 256, 1024, None)

# Config 3 is two bare shift linears at DeiT-Small shapes.
C3_M = 64 * 197
C3_SHAPES = ((384, 1536), (1536, 384))     # (K, N)

BLOCK_CONFIGS = {1: C1, 2: C2, 4: C4, 5: C5}

# tensor ids (second word of the seed sequence)
_Q, _K, _V, _PROJ, _W1, _W2, _ROUTER, _MW1, _MW2, _X8, _XF = range(11)
_XIN, _LN1, _LN2, _WQ, _WK, _WV, _WO, _WG = range(11, 19)


def _rng(cfg_id: int, tensor_id: int, extra: int = 0) -> np.random.Generator:
    return np.random.default_rng([cfg_id, tensor_id, extra])


def scaled_down(cfg: BlockConfig, B: int | None = None, N: int | None = None) -> BlockConfig:
    """Same widths, fewer tokens: sizes the oracle finishes in seconds."""
    return dataclasses.replace(cfg, B=cfg.B if B is None else B, N=cfg.N if N is None else N)


# ---------------------------------------------------------------- attention --

def qkv(cfg: BlockConfig):
    """Q, K [B,N,H,d] and V [B,N,H,dv], fp32 ~ N(0,1)."""
    shape_qk = (cfg.B, cfg.N, cfg.H, cfg.d)
    shape_v = (cfg.B, cfg.N, cfg.H, cfg.dv)
    q = _rng(cfg.cfg_id, _Q).standard_normal(shape_qk, dtype=np.float32)
    k = _rng(cfg.cfg_id, _K).standard_normal(shape_qk, dtype=np.float32)
    v = _rng(cfg.cfg_id, _V).standard_normal(shape_v, dtype=np.float32)
    return q, k, v


def proj(cfg: BlockConfig) -> np.ndarray:
    """Seeded Gaussian hash matrix [d, nbits], the stand-in for learned hashing."""
    return _rng(cfg.cfg_id, _PROJ).standard_normal((cfg.d, cfg.nbits), dtype=np.float32)


def attention_scale(cfg: BlockConfig) -> float:
    """Post-add scale: keeps the linear output ~N(0,1); softmax temperature for Hamming."""
    if cfg.attention == "linear":
        return float(np.float32(1.0 / math.sqrt(cfg.N * cfg.nbits)))
    return float(np.float32(1.0 / math.sqrt(cfg.nbits)))


def random_codes(seed: int, shape, nbits: int) -> np.ndarray:
    """Uniform random packed codes [*shape, nbits // 64] uint64 (for attention stage tests)."""
    g = np.random.default_rng([99, seed])
    return g.integers(0, 2**64, size=tuple(shape) + (nbits // 64,), dtype=np.uint64)


# ------------------------------------------------------------ shift weights --

def shift_weight_raw(cfg_id: int, tensor_id: int, n_out: int, k_in: int):
    """sign in {-1,+1} uniform, e = p + 7 in {0..7} uniform; both [n_out, k_in]."""
    g = _rng(cfg_id, tensor_id)
    neg = g.integers(0, 2, size=(n_out, k_in), dtype=np.uint8)
    e = g.integers(0, 8, size=(n_out, k_in), dtype=np.uint8)
    return neg, e


def pack_w4(neg: np.ndarray, e: np.ndarray) -> np.ndarray:
    """Storage layout of the 4-bit weights: [n_out, k_in // 2] uint8."""
    nib = ((neg.astype(np.uint8) << 3) | e.astype(np.uint8)).astype(np.uint8)
    return (nib[:, 0::2] | (nib[:, 1::2] << 4)).astype(np.uint8)


def shift_weights(cfg_id: int, tensor_id: int, n_out: int, k_in: int) -> np.ndarray:
    neg, e = shift_weight_raw(cfg_id, tensor_id, n_out, k_in)
    return pack_w4(neg, e)


def int8_activations(cfg_id: int, m: int, k: int, extra: int = 0) -> np.ndarray:
    """int8 uniform in [-127, 127], shape [m, k]."""
    return _rng(cfg_id, _X8, extra).integers(-127, 128, size=(m, k), dtype=np.int8)


def float_activations(cfg_id: int, m: int, k: int, std: float = 1.0) -> np.ndarray:
    return (_rng(cfg_id, _XF).standard_normal((m, k), dtype=np.float32) * np.float32(std))


# ---------------------------------------------------------------- MLP / MoE --

@dataclasses.dataclass
class MlpParams:
    w1: np.ndarray          # [hid, E/2] packed 4-bit
    w2: np.ndarray          # [E, hid/2] packed 4-bit
    act_inv_scale: float    # fp32 -> int8 activation quantisation (passed in, static)
    requant_scale: float    # int32 fc1 accumulator -> int8 hidden pre-activation
    lut: np.ndarray         # [256] int8, index = hidden pre-activation + 128
    out_scale: float        # int32 fc2 accumulator -> fp32 output
    mw1: np.ndarray | None  # [hid, E] fp16 (Mult expert)
    mw2: np.ndarray | None  # [E, hid] fp16


_HIDDEN_UNITS_PER_ONE = 32.0      # int8 hidden code 32 stands for the real value 1.0
_RMS_W = math.sqrt((4.0**8 - 1.0) / (3.0 * 8.0))   # rms of 2^e, e uniform in 0..7


def activation_lut() -> np.ndarray:
    """Static int8 -> int8 table placed between the two shift linears (input data).

    Entry i is the table value for hidden code q = i - 128: a GELU-shaped curve
    sampled at q / 32 and stored at the same 1/32 resolution.
    """
    q = np.arange(-128, 128, dtype=np.float64)
    z = q / _HIDDEN_UNITS_PER_ONE
    erf = np.vectorize(math.erf)
    g = 0.5 * z * (1.0 + erf(z / math.sqrt(2.0)))
    return np.clip(np.rint(g * _HIDDEN_UNITS_PER_ONE), -127, 127).astype(np.int8)


def attention_out_std(cfg: BlockConfig) -> float:
    """Rough std of the attention output, used only to choose a static int8 clip."""
    if cfg.attention == "hamming":
        return 0.125
    return 1.0


def mlp_params(cfg: BlockConfig) -> MlpParams:
    E, hid = cfg.E, cfg.hid
    w1 = shift_weights(cfg.cfg_id, _W1, hid, E)
    w2 = shift_weights(cfg.cfg_id, _W2, E, hid)
    x_std = attention_out_std(cfg)
    act_inv_scale = float(np.float32(127.0 / (4.0 * x_std)))          # clip at 4 sigma
    y1_std = (127.0 / 4.0) * _RMS_W * math.sqrt(E)
    requant_scale = float(np.float32(_HIDDEN_UNITS_PER_ONE / y1_std))
    y2_std = 0.6 * _HIDDEN_UNITS_PER_ONE * _RMS_W * math.sqrt(hid)
    out_scale = float(np.float32(1.0 / y2_std))
    mw1 = mw2 = None
    if cfg.shift_frac is not None:
        mw1 = (_rng(cfg.cfg_id, _MW1).standard_normal((hid, E), dtype=np.float32)
               / np.float32(math.sqrt(E))).astype(np.float16)
        mw2 = (_rng(cfg.cfg_id, _MW2).standard_normal((E, hid), dtype=np.float32)
               / np.float32(math.sqrt(hid))).astype(np.float16)
    return MlpParams(w1, w2, act_inv_scale, requant_scale, activation_lut(), out_scale, mw1, mw2)


def router_logits(cfg: BlockConfig) -> np.ndarray:
    """fp32 [T, 2] with an exact, tie-free split: round(shift_frac * T) rows favour column 1.

    A seeded permutation picks which tokens; margins are |g| + 0.01 with
    g ~ N(0,1), logits = (-margin/2, +margin/2) signed by the chosen side.
    The latency-aware loss (Eq. 4) acts at training time only; at inference
    its effect is this load ratio, which the synthetic logits build in.
    """
    T = cfg.T
    g = _rng(cfg.cfg_id, _ROUTER)
    order = g.permutation(T)
    margin = np.abs(g.standard_normal(T, dtype=np.float32)) + np.float32(0.01)
    n_shift = int(math.floor(cfg.shift_frac * T + 0.5))
    delta = -margin
    delta[order[:n_shift]] = margin[order[:n_shift]]
    logits = np.stack([-delta / 2, delta / 2], axis=1).astype(np.float32)
    return np.ascontiguousarray(logits)


def random_logits(seed: int, T: int, tie_every: int = 0) -> np.ndarray:
    """Unstructured router logits for dispatch tests; optional exact ties."""
    g = np.random.default_rng([98, seed])
    logits = g.standard_normal((T, 2), dtype=np.float32)
    if tie_every:
        logits[::tie_every, 1] = logits[::tie_every, 0]
    return logits


# ------------------------------------------------ the whole layer of Eq. 2 --

@dataclasses.dataclass
class LayerParams:
    """Attention-side parameters of the complete block: two LayerNorms, the four attention
    Linears as packed 4-bit shift weights [E, E/2], their static scales, and the router."""
    gamma1: np.ndarray
    beta1: np.ndarray
    gamma2: np.ndarray
    beta2: np.ndarray
    eps: float
    ln_inv_scale: float     # LayerNorm output (unit variance) -> int8, clip at 4 sigma
    wq: np.ndarray
    wk: np.ndarray
    wv: np.ndarray
    wo: np.ndarray
    qkv_scale: float        # int32 accumulator -> fp32 Q, K, V (~ unit variance)
    o_scale: float          # int32 accumulator of Wo -> fp32 (~ unit variance)
    wg: np.ndarray | None   # [E, 2] fp32 router weight (None: no MoE)
    bg: np.ndarray | None   # [2]


def layer_input(cfg: BlockConfig) -> np.ndarray:
    """Tokens entering the layer, fp32 [T, E] ~ N(0,1)."""
    return _rng(cfg.cfg_id, _XIN).standard_normal((cfg.T, cfg.E), dtype=np.float32)


def layer_params(cfg: BlockConfig) -> LayerParams:
    E = cfg.E

    def affine(tid):
        g = _rng(cfg.cfg_id, tid)
        gamma = (1.0 + 0.1 * g.standard_normal(E)).astype(np.float32)
        beta = (0.1 * g.standard_normal(E)).astype(np.float32)
        return gamma, beta

    gamma1, beta1 = affine(_LN1)
    gamma2, beta2 = affine(_LN2)
    acc_std = (127.0 / 4.0) * _RMS_W * math.sqrt(E)
    scale = float(np.float32(1.0 / acc_std))
    wg = bg = None
    if cfg.shift_frac is not None:
        import statistics
        wg = (_rng(cfg.cfg_id, _WG).standard_normal((E, 2), dtype=np.float32) / np.float32(math.sqrt(E)))
        # logit difference ~ N(b, 2): b places the requested share of tokens on the Shift expert
        b = math.sqrt(2.0) * statistics.NormalDist().inv_cdf(cfg.shift_frac)
        bg = np.array([0.0, b], dtype=np.float32)
    return LayerParams(gamma1, beta1, gamma2, beta2, 1e-6, float(np.float32(127.0 / 4.0)),
                       shift_weights(cfg.cfg_id, _WQ, E, E), shift_weights(cfg.cfg_id, _WK, E, E),
                       shift_weights(cfg.cfg_id, _WV, E, E), shift_weights(cfg.cfg_id, _WO, E, E),
                       scale, scale, wg, bg)
