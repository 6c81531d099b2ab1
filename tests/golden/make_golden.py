"""Writes tests/golden/oracle_regression.json: the CPU oracle's own results on tiny seeded inputs.

The paper prints no worked numeric example for any of these operations (no kernel input / output pair
appears in its text, tables or appendix), so nothing here is a value from the paper; the file is a
regression guard for the oracle itself: a later change to its arithmetic shows up as a diff and has to
be justified.  The script calls only oracle/ and the seeded input generators.

    python tests/golden/make_golden.py
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle  # noqa: E402
from paper_2306_06446_amd import workloads as wl  # noqa: E402


def build():
    cfg = wl.BlockConfig(9, "golden-tiny", 1, 5, 2, 64, 64, 64, "hamming", 128, 128, 0.6)
    q, k, v = wl.qkv(cfg)
    pr = wl.proj(cfg)
    qc, kc = oracle.binarize(q, pr, 64), oracle.binarize(k, pr, 64)
    lin, kv = oracle.additive_attention(qc, kc, v, 64, wl.attention_scale(dataclass_linear(cfg)))
    ham = oracle.hamming_attention(qc, kc, v, 64, 0.125)
    x = wl.int8_activations(9, 4, 64)
    w4 = wl.shift_weights(9, 4, 6, 64)
    logits = wl.random_logits(9, 7, tie_every=3)
    perm, eo, cnt, gate = oracle.moe_dispatch(logits)
    lp, p = wl.layer_params(cfg), wl.mlp_params(cfg)
    layer = oracle.layer_forward(cfg, wl.layer_input(cfg), lp, p, pr, 0.125)
    w = (np.random.default_rng([9, 50]).standard_normal((2, 8)) * 0.3).astype(np.float32)
    out01, _, ksum, den = oracle.linear_attention_01(qc, kc, v, 64, 1.0)
    losses, _ = oracle.moe_balance_loss(logits, np.array([0.7, 0.3], np.float32), 0.1)
    return {
        "q_codes": [int(c) for c in qc.ravel()],
        "k_codes": [int(c) for c in kc.ravel()],
        "hamming_scores": oracle.hamming_scores(qc, kc, 64).ravel().tolist(),
        "linear_attention_row0": [round(float(t), 12) for t in lin[0, 0, 0, :8]],
        "ktv_row0": [round(float(t), 12) for t in kv[0, 0, 0, :8]],
        "hamming_attention_row0": [round(float(t), 12) for t in ham[0, 0, 0, :8]],
        "shift_linear": oracle.shift_linear(x, w4).ravel().tolist(),
        "dispatch_perm": perm.tolist(), "dispatch_counts": cnt.tolist(),
        "dispatch_gate": [round(float(g), 12) for g in gate],
        "layer_y_row0": [round(float(t), 9) for t in layer["y"][0, :8]],
        "layer_logits_row0": [round(float(t), 9) for t in layer["logits"][0]],
        "weights_from_float": oracle.shift_weights_from_float(w).ravel().tolist(),
        "linear_attention_01_row0": [round(float(t), 12) for t in out01[0, 0, 0, :8]],
        "linear_attention_01_den": den.ravel().tolist(), "ksum_head0": ksum[0, 0, :8].tolist(),
        "balance_losses": [round(float(t), 12) for t in losses],
    }


def dataclass_linear(cfg):
    import dataclasses
    return dataclasses.replace(cfg, attention="linear")


if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "oracle_regression.json")
    with open(path, "w") as f:
        json.dump(build(), f, indent=1, sort_keys=True)
        f.write("\n")
    print("wrote", path)
