#!/usr/bin/env python3
"""Block throughput of libshiftadd on one MI355X, with roofline and CPU-oracle baseline.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config c4]

A step is one pass of the whole block (hash Q and K, attention, activation
quantisation, routing, both experts, combine) over one batch of seeded synthetic
input that is already resident in HBM.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0            # MI355X HBM3E
PEAK_TFLOPS = {                  # dense peaks of MI355X
    "alu_fp32": 157.3,           # fp32 vector FMA: 256 CU x 128 lanes x 2 flop x 2.4 GHz (needs packed ops)
    "alu_int": 39.3,             # 32-bit integer vector ops: 256 CU x 64 lanes x 2.4 GHz
    "mfma_i8": 5000.0,
    "mfma_f16": 2500.0,
    # an fp32 contraction with one exactly-representable (+-1 or two-term) operand runs as three bf16
    # matrix-core products of the fp32 operand's exact bf16 terms: its algorithmic flops are priced at
    # the bf16 peak / 3 (above the fp32 matrix peak of 157.3, which such a kernel can beat)
    "mfma_bf16x3": 2500.0 / 3,
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", default="c4", choices=["c1", "c2", "c3", "c4", "c5"],
                    help="c3 times the two shift linear layers alone, in both variants")
    ap.add_argument("--streams", type=int, default=1, choices=[1, 2, 3, 4],
                    help="HIP streams the K steps are enqueued on in turn (each step is one whole pass on one stream, on "
                         "input sets of that stream's own).  1 (the default, and what `value` reports) = strictly one step "
                         "after another; with 2, the attention kernels of one step overlap the expert GEMMs of the previous "
                         "one, as two concurrent requests would")
    ap.add_argument("--also-streams", type=int, default=2, choices=[0, 2, 3, 4],
                    help="the same K steps are timed once more on this many streams and reported beside the headline as "
                         "`multi_stream` (0 = skip)")
    ap.add_argument("--settle-ms", type=float, default=250.0,
                    help="untimed steps are run for this long before the W warm-up steps: the device takes on the order "
                         "of 100 ms of load to reach its steady clocks, longer than a small W covers (0 = off)")
    ap.add_argument("--rotate", type=int, default=0,
                    help="input/workspace sets cycled through (0 = enough to exceed the 256 MiB last-level cache)")
    ap.add_argument("--shift-variant", type=int, default=1, choices=[0, 1, 2, 3],
                    help="0 VALU shift-and-accumulate; 1 (default, what `value` reports) matrix cores, reading the packed "
                         "4-bit weights in every step (their decode to int8 planes is inside the timed region); 2 auto; "
                         "3 matrix cores on planes decoded once before the timed region (a layout change of the constant "
                         "weights; reported beside the headline as `prepared_planes`)")
    ap.add_argument("--no-prepared", action="store_true", help="skip the extra timing of the prepared-planes variant")
    ap.add_argument("--additive-valu", action="store_true",
                    help="linear attention: run the sign-select-and-accumulate kernels on the vector ALU instead of the "
                         "matrix cores (the measured alternative; per-kernel timings and profiles of both back the choice)")
    ap.add_argument("--probe", action="store_true",
                    help="no workload: a register-only loop of matrix instructions (sa_probe_mfma) on every CU, to read off the "
                         "rate and the shader clock the matrix cores sustain with low-toggle, random and Shift-layer-like operands")
    ap.add_argument("--sweep", action="store_true",
                    help="kernel sweep over pyramid-ViT stage shapes at batch 1 and 32: the Add kernels (K^T V, Q(K^T V)) and "
                         "the Shift linear layers, each beside a dense fp32 library GEMM of the same contraction")
    ap.add_argument("--cu-split", type=float, default=0.0,
                    help="with --experts: also run the two experts side by side on two streams that each own a share of the "
                         "compute units (this fraction to the Mult expert, the rest to the Shift expert; HIP stream CU masks)")
    ap.add_argument("--experts", action="store_true",
                    help="the two experts of the MoE MLP one after the other on one stream and side by side on two, with the "
                         "paper's modularized figure (slower expert alone) beside the wall-clock ones")
    ap.add_argument("--layer", action="store_true",
                    help="time the complete block of Eq. 2 (sa_layer_forward: LayerNorms, the four attention Linears "
                         "as shift layers, residuals, router) on tokens of the chosen configuration's shape")
    ap.add_argument("--sign-hash", action="store_true",
                    help="with --layer: the sign-hash variant (no projection, nbits = head width), whose code bits are "
                         "taken in the epilogue of the fused Q/K/V projection")
    ap.add_argument("--zero-one", action="store_true",
                    help="time the {0,1}-code normalised linear attention with the depthwise convolution on V "
                         "(sa_linear_attention_01 + sa_dwconv3x3) at the chosen configuration's attention shape (c2, c5)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernels", action="store_true", help="skip the per-kernel timing pass")
    ap.add_argument("--cpu-sample-batch", type=int, default=0)
    ap.add_argument("--kernels-only", action="store_true",
                    help="skip the block steps and run only the per-kernel timing pass (for a rocprofv3 trace whose "
                         "per-kernel averages cover exactly the launches the live timings cover)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one 256 MiB device copy first: a kernel of known traffic for scaling rocprofv3 "
                         "FETCH_SIZE / WRITE_SIZE readings")
    return ap.parse_args()


def kernel_table(cfg, p, counts, shift_variant=1):
    """Algorithmic bytes and operations of every kernel of the block (what the method must move and
    compute: packed codes, 4-bit weights, int8 activations; never the dense fp32 work it avoids).
    `bytes_fetched`, where given, is what the timed kernel of this variant actually requests when that differs:
    the matrix-core Shift GEMMs read two int8 planes per weight matrix (2 bytes per weight) where the method
    stores 4 bits; with variant 1 a decode launch per step reads the 4-bit rows and writes those planes."""
    T, E, H, N, B = cfg.T, cfg.E, cfg.H, cfg.N, cfg.B
    rows = T * H
    tab = []
    bin_bytes = rows * cfg.d * 4 + cfg.d * cfg.nbits * 4 + rows * cfg.nbits // 8
    bin_flop = 2 * rows * cfg.nbits * cfg.d
    # Q and K are hashed by one launch
    tab.append(dict(name="binarize_qk", bytes=2 * bin_bytes - cfg.d * cfg.nbits * 4, ops=2 * bin_flop,
                    compute="mfma_bf16x3" if cfg.d in (32, 64, 128) else "alu_fp32"))
    code_b = rows * cfg.nbits // 8
    v_b = rows * cfg.dv * 4
    if cfg.attention == "linear":
        kv_b = B * H * cfg.nbits * cfg.dv * 4
        flops = 2 * rows * cfg.nbits * cfg.dv     # one sign-selected accumulate per (token, bit, column)
        tab.append(dict(name="ktv", bytes=code_b + v_b + kv_b, ops=flops, compute="mfma_bf16x3"))
        tab.append(dict(name="qkv", bytes=code_b + kv_b + v_b, ops=flops, compute="mfma_bf16x3"))
    else:
        pairs = B * H * N * N
        # P * V is the dense fp32 contraction of this kernel (it runs as three bf16 matrix-core products);
        # with an MLP behind it the kernel also writes its output as int8 codes (and fp16 for a Mult expert)
        extra = T * E * (1 + (2 if counts is not None else 0)) if cfg.E else 0
        tab.append(dict(name="hamming", bytes=2 * code_b + 2 * v_b + extra, ops=2 * pairs * cfg.dv,
                        compute="mfma_bf16x3"))
    if cfg.E:
        if cfg.attention == "linear":
            tab.append(dict(name="quantize", bytes=T * E * (5 + (2 if counts is not None else 0)), ops=2 * T * E,
                            compute="alu_fp32"))
        t_shift, t_mult = (counts[1], counts[0]) if counts is not None else (T, 0)
        if counts is not None:
            tab.append(dict(name="dispatch", bytes=T * (8 + 12), ops=4 * T, compute="alu_fp32"))
            tab.append(dict(name="mult_fc1", bytes=t_mult * E * 2 + E * cfg.hid * 2 + t_mult * cfg.hid * 2,
                            ops=2 * t_mult * E * cfg.hid, compute="mfma_f16"))
            tab.append(dict(name="mult_fc2", bytes=t_mult * cfg.hid * 2 + E * cfg.hid * 2 + t_mult * E * 4,
                            ops=2 * t_mult * E * cfg.hid, compute="mfma_f16"))
        planes = shift_variant in (1, 2, 3)
        if shift_variant in (1, 2):
            # reads both packed matrices, writes two int8 planes for each: an overhead of this kernel design (no
            # algorithmic bytes of its own: the 4-bit weights are counted with the layers that use them)
            tab.append(dict(name="shift_decode", bytes=0, ops=0, compute="alu_int", bytes_fetched=E * cfg.hid + 4 * E * cfg.hid))
        for name, a_in, a_out in (("shift_fc1", t_shift * E, t_shift * cfg.hid), ("shift_fc2", t_shift * cfg.hid, t_shift * E * 4)):
            row = dict(name=name, bytes=a_in + E * cfg.hid // 2 + a_out, ops=2 * t_shift * E * cfg.hid, compute="mfma_i8")
            if planes:
                row["bytes_fetched"] = a_in + 2 * E * cfg.hid + a_out
            tab.append(row)
    return tab


def floors_us(k, shift_variant):
    comp = k["compute"]
    if comp == "mfma_i8" and shift_variant == 0:
        comp = "alu_int"
    t_hbm = (k["bytes"] or k.get("bytes_fetched", 0)) / (HBM_PEAK_GBS * 1e9) * 1e6
    t_cmp = k["ops"] / (PEAK_TFLOPS[comp] * 1e12) * 1e6
    return t_hbm, t_cmp, comp


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU only: this build has no multi-GPU path (got --gpus %d)" % args.gpus,
              file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch

    from paper_2306_06446_amd import binding as sa, workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    sa.load_library()
    if args.probe:
        return bench_probe(args, sa, torch)
    if args.sweep:
        return bench_sweep(args, sa, wl, torch, np)
    if args.config == "c3":
        return bench_shift_linear(args, sa, wl, torch, np)
    cfg = {"c1": wl.C1, "c2": wl.C2, "c4": wl.C4, "c5": wl.C5}[args.config]
    if args.layer:
        return bench_layer(args, sa, wl, torch, np, cfg)
    if args.zero_one:
        return bench_zero_one(args, sa, wl, torch, np, cfg)
    if args.experts:
        return bench_experts(args, sa, wl, torch, np, cfg)
    moe = cfg.E > 0 and cfg.shift_frac is not None

    def dev(a):
        a = np.ascontiguousarray(a)
        if a.dtype == np.uint64:
            a = a.view(np.int64)
        return torch.from_numpy(a).cuda()

    # ---- inputs (host, seeded) and device copies
    q, k, v = wl.qkv(cfg)
    pr = wl.proj(cfg)
    scale = wl.attention_scale(cfg)
    p = wl.mlp_params(cfg) if cfg.E else None
    logits = wl.router_logits(cfg) if moe else None
    shared = dict(proj=dev(pr))
    if p is not None:
        shared.update(w1=dev(p.w1), w2=dev(p.w2), lut=dev(p.lut))
        if moe:
            shared.update(mw1=dev(p.mw1), mw2=dev(p.mw2))
    per_set_bytes = (q.nbytes + k.nbytes + v.nbytes) + 2 * cfg.T * max(cfg.E, cfg.H * cfg.dv) * 4
    n_sets = args.rotate or max(1, min(8, math.ceil(600e6 / per_set_bytes)))
    per = math.lcm(args.streams, args.also_streams or 1)
    n_sets = (n_sets + per - 1) // per * per                                 # every set stays on one stream
    inputs = [dict(q=dev(q), k=dev(k), v=dev(v), logits=dev(logits) if moe else None) for _ in range(n_sets)]

    def make_blocks(variant):
        """One Block (descriptor + workspace + outputs) per input set; the Shift weights as the variant reads them."""
        w = dict(shared)
        if p is not None and variant == 3:
            w.update(w1=sa.sa_shift_planes_prepare(shared["w1"]), w2=sa.sa_shift_planes_prepare(shared["w2"]))
        out = []
        for inp in inputs:
            kw = dict(B=cfg.B, N=cfg.N, H=cfg.H, d=cfg.d, nbits=cfg.nbits, dv=cfg.dv,
                      attention=0 if cfg.attention == "linear" else 1, hid=cfg.hid, moe=moe, attn_scale=scale,
                      q=inp["q"], k=inp["k"], v=inp["v"], proj=w["proj"], shift_variant=variant)
            if p is not None:
                kw.update(act_inv_scale=p.act_inv_scale, requant_scale=p.requant_scale, out_scale=p.out_scale,
                          w1=w["w1"], w2=w["w2"], lut=w["lut"])
                if moe:
                    kw.update(logits=inp["logits"], mw1=w["mw1"], mw2=w["mw2"])
            out.append((sa.Block(**kw), kw))
        return out

    blocks = make_blocks(args.shift_variant)

    if args.calibrate_copy:
        src = torch.full((64 << 20,), 1.0, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)                     # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst

    # ---- the timed region: W warm-up steps, then exactly K steps
    n_warm, n_steps = (0, 1) if args.kernels_only else (args.warmup, args.steps)

    def timed_ms_per_step(blks, n_streams):
        run_steps = make_step_runner(torch, n_streams, n_sets, lambda i: blks[i][0].forward())
        if not args.kernels_only:
            settle(torch, run_steps, args.settle_ms)
        run_steps(n_warm)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run_steps(n_steps)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / n_steps

    ms_per_step = timed_ms_per_step(blocks, args.streams)
    tokens_per_s = cfg.T / (ms_per_step * 1e-3)

    # ---- the same steps once more with a HIP event after each (median / min of single steps), cold (rotating
    #      buffer sets, larger than the last-level cache together) and hot (one set, cache-resident inputs)
    def step_times(blks, pick):
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(n_steps + 1)]
        evs[0].record()
        for i in range(n_steps):
            blks[pick(i)][0].forward()
            evs[i + 1].record()
        torch.cuda.synchronize()
        us = sorted(evs[i].elapsed_time(evs[i + 1]) * 1e3 for i in range(n_steps))
        return {"median": round(us[len(us) // 2], 2), "min": round(us[0], 2)}

    step_us = multi_stream = prepared = None
    if not args.kernels_only:
        step_us = {"cold": step_times(blocks, lambda i: i % n_sets), "hot": step_times(blocks, lambda i: 0)}
        if args.also_streams and args.also_streams != args.streams:
            ms2 = timed_ms_per_step(blocks, args.also_streams)
            multi_stream = {"streams": args.also_streams, "ms_per_step": round(ms2, 5), "tokens_per_s": round(cfg.T / (ms2 * 1e-3), 1),
                            "note": "successive steps enqueued on the streams in turn, all K complete inside the timed region"}
        if p is not None and args.shift_variant == 1 and not args.no_prepared:
            blocks3 = make_blocks(3)
            ms3 = timed_ms_per_step(blocks3, args.streams)
            prepared = {"shift_variant": 3, "ms_per_step": round(ms3, 5), "tokens_per_s": round(cfg.T / (ms3 * 1e-3), 1),
                        "step_us": step_times(blocks3, lambda i: i % n_sets),
                        "note": "Shift weights as int8 planes decoded once before the timed region: the timed GEMMs read "
                                "16 bits per weight instead of the 4 stored ones, and no decode kernel runs"}
            del blocks3

    # ---- per-kernel durations, HIP events on the launch stream, same buffers, same rotation
    counts = None
    if moe:
        n_shift = int(math.floor(cfg.shift_frac * cfg.T + 0.5))
        counts = (cfg.T - n_shift, n_shift)
    table = kernel_table(cfg, p, counts, args.shift_variant)
    kernels = {}
    derived = set()
    if not args.no_kernels:
        stage_sets = [make_stages(sa, torch, cfg, kw, p, moe, args.shift_variant) for _, kw in blocks]

        def time_stage(name, steps):
            for s in stage_sets:              # warm-up, also fills the intermediates later stages read
                s[name]()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for i in range(steps):
                stage_sets[i % n_sets][name]()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) * 1e3 / steps                    # us per launch

        for name in [t["name"] for t in table]:
            if name != "shift_decode":
                kernels[name] = time_stage(name, args.steps)
        if "shift_mlp_both" in stage_sets[0]:
            # the decode launch is not an entry point of its own: both layers with it, minus the two layers alone
            both = time_stage("shift_mlp_both", args.steps)
            kernels["shift_decode"] = max(0.0, both - kernels["shift_fc1"] - kernels["shift_fc2"])
            derived.add("shift_decode")
        # the measured alternatives of the linear-attention kernels (vector ALU instead of matrix cores)
        alternatives = {n: round(time_stage(n, max(3, args.steps // 10)), 2) for n in ("ktv_valu", "qkv_valu") if n in stage_sets[0]}

    report = []
    for t in table:
        t_hbm, t_cmp, comp = floors_us(t, args.shift_variant)
        us = kernels.get(t["name"])
        row = dict(name=t["name"], us=None if us is None else round(us, 2), bytes=t["bytes"], ops=t["ops"],
                   hbm_floor_us=round(t_hbm, 2), compute_floor_us=round(t_cmp, 2),
                   bound="hbm" if t_hbm >= t_cmp else ("mfma" if comp.startswith("mfma") else "alu"),
                   compute_peak=comp)
        if "bytes_fetched" in t:
            row["bytes_fetched"] = t["bytes_fetched"]
        if t["name"] in derived:
            row["derived"] = "both layers in one call minus the two layers alone"
        if us:
            row["hbm_frac"] = round(t_hbm / us, 4)
            row["binding_frac"] = round(max(t_hbm, t_cmp) / us, 4)
        report.append(row)

    roofline = None
    timed = [r for r in report if r["us"]]
    if timed:
        dom = max(timed, key=lambda r: r["us"])
        if dom["bound"] == "hbm":
            ach, peak, unit = dom["bytes"] / (dom["us"] * 1e-6) / 1e9, HBM_PEAK_GBS, "GB/s"
        else:
            ach, peak, unit = dom["ops"] / (dom["us"] * 1e-6) / 1e12, PEAK_TFLOPS[dom["compute_peak"]], "TFLOP/s"
        roofline = dict(kernel=dom["name"], bound=dom["bound"], achieved=round(ach, 3), peak=peak, unit=unit,
                        frac=round(ach / peak, 4), traffic=read_traffic(args.config, dom["name"]),
                        traffic_source="profiles/traffic_%s.txt: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of an earlier run of "
                                       "this command, scaled by a 256 MiB copy (not measured in this run)" % args.config,
                        us_per_launch=dom["us"])
    # experts timed one after the other, counted as if they ran perfectly in parallel (the paper's
    # "modularized" latency: the layer costs its slower expert)
    modularized_us = None
    if timed and moe:
        by = {r["name"]: r["us"] for r in timed}
        experts = [by.get("mult_fc1", 0) + by.get("mult_fc2", 0), by.get("shift_fc1", 0) + by.get("shift_fc2", 0)]
        rest = sum(us for n, us in by.items() if not n.startswith(("mult_", "shift_")) and n != "dispatch")
        modularized_us = round(rest + max(experts), 2)
    block_bytes = sum(t["bytes"] for t in table)
    block_hbm_frac = block_bytes / (ms_per_step * 1e-3) / (HBM_PEAK_GBS * 1e9)

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(cfg, args.cpu_sample_batch)

    out = {
        "metric": "block tokens/s (additive attn + shift MLP) at 1 GPU; % HBM roofline",
        "value": round(tokens_per_s, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32+u64 codes+i8/i32 shift+f16 mult",
        "data": "synthetic",
        "config": {"workload": cfg.name, "B": cfg.B, "N": cfg.N, "H": cfg.H, "d": cfg.d, "nbits": cfg.nbits,
                   "E": cfg.E, "hid": cfg.hid, "attention": cfg.attention,
                   "mlp": ("moe %.0f%% shift / %.0f%% fp16 mult" % (100 * cfg.shift_frac, 100 - 100 * cfg.shift_frac))
                   if moe else ("shift" if cfg.E else "none"),
                   "input_sets_rotated": n_sets, "shift_variant": args.shift_variant, "streams": args.streams,
                   "settle_ms": args.settle_ms},
        "step_us": step_us, "multi_stream": multi_stream, "prepared_planes": prepared,
        "block_hbm_roofline_frac": round(block_hbm_frac, 4),
        "block_algorithmic_bytes": block_bytes,
        "block_us_sum_of_kernels_modularized": modularized_us,
        "roofline": roofline, "cpu_baseline": cpu, "kernels": report,
    }
    if not args.no_kernels and alternatives:
        out["kernel_alternatives_us"] = alternatives
    print(json.dumps(out))


def make_step_runner(torch, n_streams, n_sets, forward_set):
    """run(k): enqueue k steps, step i on stream i % n_streams and on input set i % n_sets (n_sets is a multiple of
    n_streams, so a set is only ever used on one stream and its steps stay ordered).  The caller synchronises."""
    if n_streams == 1:
        def run(k):
            for i in range(k):
                forward_set(i % n_sets)
        return run
    streams = [torch.cuda.Stream() for _ in range(n_streams)]

    def run(k):
        for s in streams:
            s.wait_stream(torch.cuda.current_stream())
        for i in range(k):
            with torch.cuda.stream(streams[i % n_streams]):
                forward_set(i % n_sets)
    return run


def settle(torch, run_steps, ms):
    """Runs untimed steps for about `ms` of wall-clock time, so that the W warm-up steps and the timed region start at
    steady clocks whatever W is."""
    t_end = time.perf_counter() + ms * 1e-3
    while ms > 0 and time.perf_counter() < t_end:
        run_steps(8)
        torch.cuda.synchronize()


def _time_us(torch, fn, steps, warm=3):
    """Average device time of fn() over `steps` back-to-back calls on the current stream (HIP events)."""
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / steps


def _time_us_graph(torch, fn, reps=20, replays=10):
    """Device time of fn() with the host out of the picture: `reps` calls are captured into one HIP graph on a side
    stream and the graph is replayed (kernels only; nothing captured here clears memory).  Small kernels take less
    time than a Python call enqueues them in, so back-to-back eager calls would time the host.  Falls back to eager
    timing if the capture fails."""
    try:
        fn()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                for _ in range(reps):
                    fn()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(replays):
            graph.replay()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / (reps * replays)
    except Exception as exc:      # noqa: BLE001 - any capture problem: time eagerly and say so
        print("graph capture failed (%s): eager timing" % exc, file=sys.stderr)
        torch.cuda.synchronize()
        return _time_us(torch, fn, reps * replays)


def bench_experts(args, sa, wl, torch, np, cfg):
    """The MoE MLP of the block with its two experts (a) one after the other on one stream, as sa_block_forward runs
    them, and (b) side by side on two streams that fork after the dispatch and join before the next step (Sec. 4.2: the
    experts are independent once the routing lists exist; the paper's tables count them as perfectly parallel, its
    'modularized' latency = the slower expert alone)."""
    assert cfg.E and cfg.shift_frac is not None, "--experts needs a configuration with a MoE MLP (c1, c4)"
    T, E, hid = cfg.T, cfg.E, cfg.hid
    p = wl.mlp_params(cfg)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    x = dev(wl.float_activations(cfg.cfg_id, T, E, std=wl.attention_out_std(cfg)))
    xq, xh = sa.sa_quantize_act_half(x, p.act_inv_scale)
    perm, eo, cnt, gate = sa.sa_moe_dispatch(dev(wl.router_logits(cfg)))
    counts = [int(c) for c in cnt.cpu()]
    w1, w2, var = dev(p.w1), dev(p.w2), args.shift_variant
    if var == 3:
        w1, w2 = sa.sa_shift_planes_prepare(w1), sa.sa_shift_planes_prepare(w2)
    lut, mw1, mw2 = dev(p.lut), dev(p.mw1), dev(p.mw2)
    lib = sa.load_library()
    sws = torch.empty(max(16, lib.sa_shift_mlp_workspace_bytes(sa._l(T), E, hid)), dtype=torch.uint8, device="cuda")
    mws = torch.empty(max(16, lib.sa_mult_mlp_workspace_bytes(sa._l(T), E, hid)), dtype=torch.uint8, device="cuda")
    y = torch.zeros((T, E), dtype=torch.float32, device="cuda")

    def mult():
        sa.sa_mult_mlp_f16_half(xh, mw1, mw2, rows=perm, counts=cnt, expert=0, max_rows=T, want_out=False, y=y, gate=gate,
                                workspace=mws)

    def shift():
        sa.sa_shift_mlp(xq, w1, w2, p.requant_scale, lut, rows=perm, counts=cnt, expert=1, max_rows=T, want_y2=False, y=y,
                        gate=gate, out_scale=p.out_scale, variant=var, workspace=sws)

    def sequential():
        mult()
        shift()

    s_m, s_s = torch.cuda.Stream(), torch.cuda.Stream()
    fork, j_m, j_s = (torch.cuda.Event() for _ in range(3))

    def concurrent():
        cur = torch.cuda.current_stream()
        fork.record(cur)
        s_m.wait_event(fork)
        s_s.wait_event(fork)
        with torch.cuda.stream(s_m):
            mult()
            j_m.record(s_m)
        with torch.cuda.stream(s_s):
            shift()
            j_s.record(s_s)
        cur.wait_event(j_m)
        cur.wait_event(j_s)

    sequential()
    torch.cuda.synchronize()
    y_seq = y.clone()
    y.zero_()
    concurrent()
    torch.cuda.synchronize()
    same = bool(torch.equal(y, y_seq))
    t_end = time.perf_counter() + args.settle_ms * 1e-3
    while time.perf_counter() < t_end:
        for _ in range(8):
            sequential()
        torch.cuda.synchronize()
    us = {"mult_alone": _time_us(torch, mult, args.steps), "shift_alone": _time_us(torch, shift, args.steps),
          "sequential": _time_us(torch, sequential, args.steps), "concurrent": _time_us(torch, concurrent, args.steps)}
    if args.cu_split > 0.0:
        # the chip partitioned between the experts: each stream may only use its own compute units
        import ctypes
        hip = ctypes.CDLL("libamdhip64.so")
        n_cu = torch.cuda.get_device_properties(0).multi_processor_count
        n_m = max(1, min(n_cu - 1, int(round(args.cu_split * n_cu))))
        words = (n_cu + 31) // 32

        def masked_stream(lo, hi):
            mask = (ctypes.c_uint32 * words)()
            for cu in range(lo, hi):
                mask[cu // 32] |= 1 << (cu % 32)
            handle = ctypes.c_void_p()
            rc = hip.hipExtStreamCreateWithCUMask(ctypes.byref(handle), ctypes.c_uint32(words), mask)
            assert rc == 0 and handle.value, "hipExtStreamCreateWithCUMask failed: %d" % rc
            return torch.cuda.ExternalStream(handle.value)

        s_m, s_s = masked_stream(0, n_m), masked_stream(n_m, n_cu)
        y.zero_()
        concurrent()
        torch.cuda.synchronize()
        same = same and bool(torch.equal(y, y_seq))
        with torch.cuda.stream(s_m):
            us["mult_alone_on_its_cus"] = _time_us(torch, mult, args.steps)
        with torch.cuda.stream(s_s):
            us["shift_alone_on_its_cus"] = _time_us(torch, shift, args.steps)
        us["concurrent_cu_split"] = _time_us(torch, concurrent, args.steps)
        us["cu_split"] = {"mult_cus": n_m, "shift_cus": n_cu - n_m}
    us = {k: (round(v, 2) if isinstance(v, float) else v) for k, v in us.items()}
    # For scale only, never part of the path: the vendor library's GEMM behind torch at the shapes of the four expert
    # layers, on compact operands (no gather, no activation, no gate, no scatter), fp16 for the Mult expert and ONE
    # int8 plane with int32 output for the Shift expert (the library's own layers run two planes each).
    library = {}
    try:
        n_m, n_s = counts[0], (counts[1] + 7) // 8 * 8
        for name, M, K, N, kind in (("mult_fc1_f16", n_m, E, hid, "f16"), ("mult_fc2_f16", n_m, hid, E, "f16"),
                                    ("shift_fc1_one_int8_plane", n_s, E, hid, "i8"), ("shift_fc2_one_int8_plane", n_s, hid, E, "i8")):
            if M == 0:
                continue
            if kind == "f16":
                a = torch.randn((M, K), device="cuda", dtype=torch.float16)
                b = (torch.randn((N, K), device="cuda", dtype=torch.float16) / 32).t()
                o = torch.empty((M, N), device="cuda", dtype=torch.float16)
                fn = lambda a=a, b=b, o=o: torch.matmul(a, b, out=o)
                peak = 2.5e15
            else:
                a = torch.randint(-127, 128, (M, K), device="cuda", dtype=torch.int8)
                b = torch.randint(-127, 128, (N, K), device="cuda", dtype=torch.int8).t()
                fn = lambda a=a, b=b: torch._int_mm(a, b)
                peak = 5.0e15
            t = _time_us_graph(torch, fn)
            library[name] = {"M": M, "K": K, "N": N, "us": round(t, 2), "frac_of_peak": round(2.0 * M * K * N / (t * 1e-6) / peak, 3)}
            del a, b
    except Exception as exc:      # noqa: BLE001 - a reference that is not available is left out
        library["unavailable"] = str(exc)[:200]
    out = {"metric": "MoE MLP tokens/s (Mult and Shift expert after the dispatch) at 1 GPU",
           "value": round(T / (us["sequential"] * 1e-6), 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": 3,
           "ms_per_step": round(us["sequential"] * 1e-3, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "i8/i32 shift+f16 mult", "data": "synthetic",
           "config": {"workload": cfg.name + "-experts", "T": T, "E": E, "hid": hid, "tokens_mult": counts[0], "tokens_shift": counts[1],
                      "shift_variant": var},
           "experts_us": us, "modularized_us": max(us["mult_alone"], us["shift_alone"]),
           "vendor_library_gemm_for_scale": library,
           "concurrent_output_identical": same,
           "note": "sequential = both experts on one stream (what sa_block_forward does); concurrent = two streams forked after "
                   "the dispatch and joined; modularized = the slower expert alone, the figure the paper's tables report for "
                   "experts counted as perfectly parallel",
           "roofline": None, "cpu_baseline": None}
    print(json.dumps(out))


def bench_probe(args, sa, torch):
    """What the matrix cores sustain before any kernel design enters: sa_probe_mfma runs 8 independent accumulator
    chains per wavefront, 4 wavefronts per workgroup, operands in registers, nothing else.  Rate from HIP events
    around one launch; clock = shader cycles / 100 MHz wall ticks of workgroup 0's loop, read inside the kernel."""
    n_cu = torch.cuda.get_device_properties(0).multi_processor_count
    iters = 20000
    out = torch.zeros(4, dtype=torch.int64, device="cuda")
    rows = []
    cases = [("int8 32x32x32", 0, 65536.0, 5.0e15, [(0, "one non-zero element per register"), (1, "random bits"),
                                                    (2, "Shift-layer-like: random int8 x powers of two / 7/8 zeros")]),
             ("fp16 32x32x16", 1, 32768.0, 2.5e15, [(0, "one non-zero element per register"), (1, "random finite halves")]),
             ("bf16 32x32x16", 2, 32768.0, 2.5e15, [(0, "one non-zero element per register"), (1, "random finite values")])]
    for name, kind, ops, peak, modes in cases:
        for operands, what in modes:
            for wgs in (1, n_cu // 8, n_cu, 2 * n_cu):
                for _ in range(2):                    # the first launch warms the clocks of this case
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record()
                    sa.sa_probe_mfma(kind, operands, wgs, iters, out=out)
                    e1.record()
                    torch.cuda.synchronize()
                ms = e0.elapsed_time(e1)
                cyc, ticks = int(out[0]), int(out[1])
                n_inst = wgs * 4 * iters * 8
                rate = n_inst * ops / (ms * 1e-3)
                rows.append({"instruction": name, "operands": what, "workgroups": wgs, "ms": round(ms, 3),
                             "rate_pops": round(rate / 1e15, 3), "frac_of_published_peak": round(rate / peak, 3),
                             "shader_mhz": round(cyc / ticks * 100.0, 0) if ticks else None,
                             "cycles_per_instruction_of_a_wavefront": round(cyc / (iters * 8), 1)})
    print("| instruction | operands | workgroups | P op/s | of peak | MHz | cycles per MFMA of a wavefront |", file=sys.stderr)
    print("|---|---|---|---|---|---|---|", file=sys.stderr)
    for r in rows:
        print("| %s | %s | %d | %.2f | %.2f | %s | %s |" % (r["instruction"], r["operands"], r["workgroups"], r["rate_pops"],
                                                          r["frac_of_published_peak"], r["shader_mhz"],
                                                          r["cycles_per_instruction_of_a_wavefront"]), file=sys.stderr)
    like = [r for r in rows if r["operands"].startswith("Shift") and r["workgroups"] == n_cu][0]
    out_line = {"metric": "int8 matrix-instruction rate sustained by a register-only loop on all CUs, Shift-layer-like operands",
                "value": like["rate_pops"] * 1e3, "unit": "TOP/s", "n_gpus": 1, "steps": 1, "warmup": 1, "ms_per_step": like["ms"],
                "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "i8", "data": "synthetic",
                "config": {"workload": "matrix-core-probe", "compute_units": n_cu, "iterations": iters},
                "probe": rows, "roofline": None, "cpu_baseline": None}
    print(json.dumps(out_line))


# Stage shapes of a small pyramid ViT at 224 x 224 input (tokens per image, embedding width, heads, MLP ratio): the
# shapes the paper's kernel figures sweep over are in figures that did not survive, so the public stage shapes of
# that model family stand in (head width 32 everywhere).
PYRAMID_STAGES = ((3136, 32, 1, 8), (784, 64, 2, 8), (196, 160, 5, 4), (49, 256, 8, 4))


def bench_sweep(args, sa, wl, torch, np):
    """The form of the paper's kernel figures (Sec. 5.4 and the appendix on kernel speed-ups at batch 1 and 32): per
    stage shape, the Add kernels against a dense fp32 MatMul of the same contraction, and the Shift linear layers
    against a dense fp32 linear with the same (decoded) weights.  The dense side is the library GEMM behind
    torch.matmul: a baseline that is reported, never part of the path."""
    rows = []
    steps = 200          # launches timed per kernel (20 per captured graph, 10 replays)
    nbits = 64
    for batch in (1, 32):
        for si, (n_tok, E, H, ratio) in enumerate(PYRAMID_STAGES):
            d = E // H
            g = np.random.default_rng([50, batch, si])
            # ---- Add layers: K^T V and Q (K^T V) on 64-bit codes of head width 32
            qc = torch.from_numpy(g.integers(0, 2**63, size=(batch, H, n_tok, nbits // 64), dtype=np.int64)).cuda()
            kc = torch.from_numpy(g.integers(0, 2**63, size=(batch, H, n_tok, nbits // 64), dtype=np.int64)).cuda()
            v = torch.from_numpy(g.standard_normal((batch, n_tok, H, d), dtype=np.float32)).cuda()
            lib = sa.load_library()
            ws = torch.empty(max(16, lib.sa_additive_attention_workspace_bytes(batch, H, n_tok, nbits, d)), dtype=torch.uint8, device="cuda")
            kv = torch.empty((batch, H, nbits, d), dtype=torch.float32, device="cuda")
            o = torch.empty((batch, n_tok, H, d), dtype=torch.float32, device="cuda")
            scale = 1.0 / math.sqrt(n_tok * nbits)
            t_ktv = _time_us_graph(torch, lambda: sa.sa_additive_attention(None, kc, v, scale, nbits, phases=1, kv=kv, workspace=ws))
            t_qkv = _time_us_graph(torch, lambda: sa.sa_additive_attention(qc, None, None, scale, nbits, phases=2, kv=kv, out=o, workspace=ws))
            sk = torch.sign(torch.randn((batch, H, n_tok, nbits), device="cuda"))             # +-1 as floats: the dense operands
            sq = torch.sign(torch.randn((batch, H, n_tok, nbits), device="cuda"))
            vh = v.permute(0, 2, 1, 3).contiguous()
            kvd = torch.empty((batch, H, nbits, d), device="cuda")
            od = torch.empty((batch, H, n_tok, d), device="cuda")
            skt = sk.transpose(-1, -2).contiguous()
            d_ktv = _time_us_graph(torch, lambda: torch.matmul(skt, vh, out=kvd))
            d_qkv = _time_us_graph(torch, lambda: torch.matmul(sq, kvd, out=od))
            rows.append(dict(kernel="MatAdd K^T V", batch=batch, stage=si + 1, shape="B%d H%d N%d bits%d dv%d" % (batch, H, n_tok, nbits, d),
                             us=round(t_ktv, 2), dense_f32_us=round(d_ktv, 2), speedup=round(d_ktv / t_ktv, 2)))
            rows.append(dict(kernel="MatAdd Q(K^T V)", batch=batch, stage=si + 1, shape="B%d H%d N%d bits%d dv%d" % (batch, H, n_tok, nbits, d),
                             us=round(t_qkv, 2), dense_f32_us=round(d_qkv, 2), speedup=round(d_qkv / t_qkv, 2)))
            del sk, sq, vh, kvd, od, skt
            # ---- Shift layers: the attention projection and the two MLP layers
            M = batch * n_tok
            for name, K, N in (("attn proj", E, E), ("mlp fc1", E, ratio * E), ("mlp fc2", ratio * E, E)):
                x8 = torch.from_numpy(g.integers(-127, 128, size=(M, K), dtype=np.int8)).cuda()
                neg = g.integers(0, 2, size=(N, K), dtype=np.uint8)
                e = g.integers(0, 8, size=(N, K), dtype=np.uint8)
                w4 = torch.from_numpy(wl.pack_w4(neg, e)).cuda()
                y32 = torch.empty((M, N), dtype=torch.int32, device="cuda")
                # vector-ALU shift-and-accumulate; matrix cores with the 4-bit weights decoded in every call (two launches);
                # matrix cores on planes decoded once beforehand
                variants = {"valu": (0, w4), "mfma": (1, w4), "mfma_prepared": (3, sa.sa_shift_planes_prepare(w4))}
                t = {}
                for vn, (vid, wv) in variants.items():
                    wsl = torch.empty(max(16, lib.sa_shift_linear_workspace_bytes(sa._l(M), K, N, vid)), dtype=torch.uint8, device="cuda")
                    t[vn] = _time_us_graph(torch, lambda: sa.sa_shift_linear(x8, wv, variant=vid, y=y32, workspace=wsl),
                                           reps=5 if vn == "valu" else 20)
                xf = x8.float()
                wf = torch.from_numpy((np.where(neg == 1, -1.0, 1.0) * np.exp2(e.astype(np.float64))).astype(np.float32)).cuda().t().contiguous()
                yf = torch.empty((M, N), device="cuda")
                dense = _time_us_graph(torch, lambda: torch.matmul(xf, wf, out=yf))
                best = min(t.values())
                rows.append(dict(kernel="MatShift " + name, batch=batch, stage=si + 1, shape="M%d K%d N%d" % (M, K, N),
                                 us=round(best, 2), us_by_variant={k_: round(v_, 2) for k_, v_ in t.items()},
                                 dense_f32_us=round(dense, 2), speedup=round(dense / best, 2)))
                del x8, w4, y32, xf, wf, yf
    print("| kernel | batch | stage | shape | ours us | dense fp32 us | ratio |", file=sys.stderr)
    print("|---|---|---|---|---|---|---|", file=sys.stderr)
    for r in rows:
        print("| %s | %d | %d | %s | %s | %s | %.2f |" % (r["kernel"], r["batch"], r["stage"], r["shape"], r["us"], r["dense_f32_us"], r["speedup"]),
              file=sys.stderr)

    def geo(kind, batch):
        sel = [r["speedup"] for r in rows if r["kernel"].startswith(kind) and r["batch"] == batch]
        return round(math.exp(sum(math.log(x) for x in sel) / len(sel)), 2)

    summary = {"MatAdd_vs_dense_f32": {"batch1": geo("MatAdd", 1), "batch32": geo("MatAdd", 32)},
               "MatShift_vs_dense_f32": {"batch1": geo("MatShift", 1), "batch32": geo("MatShift", 32)}}
    out = {"metric": "kernel sweep over pyramid-ViT stage shapes: geometric-mean speed-up over a dense fp32 library GEMM",
           "value": summary["MatShift_vs_dense_f32"]["batch32"], "unit": "x (MatShift, batch 32)", "n_gpus": 1, "steps": steps,
           "warmup": 3, "ms_per_step": None, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "f32 adds on u64 codes; i8 x 4-bit -> i32", "data": "synthetic",
           "config": {"workload": "pyramid-vit-stage-sweep", "stages": [list(s_) for s_ in PYRAMID_STAGES], "batches": [1, 32],
                      "code_bits": nbits},
           "summary": summary, "sweep": rows, "roofline": None, "cpu_baseline": None}
    print(json.dumps(out))


def bench_shift_linear(args, sa, wl, torch, np):
    """Config 3: the two shift linear layers at DeiT-Small shapes, alone, VALU and matrix-core variants."""
    M = wl.C3_M
    rows = []
    total_us = {0: 0.0, 1: 0.0}
    for li, (K, N) in enumerate(wl.C3_SHAPES):
        x = torch.from_numpy(wl.int8_activations(3, M, K, extra=li)).cuda()
        w4 = torch.from_numpy(wl.shift_weights(3, 4 + li, N, K)).cuda()
        n_sets = 4
        ys = [torch.empty((M, N), dtype=torch.int32, device="cuda") for _ in range(n_sets)]
        lib = sa.load_library()
        for variant in (1, 0):
            ws = torch.empty(max(16, lib.sa_shift_linear_workspace_bytes(sa._l(M), K, N, variant)), dtype=torch.uint8,
                             device="cuda")
            steps = args.steps if variant == 1 else max(3, args.steps // 10)
            for y in ys:
                sa.sa_shift_linear(x, w4, variant=variant, y=y, workspace=ws)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for i in range(steps):
                sa.sa_shift_linear(x, w4, variant=variant, y=ys[i % n_sets], workspace=ws)
            e1.record()
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) * 1e3 / steps
            total_us[variant] += us
            nbytes = M * K + K * N // 2 + 4 * M * N                  # int8 in, 4-bit weights, int32 out
            ops = 2 * M * K * N
            comp = "mfma_i8" if variant == 1 else "alu_int"
            t_hbm, t_cmp = nbytes / (HBM_PEAK_GBS * 1e9) * 1e6, ops / (PEAK_TFLOPS[comp] * 1e12) * 1e6
            rows.append(dict(name="shift_%dx%d_%s" % (K, N, "mfma" if variant == 1 else "valu"), us=round(us, 2), bytes=nbytes,
                             ops=ops, hbm_floor_us=round(t_hbm, 2), compute_floor_us=round(t_cmp, 2),
                             bound="hbm" if t_hbm >= t_cmp else ("mfma" if variant == 1 else "alu"), compute_peak=comp,
                             hbm_frac=round(t_hbm / us, 4), binding_frac=round(max(t_hbm, t_cmp) / us, 4)))
    dom = max((r for r in rows if r["name"].endswith("mfma")), key=lambda r: r["us"])
    roofline = dict(kernel=dom["name"], bound=dom["bound"], achieved=round(dom["bytes"] / (dom["us"] * 1e-6) / 1e9, 3),
                    peak=HBM_PEAK_GBS, unit="GB/s", frac=dom["hbm_frac"], traffic=None, us_per_launch=dom["us"])
    ms = total_us[1] * 1e-3
    out = {"metric": "shift linear tokens/s (both layers, int8 matrix-core variant) at 1 GPU; % HBM roofline",
           "value": round(M / (ms * 1e-3), 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": round(ms, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "i8 x 4-bit -> i32", "data": "synthetic",
           "config": {"workload": "c3-deit-small-shift-linear", "M": M, "layers": [list(s) for s in wl.C3_SHAPES]},
           "valu_variant_ms_per_step": round(total_us[0] * 1e-3, 5), "roofline": roofline, "cpu_baseline": None,
           "kernels": rows}
    print(json.dumps(out))


def bench_zero_one(args, sa, wl, torch, np, cfg):
    """Hash Q and K, linear attention on {0,1} codes with its normaliser, depthwise 3x3 on V added to the output."""
    gh = int(round(math.sqrt(cfg.N)))
    assert gh * gh == cfg.N, "--zero-one needs a square token grid (c2: 56 x 56, c5: 128 x 128)"
    B, N, H, d, dv, nbits = cfg.B, cfg.N, cfg.H, cfg.d, cfg.dv, cfg.nbits
    E = H * dv
    q, k, v = wl.qkv(cfg)
    rng = np.random.default_rng([cfg.cfg_id, 40])
    wconv = (rng.standard_normal((E, 3, 3)) / 3.0).astype(np.float32)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    pr, dw = dev(wl.proj(cfg)), dev(wconv)
    n_sets = args.rotate or max(2, min(8, math.ceil(600e6 / (4 * q.nbytes))))
    sets = []
    lib = sa.load_library()
    for _ in range(n_sets):
        dq, dk, dv_ = dev(q), dev(k), dev(v)
        sets.append(dict(q=dq, k=dk, v=dv_, qc=torch.empty((B, H, N, nbits // 64), dtype=torch.int64, device="cuda"),
                         kc=torch.empty((B, H, N, nbits // 64), dtype=torch.int64, device="cuda"),
                         kv=torch.empty((B, H, nbits, dv), dtype=torch.float32, device="cuda"),
                         ksum=torch.empty((B, H, nbits), dtype=torch.int32, device="cuda"),
                         o=torch.empty((B, N, H, dv), dtype=torch.float32, device="cuda"),
                         ws=torch.empty(max(16, lib.sa_linear_attention_01_workspace_bytes(B, H, N, N, nbits, dv)),
                                        dtype=torch.uint8, device="cuda")))
    eps = 1.0
    stages = [
        ("binarize_qk", lambda s: sa.sa_binarize_pair(s["q"], s["k"], pr, nbits, q_codes=s["qc"], k_codes=s["kc"])),
        ("ktv01_counts", lambda s: sa.sa_linear_attention_01(None, s["kc"], s["v"], eps, nbits, phases=1, kv=s["kv"], ksum=s["ksum"],
                                                             workspace=s["ws"])),
        ("qkv01_normalised", lambda s: sa.sa_linear_attention_01(s["qc"], None, None, eps, nbits, phases=2, kv=s["kv"], ksum=s["ksum"],
                                                                 out=s["o"], workspace=s["ws"])),
        ("dwconv3x3_add", lambda s: sa.sa_dwconv3x3(s["v"].view(B, gh, gh, E), dw, None, out=s["o"].view(B, gh, gh, E), accumulate=True)),
    ]

    def step(s):
        for _, fn in stages:
            fn(s)

    for i in range(args.warmup):
        step(sets[i % n_sets])
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(sets[i % n_sets])
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    rows = B * N * H
    code_b, v_b, kv_b = rows * nbits // 8, rows * dv * 4, B * H * nbits * dv * 4
    algo = {"binarize_qk": (2 * (rows * d * 4 + code_b) + d * nbits * 4, 4 * rows * nbits * d, "mfma_bf16x3"),
            "ktv01_counts": (2 * code_b + v_b + kv_b, 2 * rows * nbits * dv, "mfma_bf16x3"),
            "qkv01_normalised": (2 * code_b + kv_b + v_b, 2 * rows * nbits * dv, "mfma_bf16x3"),
            "dwconv3x3_add": (3 * v_b, 18 * rows * dv, "alu_fp32")}
    report = []
    for name, fn in stages:
        us = None
        if not args.no_kernels:
            for s_ in sets:
                fn(s_)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for i in range(args.steps):
                fn(sets[i % n_sets])
            e1.record()
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) * 1e3 / args.steps
        nbytes, ops, comp = algo[name]
        t_hbm, t_cmp = nbytes / (HBM_PEAK_GBS * 1e9) * 1e6, ops / (PEAK_TFLOPS[comp] * 1e12) * 1e6
        row = dict(name=name, us=None if us is None else round(us, 2), bytes=nbytes, ops=ops, hbm_floor_us=round(t_hbm, 2),
                   compute_floor_us=round(t_cmp, 2), bound="hbm" if t_hbm >= t_cmp else ("mfma" if comp.startswith("mfma") else "alu"),
                   compute_peak=comp)
        if us:
            row.update(hbm_frac=round(t_hbm / us, 4), binding_frac=round(max(t_hbm, t_cmp) / us, 4))
        report.append(row)
    roofline = None
    timed = [r for r in report if r["us"]]
    if timed:
        dom = max(timed, key=lambda r: r["us"])
        roofline = dict(kernel=dom["name"], bound=dom["bound"], achieved=round(dom["bytes"] / (dom["us"] * 1e-6) / 1e9, 3),
                        peak=HBM_PEAK_GBS, unit="GB/s", frac=dom["hbm_frac"], traffic=None, us_per_launch=dom["us"])
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        oracle.build()
        bs = min(cfg.B, args.cpu_sample_batch or 1)
        t0 = time.perf_counter()
        qc = oracle.binarize(q[:bs], wl.proj(cfg), nbits)
        kc = oracle.binarize(k[:bs], wl.proj(cfg), nbits)
        oracle.linear_attention_01(qc, kc, v[:bs], nbits, eps)
        oracle.dwconv3x3(v[:bs].reshape(bs, gh, gh, E), wconv)
        dt = time.perf_counter() - t0
        cpu = {"value": round(bs * N / dt, 1), "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
               "sample": "%d of %d batch items (%d tokens)" % (bs, B, bs * N)}
    total_bytes = sum(r["bytes"] for r in report)
    out = {"metric": "tokens/s of hash + normalised linear attention on {0,1} codes + depthwise conv on V at 1 GPU; % HBM roofline",
           "value": round(B * N / (ms_per_step * 1e-3), 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
           "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": "f32+u64 codes", "data": "synthetic",
           "config": {"workload": cfg.name + "-zero-one-normalised", "B": B, "N": N, "H": H, "d": d, "nbits": nbits, "dv": dv,
                      "grid": [gh, gh], "input_sets_rotated": n_sets},
           "hbm_roofline_frac": round(total_bytes / (ms_per_step * 1e-3) / (HBM_PEAK_GBS * 1e9), 4),
           "algorithmic_bytes": total_bytes, "roofline": roofline, "cpu_baseline": cpu, "kernels": report}
    print(json.dumps(out))


def bench_layer(args, sa, wl, torch, np, cfg):
    """The complete block of Eq. 2 (sa_layer_forward) and each of its kernels through the stage entry points."""
    assert cfg.E, "--layer needs a configuration with an MLP (c1, c4, c5)"
    if args.sign_hash:
        import dataclasses
        cfg = dataclasses.replace(cfg, nbits=cfg.E // cfg.H, name=cfg.name + "-sign-hash")
    T, E, H, hid = cfg.T, cfg.E, cfg.H, cfg.hid
    moe = cfg.shift_frac is not None
    lp, p = wl.layer_params(cfg), wl.mlp_params(cfg)
    scale = wl.attention_scale(cfg)

    def dev(a):
        return torch.from_numpy(np.ascontiguousarray(a)).cuda()

    var = args.shift_variant
    ws_ = [dev(np.concatenate([lp.wq, lp.wk, lp.wv], axis=0)), dev(lp.wo), dev(p.w1), dev(p.w2)]
    if var == 3:
        ws_ = [sa.sa_shift_planes_prepare(w) for w in ws_]
    wqkv, wo, w1, w2 = ws_
    shared = dict(B=cfg.B, N=cfg.N, H=H, nbits=cfg.nbits, E=E, hid=hid, attention=0 if cfg.attention == "linear" else 1,
                  moe=int(moe), shift_variant=var, eps=lp.eps, ln_inv_scale=lp.ln_inv_scale, qkv_scale=lp.qkv_scale,
                  attn_scale=scale, act_inv_scale=p.act_inv_scale, o_scale=lp.o_scale, requant_scale=p.requant_scale,
                  out_scale=p.out_scale, gamma1=dev(lp.gamma1), beta1=dev(lp.beta1), gamma2=dev(lp.gamma2),
                  beta2=dev(lp.beta2), wqkv=wqkv, wo=wo, proj=None if args.sign_hash else dev(wl.proj(cfg)), w1=w1, w2=w2,
                  lut=dev(p.lut))
    if moe:
        shared.update(wg=dev(lp.wg), bg=dev(lp.bg), mw1=dev(p.mw1), mw2=dev(p.mw2))
    x_host = wl.layer_input(cfg)
    n_sets = args.rotate or max(2, min(8, math.ceil(600e6 / (10 * x_host.nbytes))))
    n_sets = (n_sets + args.streams - 1) // args.streams * args.streams
    layers = [sa.Layer(x=dev(x_host), **shared) for _ in range(n_sets)]
    run_steps = make_step_runner(torch, args.streams, n_sets, lambda i: layers[i].forward())
    settle(torch, run_steps, args.settle_ms)
    run_steps(args.warmup)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run_steps(args.steps)
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps

    # ---- per kernel, through the stage entry points on one buffer set (the chain of the layer)
    x = layers[0]._keep[0]
    B, N, d = cfg.B, cfg.N, E // H
    z8 = torch.empty((T, E), dtype=torch.int8, device="cuda")
    q, k, v, x1 = (torch.empty((T, E), dtype=torch.float32, device="cuda") for _ in range(4))
    q4, k4, v4 = (t.view(B, N, H, d) for t in (q, k, v))
    qc = torch.empty((B, H, N, cfg.nbits // 64), dtype=torch.int64, device="cuda")
    kc = torch.empty_like(qc)
    lib = sa.load_library()
    lin_ws = torch.empty(max(16, lib.sa_shift_linear_workspace_bytes(sa._l(T), E, 3 * E, var)), dtype=torch.uint8, device="cuda")
    n_shift = int(math.floor(cfg.shift_frac * T + 0.5)) if moe else T
    n_mult = T - n_shift
    rows = T * H
    code_b, v_b = rows * cfg.nbits // 8, rows * d * 4
    stages = []

    def add(name, fn, nbytes, ops, comp):
        stages.append((name, fn, nbytes, ops, comp))

    add("ln1_quant", lambda: sa.sa_layernorm_quant(x, shared["gamma1"], shared["beta1"], lp.eps, lp.ln_inv_scale,
                                                   want_ln=False, q=z8), T * E * 5, 8 * T * E, "alu_fp32")
    if args.sign_hash and var != 0:
        add("qkv_linear_codes", lambda: sa.sa_shift_linear_qkv_codes(z8, wqkv, B, N, H, lp.qkv_scale, variant=var, workspace=lin_ws, q_codes=qc,
                                                                     k_codes=kc, v=v),
            T * E + 3 * E * E // 2 + T * E * 4 + 2 * code_b, 2 * T * E * 3 * E, "mfma_i8")
    else:
        add("qkv_linear", lambda: sa.sa_shift_linear_f32(z8, wqkv, lp.qkv_scale, parts=3, variant=var, ys=(q, k, v), workspace=lin_ws),
            T * E + 3 * E * E // 2 + 3 * T * E * 4, 2 * T * E * 3 * E, "mfma_i8")
        add("binarize_qk", lambda: sa.sa_binarize_pair(q4, k4, shared["proj"], cfg.nbits, q_codes=qc, k_codes=kc),
            2 * (rows * d * 4 + code_b) + (d * cfg.nbits * 4 if shared["proj"] is not None else 0),
            4 * rows * cfg.nbits * d if shared["proj"] is not None else 2 * rows * d, "mfma_bf16x3")
    o = torch.empty((B, N, H, d), dtype=torch.float32, device="cuda")
    if cfg.attention == "linear":
        kv = torch.empty((B, H, cfg.nbits, d), dtype=torch.float32, device="cuda")
        aws = torch.empty(max(16, lib.sa_additive_attention_workspace_bytes(B, H, N, cfg.nbits, d)), dtype=torch.uint8, device="cuda")
        kv_b = B * H * cfg.nbits * d * 4
        add("ktv", lambda: sa.sa_additive_attention(None, kc, v4, scale, cfg.nbits, phases=1, kv=kv, workspace=aws),
            code_b + v_b + kv_b, 2 * rows * cfg.nbits * d, "mfma_bf16x3")
        add("qkv", lambda: sa.sa_additive_attention(qc, None, None, scale, cfg.nbits, phases=2, kv=kv, out=o, workspace=aws),
            code_b + v_b + kv_b, 2 * rows * cfg.nbits * d, "mfma_bf16x3")
        add("quantize", lambda: sa.sa_quantize_act(o.view(T, E), p.act_inv_scale, q=z8), T * E * 5, 2 * T * E, "alu_fp32")
    else:
        add("hamming", lambda: sa.sa_hamming_attention_fused(qc, kc, v4, scale, cfg.nbits, p.act_inv_scale, xq=z8, want_xh=False,
                                                             want_out=False),
            2 * code_b + v_b + T * E, 2 * B * H * N * N * d, "mfma_bf16x3")
    add("o_linear", lambda: sa.sa_shift_linear_f32(z8, wo, lp.o_scale, residual=x, variant=var, ys=(x1,), workspace=lin_ws),
        T * E + E * E // 2 + 2 * T * E * 4, 2 * T * E * E, "mfma_i8")
    xh = torch.empty((T, E), dtype=torch.float16, device="cuda") if moe else None
    logits = torch.empty((T, 2), dtype=torch.float32, device="cuda") if moe else None
    add("ln2_quant_router", lambda: sa.sa_layernorm_quant(x1, shared["gamma2"], shared["beta2"], lp.eps, lp.ln_inv_scale,
                                                          want_ln=False, q=z8, xh=xh, wg=shared.get("wg"),
                                                          bg=shared.get("bg"), logits=logits),
        T * E * (5 + (2 if moe else 0)) + (T * 8 if moe else 0), (8 + (4 if moe else 0)) * T * E, "alu_fp32")
    acc = sa.SA_MLP_ACCUMULATE
    sws = torch.empty(max(16, lib.sa_shift_mlp_workspace_bytes(sa._l(T), E, hid)), dtype=torch.uint8, device="cuda")
    if moe:
        disp = None
        perm = torch.empty(T, dtype=torch.int32, device="cuda")
        eo = torch.empty(T, dtype=torch.int32, device="cuda")
        cnt = torch.empty(4, dtype=torch.int32, device="cuda")[:2]
        gate = torch.empty(T, dtype=torch.float32, device="cuda")
        dws = torch.empty(max(16, lib.sa_moe_dispatch_workspace_bytes(sa._l(T), 2)), dtype=torch.uint8, device="cuda")
        mws = torch.empty(max(16, lib.sa_mult_mlp_workspace_bytes(sa._l(T), E, hid)), dtype=torch.uint8, device="cuda")
        add("dispatch", lambda: sa.sa_moe_dispatch(logits, out=(perm, eo, cnt, gate), workspace=dws), T * 20, 4 * T, "alu_fp32")
        for st_, nm in ((1, "mult_fc1"), (2 | acc, "mult_fc2")):
            add(nm, (lambda st_=st_: sa.sa_mult_mlp_f16_half(xh, shared["mw1"], shared["mw2"], rows=perm, counts=cnt, expert=0,
                                                            max_rows=T, want_out=False, y=x1, gate=gate, stages=st_, workspace=mws)),
                n_mult * E * 2 + E * hid * 2 + n_mult * hid * 2 + (n_mult * E * 6 if st_ != 1 else 0), 2 * n_mult * E * hid, "mfma_f16")
        sel = dict(rows=perm, counts=cnt, expert=1, max_rows=T, gate=gate)
    else:
        sel = {}
    for st_, nm in ((1, "shift_fc1"), (2 | acc, "shift_fc2")):
        add(nm, (lambda st_=st_: sa.sa_shift_mlp(z8, w1, w2, p.requant_scale, shared["lut"], want_y2=False, y=x1,
                                                out_scale=p.out_scale, variant=var, stages=st_, workspace=sws, **sel)),
            n_shift * (E + hid) + E * hid // 2 + (n_shift * E * 7 if st_ != 1 else 0), 2 * n_shift * E * hid, "mfma_i8")

    report = []
    for name, fn, nbytes, ops, comp in stages:
        fn()
        us = None
        if not args.no_kernels:
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(args.steps):
                fn()
            e1.record()
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) * 1e3 / args.steps
        t_hbm, t_cmp = nbytes / (HBM_PEAK_GBS * 1e9) * 1e6, ops / (PEAK_TFLOPS[comp] * 1e12) * 1e6
        row = dict(name=name, us=None if us is None else round(us, 2), bytes=nbytes, ops=ops, hbm_floor_us=round(t_hbm, 2),
                   compute_floor_us=round(t_cmp, 2), bound="hbm" if t_hbm >= t_cmp else ("mfma" if comp.startswith("mfma") else "alu"),
                   compute_peak=comp)
        if us:
            row.update(hbm_frac=round(t_hbm / us, 4), binding_frac=round(max(t_hbm, t_cmp) / us, 4))
        report.append(row)
    roofline = None
    timed = [r for r in report if r["us"]]
    if timed:
        dom = max(timed, key=lambda r: r["us"])
        if dom["bound"] == "hbm":
            ach, peak, unit = dom["bytes"] / (dom["us"] * 1e-6) / 1e9, HBM_PEAK_GBS, "GB/s"
        else:
            ach, peak, unit = dom["ops"] / (dom["us"] * 1e-6) / 1e12, PEAK_TFLOPS[dom["compute_peak"]], "TFLOP/s"
        roofline = dict(kernel=dom["name"], bound=dom["bound"], achieved=round(ach, 3), peak=peak, unit=unit,
                        frac=round(ach / peak, 4), traffic=None, us_per_launch=dom["us"])
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        oracle.build()
        bs = args.cpu_sample_batch or {1: 1, 4: 16, 5: 1}.get(cfg.cfg_id, 1)
        small = wl.scaled_down(cfg, B=min(bs, cfg.B))
        xs = x_host[: small.T]
        t0 = time.perf_counter()
        oracle.layer_forward(small, xs, lp, p, None if args.sign_hash else wl.proj(cfg), scale)
        dt = time.perf_counter() - t0
        cpu = {"value": round(small.T / dt, 1), "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
               "sample": "%d of %d batch items (%d tokens), one pass of oracle.layer_forward" % (small.B, cfg.B, small.T)}
    layer_bytes = sum(r["bytes"] for r in report)
    out = {"metric": "layer tokens/s (complete block of Eq. 2: LayerNorms, shift Linears, attention, MoE, residuals) at 1 GPU; % HBM roofline",
           "value": round(T / (ms_per_step * 1e-3), 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
           "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": "f32+u64 codes+i8/i32 shift+f16 mult", "data": "synthetic",
           "config": {"workload": cfg.name.replace("block", "layer"), "B": cfg.B, "N": cfg.N, "H": H, "nbits": cfg.nbits, "E": E,
                      "hid": hid, "attention": cfg.attention, "mlp": "moe" if moe else "shift", "input_sets_rotated": n_sets,
                      "shift_variant": var, "streams": args.streams, "settle_ms": args.settle_ms},
           "layer_hbm_roofline_frac": round(layer_bytes / (ms_per_step * 1e-3) / (HBM_PEAK_GBS * 1e9), 4),
           "layer_algorithmic_bytes": layer_bytes, "roofline": roofline, "cpu_baseline": cpu, "kernels": report}
    print(json.dumps(out))


def make_stages(sa, torch, cfg, kw, p, moe, variant):
    """One callable per kernel of the block, on buffers of its own (same shapes as the block's)."""
    T, E = cfg.T, cfg.E
    d = kw["q"].device
    qc = torch.empty((cfg.B, cfg.H, cfg.N, cfg.W), dtype=torch.int64, device=d)
    kc = torch.empty_like(qc)
    o = torch.empty((cfg.B, cfg.N, cfg.H, cfg.dv), dtype=torch.float32, device=d)
    lib = sa.load_library()
    st = {"binarize_qk": lambda: sa.sa_binarize_pair(kw["q"], kw["k"], kw["proj"], cfg.nbits, q_codes=qc, k_codes=kc)}
    if cfg.attention == "linear":
        kv = torch.empty((cfg.B, cfg.H, cfg.nbits, cfg.dv), dtype=torch.float32, device=d)
        ws = torch.empty(max(16, lib.sa_additive_attention_workspace_bytes(cfg.B, cfg.H, cfg.N, cfg.nbits, cfg.dv)),
                         dtype=torch.uint8, device=d)
        st["ktv"] = lambda: sa.sa_additive_attention(None, kc, kw["v"], kw["attn_scale"], cfg.nbits, phases=1,
                                                     kv=kv, workspace=ws)
        st["qkv"] = lambda: sa.sa_additive_attention(qc, None, None, kw["attn_scale"], cfg.nbits, phases=2,
                                                     kv=kv, out=o, workspace=ws)
        st["ktv_valu"] = lambda: sa.sa_additive_attention(None, kc, kw["v"], kw["attn_scale"], cfg.nbits, phases=1 | 4,
                                                          kv=kv, workspace=ws)
        st["qkv_valu"] = lambda: sa.sa_additive_attention(qc, None, None, kw["attn_scale"], cfg.nbits, phases=2 | 4,
                                                          kv=kv, out=o, workspace=ws)
    x = o.view(T, E) if E else None
    xq = torch.empty((T, E), dtype=torch.int8, device=d) if E else None
    xh = torch.empty((T, E), dtype=torch.float16, device=d) if (E and moe) else None
    if cfg.attention != "linear":
        if E:       # as in the block: the kernel also leaves the forms the MLP reads
            st["hamming"] = lambda: sa.sa_hamming_attention_fused(qc, kc, kw["v"], kw["attn_scale"], cfg.nbits,
                                                                  p.act_inv_scale, out=o, xq=xq, xh=xh,
                                                                  want_xh=False)
        else:
            st["hamming"] = lambda: sa.sa_hamming_attention(qc, kc, kw["v"], kw["attn_scale"], cfg.nbits, out=o)
    if not E:
        return st
    y = torch.empty((T, E), dtype=torch.float32, device=d)
    if cfg.attention == "linear":
        if moe:
            st["quantize"] = lambda: sa.sa_quantize_act_half(x, p.act_inv_scale, q=xq, xh=xh)
        else:
            st["quantize"] = lambda: sa.sa_quantize_act(x, p.act_inv_scale, q=xq)
    sws = torch.empty(max(16, lib.sa_shift_mlp_workspace_bytes(sa._l(T), E, cfg.hid)), dtype=torch.uint8, device=d)
    rows = dict()
    if moe:
        outs = (torch.empty(T, dtype=torch.int32, device=d), torch.empty(T, dtype=torch.int32, device=d),
                torch.empty(4, dtype=torch.int32, device=d)[:2], torch.empty(T, dtype=torch.float32, device=d))
        dws = torch.empty(max(16, lib.sa_moe_dispatch_workspace_bytes(sa._l(T), 2)), dtype=torch.uint8, device=d)
        st["dispatch"] = lambda: sa.sa_moe_dispatch(kw["logits"], out=outs, workspace=dws)
        mws = torch.empty(max(16, lib.sa_mult_mlp_workspace_bytes(sa._l(T), E, cfg.hid)), dtype=torch.uint8, device=d)
        mrows = dict(rows=outs[0], counts=outs[2], expert=0, max_rows=T, gate=outs[3])
        st["mult_fc1"] = lambda: sa.sa_mult_mlp_f16_half(xh, kw["mw1"], kw["mw2"], want_out=False, y=y, stages=1,
                                                         workspace=mws, **mrows)
        st["mult_fc2"] = lambda: sa.sa_mult_mlp_f16_half(xh, kw["mw1"], kw["mw2"], want_out=False, y=y, stages=2,
                                                         workspace=mws, **mrows)
        rows = dict(rows=outs[0], counts=outs[2], expert=1, max_rows=T, gate=outs[3])
    # the two layers alone: with the per-call decode (variant 1 / 2) they are timed on planes made beforehand (the same
    # GEMM kernels on the same planes), and the decode launch by the difference to both layers in one call
    w1, w2, v_layers = kw["w1"], kw["w2"], variant
    if variant in (1, 2):
        w1, w2, v_layers = sa.sa_shift_planes_prepare(kw["w1"]), sa.sa_shift_planes_prepare(kw["w2"]), 3
        st["shift_mlp_both"] = lambda: sa.sa_shift_mlp(xq, kw["w1"], kw["w2"], p.requant_scale, kw["lut"], want_y2=False, y=y,
                                                       out_scale=p.out_scale, variant=variant, stages=3, workspace=sws, **rows)
    for name, stage in (("shift_fc1", 1), ("shift_fc2", 2)):
        st[name] = (lambda stage=stage: sa.sa_shift_mlp(xq, w1, w2, p.requant_scale, kw["lut"],
                                                        want_y2=False, y=y, out_scale=p.out_scale, variant=v_layers,
                                                        stages=stage, workspace=sws, **rows))
    return st


def read_traffic(config, kernel):
    """HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE + WRITE_SIZE), kept as text in
    profiles/; None when no measurement is stored for this kernel and workload."""
    path = os.path.join(ROOT, "profiles", "traffic_%s.txt" % config)
    if not os.path.exists(path):
        return None
    for line in open(path):
        parts = line.split()
        if len(parts) >= 2 and parts[0] == kernel:
            try:
                return int(float(parts[1]))
            except ValueError:
                return None
    return None


def cpu_baseline(cfg, sample_batch):
    """The CPU oracle, as it stands, on a bounded sample of the same workload (same widths, fewer
    batch elements), on this host's cores."""
    import numpy as np

    import oracle
    from paper_2306_06446_amd import workloads as wl

    default = {1: 1, 2: 8, 4: 64, 5: 2}[cfg.cfg_id]      # config 4 whole (about 10 s on 16 cores); 2 and 5 a bounded share
    sb = sample_batch or default
    n = cfg.N if cfg.cfg_id != 5 else 2048
    small = wl.scaled_down(cfg, B=sb, N=n)
    q, k, v = wl.qkv(small)
    pr, scale = wl.proj(small), wl.attention_scale(small)
    p = wl.mlp_params(small) if small.E else None
    logits = wl.router_logits(small) if (small.E and small.shift_frac is not None) else None
    oracle.build()
    t0, c0 = time.perf_counter(), time.process_time()
    oracle.block_forward(small, q, k, v, pr, scale, logits, p)
    dt, cpu_s = time.perf_counter() - t0, time.process_time() - c0
    return {"value": round(small.T / dt, 2), "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": "%s with B=%d, N=%d (%d tokens), one pass, %.2f s wall, %.1f s of CPU time" % (cfg.name, sb, n, small.T, dt, cpu_s)}


if __name__ == "__main__":
    main()
