#!/usr/bin/env python3
"""Benchmark of the IM-attention hot path on one MI355X.

One "step" = one im_attention_fwd + one im_attention_bwd through the C ABI
(schedule, shared QKV projection, live-block scores / softmax / aggregation,
output projection and the whole backward) on one batch of synthetic inputs that
is already resident in HBM.  The headline value is live-block attention
TFLOP/s: (4 + 10) * P * d flops per step, P = number of (valid query, valid live
key) pairs over the batch, divided by the time of the WHOLE step (projections
and weight gradients included in the time, not in the flops).

Prints ONE JSON line.  `roofline` is for the dominant attention kernel of the
step, timed with HIP events recorded by the library on the call's stream over
the timed steps (im_profile_enable); `kernel_frac` gives the same fraction for
every attention kernel and `attn_core_frac` for the three together (separate
pass after the timed region); `cpu_baseline` is the fp64 CPU oracle timed on a
bounded sample of the same workload.  `measured_peaks` are two micro-benchmarks
run in the same process (register-resident MFMA loop, streaming copy);
`--calibrate` prints only those.

Other rows: --config c2|c3|c3p|c3v|c4|c4v|c4train|gsit, --mask <any named
pattern>|info_disorder, --shape mosi|mosei|sims|mintrec (small-model configs).
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# MI355X published peaks
PEAK_HBM_GBS = 8000.0
PEAK_MFMA_BF16_TFLOPS = 2500.0
PEAK_FP32_VALU_TFLOPS = 157.3        # published fp32 vector rate: counts packed (two-wide) fp32 instructions
PEAK_FP32_VALU_UNPACKED_TFLOPS = 78.6  # 256 CU x 64 lanes x 2 flop x 2.4 GHz: the rate of code without packed fp32,
                                       # which is what the library is compiled to (packed fp32 selection is switched off)

# Maximum sequence lengths of the datasets (App. "Datasets"), reordered to text / vision / audio the way the
# benchmark configuration's 50 / 500 / 375 reads the first row.
DATASET_SHAPES = {"mosi": (50, 500, 375), "mosei": (50, 500, 500), "sims": (39, 400, 55), "mintrec": (30, 230, 480)}
# Sec. "Information Disorder": the text rows see two live blocks (vision and audio keys) under ONE softmax
INFO_DISORDER_MASK = (1 << 1) | (1 << 2) | (1 << 5) | (1 << 6)

# MFMA instructions (32x32x16 bf16, 32768 flops each) the kernels execute per 32 x 32 block of scores of one head
MFMA_PER_BLOCK = {64: {"attn_fwd": 8, "attn_dq": 12, "attn_dkv": 16},     # head dim 64
                  0: {"attn_fwd": 3, "attn_dq": 4, "attn_dkv": 6}}        # sub-head mode (head dims 8 / 16)
ALG_COEF = {"attn_fwd": 4.0, "attn_dq": 2.0, "attn_dkv": 8.0}   # algorithmic flops per (pair x model column): forward 4 P d, dQ kernel 2 P d, dK/dV kernel 8 P d


def mask_of(name, B):
    return INFO_DISORDER_MASK if name == "info_disorder" else B.NAMED_MASKS[name]


def pair_counts(seg_len, live_mask, batch, valid_len, key_pad):
    """Integer bookkeeping of the workload: (P_valid, P_rows).  P_valid counts (valid query, valid live key)
    pairs over the batch -- valid lengths on both sides; P_rows counts every query ROW in memory (padding rows
    included) against its valid live keys, which is what the kernels execute with padded rows."""
    import numpy as np
    n = len(seg_len)
    off = np.concatenate([[0], np.cumsum(seg_len)])
    p_valid = p_rows = 0
    for b in range(batch):
        vlen = []
        for j in range(n):
            k = seg_len[j] if valid_len is None else min(seg_len[j], int(valid_len[b, j]))
            if key_pad is not None:
                k = int((key_pad[b, off[j]:off[j] + k] == 0).sum())
            vlen.append(k)
        for i in range(n):
            for j in range(n):
                if (live_mask >> (i * n + j)) & 1:
                    p_valid += vlen[i] * vlen[j]
                    p_rows += seg_len[i] * vlen[j]
    return p_valid, p_rows


def measure(step, args, B, torch, fwd=None, bwd=None):
    """Warm-up; a 3-step probe that finds the dominant attention family; the timed region (EXACTLY args.steps
    steps between synchronisations, only the dominant family bracketed with events -- an event pair costs
    stream time); then, outside the timed region: a pass with one event pair per step (median / min), forward-only
    and backward-only passes, and a pass with every kernel family bracketed (the per-family table)."""
    def profiled(n, only=None, fn=step):
        torch.cuda.synchronize()
        B.im_profile_enable(True, only=only)
        t0 = time.perf_counter()
        for _ in range(n):
            fn()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        B.im_profile_enable(False)
        return (t1 - t0) * 1e3 / n, {k: (v[0] / n, v[1] / n) for k, v in B.im_profile_get().items() if v[1] > 0}

    def per_call(fn, n):
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
        torch.cuda.synchronize()
        for a, b in ev:
            a.record()
            fn()
            b.record()
        torch.cuda.synchronize()
        t = [a.elapsed_time(b) for a, b in ev]
        return statistics.median(t), min(t)

    for _ in range(args.warmup):
        step()
    _, probe = profiled(3)
    cands = [k for k in ("attn_fwd", "attn_dq", "attn_dkv") if k in probe]
    dom = max(cands, key=lambda k: probe[k][0])
    ms_step, timed = profiled(args.steps, only=dom)
    r = {"ms_step": ms_step, "dom": dom}
    r["median"], r["min"] = per_call(step, args.steps)
    if fwd is not None:
        r["fwd_median"], r["fwd_min"] = per_call(fwd, args.steps)
        r["bwd_median"], r["bwd_min"] = per_call(bwd, args.steps)   # reads the tensors the last forward saved
    _, table = profiled(max(3, args.warmup))
    table.update(timed)
    r["per_step"] = {k: v[0] for k, v in table.items()}
    r["launches"] = {k: v[1] for k, v in table.items()}
    return r


def measured_peaks(B, torch, quick=True):
    """What this GPU sustains: a register-resident bf16 MFMA loop (TFLOP/s) and a streaming device copy
    (GB/s, bytes read + bytes written).  Best of a few launches each."""
    sink = torch.zeros(64, dtype=torch.float32, device="cuda")
    iters = 8000   # ~4 ms per launch: shorter loops under-read the sustained rate by up to 10 % (ramp-up)
    best_mfma = 0.0
    for _ in range(4):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        flops = B.im_calibrate_mfma(iters, sink)
        b.record()
        torch.cuda.synchronize()
        best_mfma = max(best_mfma, flops / (a.elapsed_time(b) * 1e-3) / 1e12)
    n = (256 << 20) if quick else (1 << 30)
    src = torch.empty(n, dtype=torch.uint8, device="cuda").fill_(1)
    dst = torch.empty_like(src)
    best_copy = 0.0
    for _ in range(4):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        B.im_calibrate_copy(dst, src)
        b.record()
        torch.cuda.synchronize()
        best_copy = max(best_copy, 2.0 * n / (a.elapsed_time(b) * 1e-3) / 1e9)
    del src, dst
    return {"mfma_bf16_tflops": round(best_mfma, 1), "hbm_copy_gbs": round(best_copy, 1),
            "how": f"im_calibrate_mfma ({iters} x 16 v_mfma_f32_32x32x16_bf16 per wave, 8 waves per CU) and "
                   f"im_calibrate_copy ({n >> 20} MiB, read + write), best of 4 launches each, HIP events"}


def stored_traffic(config, family):
    """(HBM bytes per launch, source note) of the dominant kernel from the committed rocprofv3 counter summary
    profiles/<config>_<family>_traffic.md -- NOT measured in this run; (None, None) if there is no summary or the
    kernel sources changed since the counters were taken."""
    import re
    from bench_traffic import source_hash
    rel = os.path.join("profiles", f"{config}_{family}_traffic.md")
    try:
        m = re.search(r"^TRAFFIC_JSON (.*)$", open(os.path.join(ROOT, rel)).read(), flags=re.M)
        rec = json.loads(m.group(1))
        if source_hash(rec["kernel"]) != rec["source_sha256"]:
            return None, None
        return rec["bytes_per_launch"], f"from {rel} (rocprofv3 FETCH_SIZE / WRITE_SIZE of an earlier run; kernel-source hash matched), not measured in this run"
    except Exception:
        return None, None


def host_threads():
    try:
        from threadpoolctl import threadpool_info
        return max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        return os.cpu_count() or 1


def attention_fracs(per_step, launches, P_exec, d, dh, bf16_mfma, peaks):
    """Per attention kernel: algorithmic flops per launch / average launch time, against the roofline of the
    path.  P_exec = pairs the kernels execute (query rows in memory x valid live keys)."""
    out = {}
    sub = MFMA_PER_BLOCK[64 if dh == 64 else 0]
    for k in ("attn_fwd", "attn_dq", "attn_dkv"):
        if k not in per_step:
            continue
        alg = ALG_COEF[k] * P_exec * d
        tf = alg / (per_step[k] * 1e-3) / 1e12
        e = {"ms": round(per_step[k], 4), "alg_tflops": round(tf, 2)}
        if bf16_mfma:
            exe = sub[k] * 32768.0 * (P_exec * (d // dh)) / 1024.0
            e["frac"] = round(tf / PEAK_MFMA_BF16_TFLOPS, 4)
            e["executed_mfma_tflops"] = round(exe / (per_step[k] * 1e-3) / 1e12, 2)
            e["executed_frac"] = round(exe / (per_step[k] * 1e-3) / 1e12 / PEAK_MFMA_BF16_TFLOPS, 4)
            e["useful_mfma_frac"] = round(alg / exe, 4)
            if peaks:
                e["frac_of_measured_peak"] = round(tf / peaks["mfma_bf16_tflops"], 4)
        else:
            e["frac"] = round(tf / PEAK_FP32_VALU_UNPACKED_TFLOPS, 4)
            e["frac_of_published_peak"] = round(tf / PEAK_FP32_VALU_TFLOPS, 4)
        out[k] = e
    return out


def roofline_of(dom, fr, bf16_mfma, peaks, traffic, traffic_src, dom_launches, sub_head):
    e = fr[dom]
    if bf16_mfma:
        roof = {"bound": "mfma", "kernel": dom, "achieved": e["alg_tflops"], "peak": PEAK_MFMA_BF16_TFLOPS, "unit": "TFLOP/s",
                "frac": e["frac"], "traffic": traffic, "traffic_source": traffic_src,
                "avg_launch_ms": round(e["ms"] / max(dom_launches, 1.0), 4),
                "executed_mfma_tflops": e["executed_mfma_tflops"], "useful_mfma_frac": e["useful_mfma_frac"]}
        if "frac_of_measured_peak" in e:
            roof["frac_of_measured_peak"] = e["frac_of_measured_peak"]
            roof["measured_peak"] = peaks["mfma_bf16_tflops"]
        if sub_head:
            roof["note"] = ("head dims 8 / 16 run on the matrix cores in sub-head mode: a head is a slice of a 64-column group, "
                            "so only useful_mfma_frac of every MFMA is algorithmic work; `achieved` counts algorithmic flops, "
                            "`executed_mfma_tflops` the flops the matrix cores execute")
    else:
        roof = {"bound": "alu", "kernel": dom, "achieved": e["alg_tflops"], "peak": PEAK_FP32_VALU_UNPACKED_TFLOPS,
                "unit": "TFLOP/s", "frac": e["frac"], "frac_of_published_peak": e["frac_of_published_peak"],
                "traffic": traffic, "traffic_source": traffic_src,
                "avg_launch_ms": round(e["ms"] / max(dom_launches, 1.0), 4),
                "note": "row-per-lane fp32 kernels: fused multiply-adds of the products counted, exp and softmax bookkeeping "
                        "not; peak = fp32 vector rate without packed instructions (256 CU x 64 lanes x 2 flop x 2.4 GHz), "
                        "the published 157.3 TFLOP/s assumes packed fp32, which the library is compiled without"}
    return roof


def bench_encoder(args, whole_model):
    """--config c4 / c4v: the 4-layer encoder forward (layer = pre-LN IM attention + GELU MLP) at the C4 shapes
    (c4v: with C3's per-sample valid lengths); --config gsit: the whole GsiT forward (two IFM encoders, feature
    concat, IEM encoder at width 2d, last steps, final linear) at the same shapes.  Forward only."""
    import numpy as np
    import torch
    from paper_2505_01068_amd import binding as B, synth

    torch.cuda.set_device(0)
    over = {}
    if args.shape:
        over["seg_len"] = DATASET_SHAPES[args.shape]
    if args.config == "c4v":
        over["padding"] = "valid_len"
    w = synth.workload("c4", **over)
    g = synth.attention_inputs(**{**w, "with_dy": False})
    dtype, tdt = g["dtype"], torch.bfloat16
    Bsz, T, d = g["x"].shape
    H, L, d_ff, seg = g["n_heads"], w["n_layers"], w["d_ff"], g["seg_len"]

    def dev(a):
        if a is None:
            return None
        t = torch.from_numpy(np.ascontiguousarray(a))
        return (t.to(tdt) if t.dtype == torch.float32 else t).cuda()

    x, vl = dev(g["x"]), dev(g["valid_len"])
    if whole_model:
        m = synth.model_params(d, d_ff, 2 * d_ff, L, L, len(seg), 1, w["seed"], dtype=dtype)
        conv = lambda layers: [{k: dev(v) for k, v in p.items()} for p in layers]
        md = {"fwd_layers": conv(m["fwd_layers"]), "bwd_layers": conv(m["bwd_layers"]),
              "intra_layers": conv(m["intra_layers"]), "wf": dev(m["wf"]), "bf": dev(m["bf"])}
        scale_intra = 1.0 / np.sqrt(2 * d / H)
        shape = B.make_shape(Bsz, seg, d, H, 0, g["scale"], dtype)
        model = B.make_model(md, d_ff, 2 * d_ff, H, scale_intra)
        ws = torch.empty(B.gsit_model_sizes(shape, model), dtype=torch.uint8, device="cuda")
        out_t = torch.empty(Bsz, 1, dtype=tdt, device="cuda")

        def step():
            B.gsit_model_fwd(shape, model, x, valid_len=vl, out=out_t, workspace=ws)
        lm_list = [(B.IM_IFM_FORWARD, d, L), (B.IM_IFM_BACKWARD, d, L), (B.IM_IEM, 2 * d, L)]
        label = (f"gsit: whole model forward, B={Bsz} L_t/L_v/L_a={'/'.join(map(str, seg))} d={d} H={H} bf16, "
                 f"{L}+{L} IFM layers, {L} IEM layers at width {2 * d}, padding={w['padding']}")
    else:
        lm = mask_of(args.mask, B)
        layers = [{k: dev(v) for k, v in synth.layer_params(d, d_ff, w["seed"], l, dtype=dtype).items()} for l in range(L)]
        shape = B.make_shape(Bsz, seg, d, H, lm, g["scale"], dtype)
        ws = torch.empty(B.gsit_layer_sizes(shape, d_ff), dtype=torch.uint8, device="cuda")
        bufs = [torch.empty_like(x), torch.empty_like(x)]

        def step():
            h = x
            for l, p in enumerate(layers):
                h = B.gsit_layer_fwd(shape, d_ff, h, p, valid_len=vl, y=bufs[l & 1], workspace=ws)
        lm_list = [(lm, d, L)]
        label = (f"{args.config}: B={Bsz} L_t/L_v/L_a={'/'.join(map(str, seg))} d={d} H={H} bf16 {L}-layer encoder forward, "
                 f"mask={args.mask}, padding={w['padding']}")

    peaks = None if args.no_calibration else measured_peaks(B, torch)
    r = measure(step, args, B, torch)
    ms_step, per_step, launches, dom = r["ms_step"], r["per_step"], r["launches"], r["dom"]
    pc = [pair_counts(seg, m_, Bsz, g["valid_len"], None) for m_, _, _ in lm_list]
    core = sum(4.0 * p[0] * w_ * n_ for p, (_, w_, n_) in zip(pc, lm_list))          # valid x valid pairs
    core_exec = sum(4.0 * p[1] * w_ * n_ for p, (_, w_, n_) in zip(pc, lm_list))     # rows in memory x valid keys
    other = sum((8.0 * w_ * w_ + 4.0 * w_ * (d_ff * w_ // d)) * Bsz * T * n_ for _, w_, n_ in lm_list)  # projections + MLP
    n_l = launches[dom]
    dh_list = sorted({w_ // (H if w_ == d else H) for _, w_, _ in lm_list})
    # all launches of the forward family together (several layers, and for the model two widths): algorithmic and
    # executed MFMA flops summed over them
    exe = sum(MFMA_PER_BLOCK[0]["attn_fwd"] * 32768.0 * p[1] * H / 1024.0 * n_ for p, (_, w_, n_) in zip(pc, lm_list))
    tf = core_exec / (per_step[dom] * 1e-3) / 1e12
    roof = {"bound": "mfma", "kernel": dom, "achieved": round(tf, 3), "peak": PEAK_MFMA_BF16_TFLOPS, "unit": "TFLOP/s",
            "frac": round(tf / PEAK_MFMA_BF16_TFLOPS, 4), "traffic": None, "traffic_source": None,
            "avg_launch_ms": round(per_step[dom] / n_l, 4), "launches_per_step": round(n_l, 1),
            "executed_mfma_tflops": round(exe / (per_step[dom] * 1e-3) / 1e12, 2),
            "useful_mfma_frac": round(core_exec / exe, 4),
            "note": f"head dims {dh_list} run on the matrix cores in sub-head mode (a head is a slice of a 64-column group): "
                    "`achieved` = algorithmic 4 P d flops of all forward launches of a step / their summed time, "
                    "`executed_mfma_tflops` = what the matrix cores execute for them; the softmax's vector instructions, "
                    "not counted as flops, take a comparable share of the time"}
    if peaks:
        roof["frac_of_measured_peak"] = round(tf / peaks["mfma_bf16_tflops"], 4)
        roof["measured_peak"] = peaks["mfma_bf16_tflops"]
    out = {
        "metric": "IM-attention fwd TFLOP/s on live blocks; % of MFMA roofline",
        "value": round(core / (ms_step * 1e-3) / 1e12, 3), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_step, 4), "ms_per_step_median": round(r["median"], 4),
        "ms_per_step_min": round(r["min"], 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": label, "live_pairs_per_layer": [p[0] for p in pc],
                   "live_pairs_rows_in_memory_per_layer": [p[1] for p in pc],
                   "core_gflop_per_step": round(core / 1e9, 2), "proj_mlp_gflop_per_step": round(other / 1e9, 2)},
        "with_projection_mlp_tflops": round((core + other) / (ms_step * 1e-3) / 1e12, 3),
        "kernel_ms_per_step": {k: round(v, 4) for k, v in per_step.items()},
        "kernel_launches_per_step": {k: round(v, 1) for k, v in launches.items()},
        "kernel_ms_note": "dominant attention family: HIP events over the timed steps; the other families: a separate pass after them with every family bracketed",
        "roofline": roof,
    }
    if peaks:
        out["measured_peaks"] = peaks
    if not args.no_cpu_baseline:
        import oracle
        n_sample = 4
        t0 = time.perf_counter()
        vls = None if g["valid_len"] is None else g["valid_len"][:n_sample]
        if whole_model:
            oracle.gsit_model_forward(g["x"][:n_sample], m, seg, H, g["scale"], H, scale_intra, valid_len=vls)
        else:
            lay = [synth.layer_params(d, d_ff, w["seed"], l, dtype=dtype) for l in range(L)]
            oracle.gsit_encoder_forward(g["x"][:n_sample], lay, seg, mask_of(args.mask, B), H, g["scale"], valid_len=vls)
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": round(core * n_sample / Bsz / dt / 1e12, 6), "unit": "TFLOP/s", "cores": int(host_threads()),
                               "kind": "oracle", "seconds": round(dt, 2),
                               "sample": f"first {n_sample} of {Bsz} batch elements of the same workload, dense fp64 numpy oracle forward"}
    print(json.dumps(out))


def bench_layer_train(args):
    """--config c4train: one encoder layer, training forward + backward, at the C4 shapes (bf16)."""
    import numpy as np
    import torch
    from paper_2505_01068_amd import binding as B, synth

    torch.cuda.set_device(0)
    lm = mask_of(args.mask, B)
    over = {"seg_len": DATASET_SHAPES[args.shape]} if args.shape else {}
    w = synth.workload("c4", **over)
    g = synth.attention_inputs(**w)
    dtype, tdt = g["dtype"], torch.bfloat16
    Bsz, T, d = g["x"].shape
    H, d_ff, seg = g["n_heads"], w["d_ff"], g["seg_len"]
    dev = lambda a: None if a is None else (lambda t: (t.to(tdt) if t.dtype == torch.float32 else t).cuda())(torch.from_numpy(np.ascontiguousarray(a)))
    pn = synth.layer_params(d, d_ff, w["seed"], 0, dtype=dtype)
    p = {k: dev(v) for k, v in pn.items()}
    x, dy = dev(g["x"]), dev(g["dy"])
    shape = B.make_shape(Bsz, seg, d, H, lm, g["scale"], dtype)
    sb, wb = B.gsit_layer_train_sizes(shape, d_ff)
    saved = torch.empty(sb, dtype=torch.uint8, device="cuda")
    ws = torch.empty(wb, dtype=torch.uint8, device="cuda")
    grads = {k: torch.empty(v.shape, dtype=torch.float32, device="cuda") for k, v in p.items()}
    y, dx = torch.empty_like(x), torch.empty_like(x)

    def fwd():
        B.gsit_layer_fwd_train(shape, d_ff, x, p, saved, y=y, workspace=ws)

    def bwd():
        B.gsit_layer_bwd(shape, d_ff, x, p, saved, dy, grads, dx=dx, workspace=ws)

    def step():
        fwd()
        bwd()

    peaks = None if args.no_calibration else measured_peaks(B, torch)
    r = measure(step, args, B, torch, fwd, bwd)
    ms_step, per_step, launches, dom = r["ms_step"], r["per_step"], r["launches"], r["dom"]
    P, P_rows = pair_counts(seg, lm, Bsz, None, None)
    core = 14.0 * P * d
    other = 3.0 * (8.0 * d * d + 4.0 * d * d_ff) * Bsz * T     # projections + MLP, forward and the two backward products
    fr = attention_fracs(per_step, launches, P_rows, d, d // H, True, peaks)
    core_ms = sum(per_step[k] for k in fr)
    out = {
        "metric": "IM-attention fwd+bwd TFLOP/s on live blocks; % of MFMA roofline",
        "value": round(core / (ms_step * 1e-3) / 1e12, 3), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_step, 4), "ms_per_step_median": round(r["median"], 4),
        "ms_per_step_min": round(r["min"], 4), "fwd_ms_median": round(r["fwd_median"], 4),
        "bwd_ms_median": round(r["bwd_median"], 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"c4train: B={Bsz} L_t/L_v/L_a={'/'.join(map(str, seg))} d={d} H={H} d_ff={d_ff} bf16, one "
                               f"encoder layer training forward + backward, mask={args.mask}, padding=none",
                   "live_pairs": P, "core_gflop_per_step": round(core / 1e9, 2), "proj_mlp_gflop_per_step": round(other / 1e9, 2)},
        "with_projection_mlp_tflops": round((core + other) / (ms_step * 1e-3) / 1e12, 3),
        "kernel_ms_per_step": {k: round(v, 4) for k, v in per_step.items()},
        "kernel_ms_note": "dominant attention family: HIP events over the timed steps; the other families: a separate pass after them with every family bracketed",
        "kernel_frac": fr,
        "attn_core_tflops": round(core / (core_ms * 1e-3) / 1e12, 3),
        "attn_core_frac": round(core / (core_ms * 1e-3) / 1e12 / PEAK_MFMA_BF16_TFLOPS, 4),
        "roofline": roofline_of(dom, fr, True, peaks, None, None, launches[dom], True),
    }
    if peaks:
        out["measured_peaks"] = peaks
    if not args.no_cpu_baseline:
        import oracle
        n_sample = 4
        t0 = time.perf_counter()
        oracle.gsit_layer_backward(g["x"][:n_sample], pn, g["dy"][:n_sample], seg, lm, H, g["scale"])
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": round(core * n_sample / Bsz / dt / 1e12, 6), "unit": "TFLOP/s", "cores": int(host_threads()),
                               "kind": "oracle", "seconds": round(dt, 2),
                               "sample": f"first {n_sample} of {Bsz} batch elements, dense fp64 numpy oracle layer forward + backward"}
    print(json.dumps(out))


def run_calibration():
    import torch
    from paper_2505_01068_amd import binding as B
    torch.cuda.set_device(0)
    p = measured_peaks(B, torch, quick=False)
    p.update({"published_mfma_bf16_tflops": PEAK_MFMA_BF16_TFLOPS, "published_hbm_gbs": PEAK_HBM_GBS,
              "mfma_frac_of_published": round(p["mfma_bf16_tflops"] / PEAK_MFMA_BF16_TFLOPS, 4),
              "hbm_frac_of_published": round(p["hbm_copy_gbs"] / PEAK_HBM_GBS, 4)})
    print(json.dumps(p))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", default="c5", choices=["c2", "c3", "c3p", "c3v", "c4", "c4v", "c4train", "c5", "gsit"],
                    help="c3p: the C3 shape with the dataset's sequence-length statistics, packed rows; "
                         "c3v: the same lengths with padded rows and valid_len; c4v: C4 with C3's valid lengths")
    ap.add_argument("--mask", default="ifm_forward",
                    help="a named pattern (ifm_forward, ifm_backward, iem, dense, structure1_a ... structure3_b, self_only) "
                         "or info_disorder (text rows see vision and audio keys under one softmax)")
    ap.add_argument("--shape", default=None, choices=sorted(DATASET_SHAPES),
                    help="small-model configs: the maximum lengths of another dataset instead of 50/500/375")
    ap.add_argument("--graph", action="store_true",
                    help="attention configs: capture one forward+backward into a HIP graph and time its replays "
                         "(the per-kernel table and the roofline still come from eager passes)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-calibration", action="store_true", help="skip the two micro-benchmarks (measured_peaks)")
    ap.add_argument("--calibrate", action="store_true", help="run only the micro-benchmarks and print their JSON line")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run one 1 GiB device copy first (reference reading for rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: the library runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2505_01068_amd import binding as B, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    if args.mask != "info_disorder" and args.mask not in B.NAMED_MASKS:
        print(f"bench.py: unknown mask {args.mask!r}; choose from {sorted(B.NAMED_MASKS) + ['info_disorder']}", file=sys.stderr)
        sys.exit(2)
    if args.calibrate:
        return run_calibration()
    if args.shape and args.config == "c5":
        print("bench.py: --shape applies to the small-model configs (c2, c3*, c4*, gsit)", file=sys.stderr)
        sys.exit(2)
    if args.config in ("c4", "c4v", "gsit"):
        return bench_encoder(args, args.config == "gsit")
    if args.config == "c4train":
        return bench_layer_train(args)
    torch.cuda.set_device(0)
    lm = mask_of(args.mask, B)
    over = {"seg_len": DATASET_SHAPES[args.shape]} if args.shape else {}

    lengths = None
    if args.config in ("c3p", "c3v"):
        # C3 shape; per-sample lengths with the mean and variance of the dataset table (App. "Datasets")
        w = synth.workload("c3", padding="none", **over)
        g = synth.attention_inputs(**w)
        st = synth.MOSI_LENGTH_STATS
        lengths = synth.dataset_lengths(w["batch"], w["seg_len"], st["mean"], st["var"], seed=w["seed"])
        g["valid_len"] = lengths
        w["padding"] = "packed rows" if args.config == "c3p" else "valid_len"
    else:
        w = synth.workload(args.config, **over)
        g = synth.attention_inputs(**w)
    dtype = g["dtype"]
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    Bsz, T, d = g["x"].shape
    H = g["n_heads"]

    def dev(a):
        if a is None:
            return None
        t = torch.from_numpy(np.ascontiguousarray(a))
        return (t.to(tdt) if t.dtype == torch.float32 else t).cuda()

    rows = Bsz * T
    if args.config == "c3p":
        cu = synth.row_offsets(lengths)
        cu_dev = torch.from_numpy(cu).cuda()
        rows = int(cu[-1])
        shape = B.make_shape(Bsz, g["seg_len"], d, H, lm, g["scale"], dtype, cu_rows=cu_dev, total_rows=rows)
        x, dy = dev(synth.pack_rows(g["x"], lengths, g["seg_len"])), dev(synth.pack_rows(g["dy"], lengths, g["seg_len"]))
        vl, kp = None, None
    else:
        shape = B.make_shape(Bsz, g["seg_len"], d, H, lm, g["scale"], dtype)
        x, dy = dev(g["x"]), dev(g["dy"])
        vl, kp = dev(g["valid_len"]), dev(g["key_pad"])
    wq, wk, wv, wo = (dev(g[n]) for n in ("wq", "wk", "wv", "wo"))
    sb, wb = B.im_attention_sizes(shape)
    saved = torch.empty(sb, dtype=torch.uint8, device="cuda")
    ws = torch.empty(wb, dtype=torch.uint8, device="cuda")
    y, dx = torch.empty_like(x), torch.empty_like(x)
    dws = [torch.empty(d, d, dtype=torch.float32, device="cuda") for _ in range(4)]

    def fwd():
        B.im_attention_fwd(shape, x, wq, wk, wv, wo, valid_len=vl, key_pad=kp, y=y, saved=saved, workspace=ws)

    def bwd():
        B.im_attention_bwd(shape, x, wq, wk, wv, wo, saved, dy, dx, *dws, valid_len=vl, key_pad=kp, workspace=ws)

    def step():
        fwd()
        bwd()

    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    peaks = None if args.no_calibration else measured_peaks(B, torch)
    r = measure(step, args, B, torch, fwd, bwd)
    ms_step, per_step, launches, dom = r["ms_step"], r["per_step"], r["launches"], r["dom"]
    ms_eager = None
    if args.graph:
        # the calls allocate nothing and record no memsets: one step is capturable as it is
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step()
        for _ in range(args.warmup):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        ms_eager, ms_step = ms_step, (time.perf_counter() - t0) * 1e3 / args.steps

    # P: valid lengths on both sides (the work that was asked for); P_rows: every query row in memory against
    # its valid keys (what the kernels execute with padded rows; equal to P with packed rows or without padding)
    P, P_rows = pair_counts(g["seg_len"], lm, Bsz, g["valid_len"], g["key_pad"])
    if args.config == "c3p":
        P_rows = P
    core_flops = 14.0 * P * d                         # 4 P d forward + 10 P d backward (summed over heads)
    proj_flops = 24.0 * rows * d * d                  # 8 fwd + 16 bwd, on the rows held in memory
    value = core_flops / (ms_step * 1e-3) / 1e12

    # ---- roofline: per attention kernel, algorithmic flops per launch / its time ----
    # forward 4 P d (two products); dK/dV kernel 8 P d (S, dP, dV, dK); dQ kernel 2 P d (the dQ product; its
    # recomputed S and dP are not algorithmic work).  P_rows is used: padded query rows are executed work.
    dh = d // H
    mfma_path = dtype == "bf16" and dh in (8, 16, 64) and d % 64 == 0
    fr = attention_fracs(per_step, launches, P_rows, d, dh, mfma_path, peaks)
    traffic, traffic_src = stored_traffic(args.config, dom) if args.mask == "ifm_forward" and not args.shape else (None, None)
    roof = roofline_of(dom, fr, mfma_path, peaks, traffic, traffic_src, launches[dom], dh != 64)
    core_ms = sum(per_step[k] for k in fr)
    core_tf = 14.0 * P_rows * d / (core_ms * 1e-3) / 1e12
    peak_core = PEAK_MFMA_BF16_TFLOPS if mfma_path else PEAK_FP32_VALU_UNPACKED_TFLOPS

    out = {
        "metric": "IM-attention fwd+bwd TFLOP/s on live blocks; % of HBM/MFMA roofline",
        "value": round(value, 3), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_step, 4), "ms_per_step_median": round(r["median"], 4), "ms_per_step_min": round(r["min"], 4),
        "fwd_ms_median": round(r["fwd_median"], 4), "fwd_ms_min": round(r["fwd_min"], 4),
        "bwd_ms_median": round(r["bwd_median"], 4), "bwd_ms_min": round(r["bwd_min"], 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"{args.config}: B={Bsz} L_t/L_v/L_a={'/'.join(map(str, g['seg_len']))} d={d} H={H} "
                               f"{dtype} fwd+bwd, mask={args.mask}, padding={w['padding']}",
                   "rows_in_memory": rows, "live_pairs": P, "live_pairs_rows_in_memory": P_rows,
                   "live_pairs_note": "live_pairs: valid query x valid live key (both sides valid); live_pairs_rows_in_memory: "
                                      "every query row in memory x its valid live keys (what the kernels execute)",
                   "core_gflop_per_step": round(core_flops / 1e9, 2), "proj_gflop_per_step": round(proj_flops / 1e9, 2)},
        "with_projection_tflops": round((core_flops + proj_flops) / (ms_step * 1e-3) / 1e12, 3),
        "kernel_ms_per_step": {k: round(v, 4) for k, v in per_step.items()},
        "kernel_ms_note": "dominant attention family: HIP events over the timed steps; the other families: a separate pass after them with every family bracketed",
        "kernel_frac": fr,
        "attn_core_tflops": round(core_tf, 3),
        "attn_core_frac": round(core_tf / peak_core, 4),
        "roofline": roof,
    }
    if peaks:
        out["measured_peaks"] = peaks
        if mfma_path:
            out["attn_core_frac_of_measured_peak"] = round(core_tf / peaks["mfma_bf16_tflops"], 4)
    if ms_eager is not None:
        out["config"]["launch"] = "HIP graph replay"
        out["ms_per_step_eager"] = round(ms_eager, 4)

    if not args.no_cpu_baseline:
        import oracle
        n_sample = Bsz                                        # ~10-30 s of CPU work on the benchmark host
        sl = slice(0, n_sample)
        t0 = time.perf_counter()
        _, cache = oracle.forward(g["x"][sl], g["wq"], g["wk"], g["wv"], g["wo"], g["seg_len"], lm, H, g["scale"],
                                  valid_len=None if g["valid_len"] is None else g["valid_len"][sl],
                                  key_pad=None if g["key_pad"] is None else g["key_pad"][sl], return_cache=True)
        oracle.backward(cache, g["dy"][sl])
        dt = time.perf_counter() - t0
        P1, _ = pair_counts(g["seg_len"], lm, n_sample, None if g["valid_len"] is None else g["valid_len"][sl],
                            None if g["key_pad"] is None else g["key_pad"][sl])
        out["cpu_baseline"] = {"value": round(14.0 * P1 * d / dt / 1e12, 6), "unit": "TFLOP/s", "cores": int(host_threads()),
                               "kind": "oracle", "seconds": round(dt, 2),
                               "sample": f"first {n_sample} of {Bsz} batch elements of the same workload, dense fp64 "
                                         "numpy oracle fwd+bwd (live-block flops counted, dense work done)"}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
