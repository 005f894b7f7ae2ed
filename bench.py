#!/usr/bin/env python3
"""Benchmark of the IM-attention hot path on one MI355X.

One "step" = one im_attention_fwd + one im_attention_bwd through the C ABI
(schedule, shared QKV projection, live-block scores / softmax / aggregation,
output projection and the whole backward) on one batch of synthetic inputs that
is already resident in HBM.  The headline value is live-block attention
TFLOP/s: (4 + 10) * P * d flops per step, P = number of (query, valid live key)
pairs over the batch, divided by the time of the WHOLE step (projections and
weight gradients included in the time, not in the flops).

Prints ONE JSON line.  The `roofline` object is for the dominant attention kernel
of the step, timed with HIP events recorded by the library on the call's stream
over the timed steps (im_profile_enable; the other kernel families are timed
in a separate pass, see timed_run); `cpu_baseline` is the fp64 CPU oracle timed on a bounded
sample (one batch element) of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# MI355X published peaks
PEAK_HBM_GBS = 8000.0
PEAK_MFMA_BF16_TFLOPS = 2500.0
PEAK_FP32_VALU_TFLOPS = 157.3


def live_pairs(seg_len, live_mask, batch, valid_len, key_pad):
    """(query row, valid live key) pairs over the batch -- integer bookkeeping of the workload."""
    import numpy as np
    n = len(seg_len)
    off = np.concatenate([[0], np.cumsum(seg_len)])
    total = 0
    for b in range(batch):
        klen = []
        for j in range(n):
            k = seg_len[j] if valid_len is None else min(seg_len[j], int(valid_len[b, j]))
            if key_pad is not None:
                k = int((key_pad[b, off[j]:off[j] + k] == 0).sum())
            klen.append(k)
        for i in range(n):
            for j in range(n):
                if (live_mask >> (i * n + j)) & 1:
                    total += seg_len[i] * klen[j]
    return total


def timed_run(step, args, B, torch):
    """Warm-up, the timed steps, then a short pass that times every kernel family.

    Event pairs around kernel families cost stream time (about 6 % of a C5 step when every family is
    bracketed), so in the timed region only the dominant attention family is bracketed -- that measurement
    feeds the roofline object.  Which family dominates is found in a 3-step probe after the warm-up; the
    per-family table (`kernel_ms_per_step`) comes from a pass of the same length as the warm-up AFTER the timed
    region, with every family bracketed.
    Returns (ms per step, {family: ms per step}, {family: launches per step}, dominant)."""
    def profiled(n, only=None):
        torch.cuda.synchronize()
        B.im_profile_enable(True, only=only)
        t0 = time.perf_counter()
        for _ in range(n):
            step()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        B.im_profile_enable(False)
        return (t1 - t0) * 1e3 / n, {k: (v[0] / n, v[1] / n) for k, v in B.im_profile_get().items() if v[1] > 0}

    for _ in range(args.warmup):
        step()
    _, probe = profiled(3)
    cands = [k for k in ("attn_fwd", "attn_dq", "attn_dkv") if k in probe]
    dom = max(cands, key=lambda k: probe[k][0])
    ms_step, timed = profiled(args.steps, only=dom)
    _, table = profiled(max(3, args.warmup))
    table.update(timed)
    return ms_step, {k: v[0] for k, v in table.items()}, {k: v[1] for k, v in table.items()}, dom


def stored_traffic(config, family):
    """HBM bytes per launch of the dominant kernel from the committed counter summary
    (profiles/<config>_<family>_traffic.md), or None if there is none or the kernel sources changed since."""
    import re
    from paper_2505_01068_amd.traffic import source_hash
    path = os.path.join(ROOT, "profiles", f"{config}_{family}_traffic.md")
    try:
        m = re.search(r"^TRAFFIC_JSON (.*)$", open(path).read(), flags=re.M)
        rec = json.loads(m.group(1))
        return rec["bytes_per_launch"] if source_hash(rec["kernel"]) == rec["source_sha256"] else None
    except Exception:
        return None


def bench_encoder(args, whole_model):
    """--config c4: the 4-layer encoder forward (layer = pre-LN IM attention + GELU MLP) at the C4 shapes;
    --config gsit: the whole GsiT forward (two IFM encoders, feature concat, IEM encoder at width 2d, last
    steps, final linear) at the same shapes.  Forward only; value = live-block attention TFLOP/s of all layers
    over the whole call."""
    import numpy as np
    import torch
    from paper_2505_01068_amd import binding as B, synth

    torch.cuda.set_device(0)
    masks = {"ifm_forward": B.IM_IFM_FORWARD, "ifm_backward": B.IM_IFM_BACKWARD, "iem": B.IM_IEM}
    w = synth.workload("c4")
    g = synth.attention_inputs(**{**w, "with_dy": False})
    dtype, tdt = g["dtype"], torch.bfloat16
    Bsz, T, d = g["x"].shape
    H, L, d_ff, seg = g["n_heads"], w["n_layers"], w["d_ff"], g["seg_len"]

    def dev(a):
        if a is None:
            return None
        t = torch.from_numpy(np.ascontiguousarray(a))
        return (t.to(tdt) if t.dtype == torch.float32 else t).cuda()

    x = dev(g["x"])
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
            B.gsit_model_fwd(shape, model, x, out=out_t, workspace=ws)
        lm_list = [(B.IM_IFM_FORWARD, d, L), (B.IM_IFM_BACKWARD, d, L), (B.IM_IEM, 2 * d, L)]
        label = (f"gsit: whole model forward, B={Bsz} L_t/L_v/L_a={'/'.join(map(str, seg))} d={d} H={H} bf16, "
                 f"{L}+{L} IFM layers, {L} IEM layers at width {2 * d}")
    else:
        lm = masks[args.mask]
        layers = [{k: dev(v) for k, v in synth.layer_params(d, d_ff, w["seed"], l, dtype=dtype).items()} for l in range(L)]
        shape = B.make_shape(Bsz, seg, d, H, lm, g["scale"], dtype)
        ws = torch.empty(B.gsit_layer_sizes(shape, d_ff), dtype=torch.uint8, device="cuda")
        bufs = [torch.empty_like(x), torch.empty_like(x)]

        def step():
            h = x
            for l, p in enumerate(layers):
                h = B.gsit_layer_fwd(shape, d_ff, h, p, y=bufs[l & 1], workspace=ws)
        lm_list = [(lm, d, L)]
        label = (f"c4: B={Bsz} L_t/L_v/L_a={'/'.join(map(str, seg))} d={d} H={H} bf16 {L}-layer encoder forward, "
                 f"mask={args.mask}, padding=none")

    ms_step, per_step, launches, dom = timed_run(step, args, B, torch)
    core = sum(4.0 * live_pairs(seg, m_, Bsz, None, None) * w_ * n_ for m_, w_, n_ in lm_list)
    other = sum((8.0 * w_ * w_ + 4.0 * w_ * (d_ff * w_ // d)) * Bsz * T * n_ for m_, w_, n_ in lm_list)  # projections + MLP
    dom_ms = per_step[dom] / launches[dom]
    achieved = core / launches[dom] / (dom_ms * 1e-3) / 1e12
    out = {
        "metric": "IM-attention fwd TFLOP/s on live blocks; % of ALU roofline",
        "value": round(core / (ms_step * 1e-3) / 1e12, 3), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": label, "core_gflop_per_step": round(core / 1e9, 2),
                   "proj_mlp_gflop_per_step": round(other / 1e9, 2)},
        "with_projection_mlp_tflops": round((core + other) / (ms_step * 1e-3) / 1e12, 3),
        "kernel_ms_per_step": {k: round(v, 4) for k, v in per_step.items()},
        "kernel_ms_note": "dominant attention family: HIP events over the timed steps; the other families: a separate pass after them with every family bracketed",
        "roofline": {"bound": "alu", "kernel": dom, "achieved": round(achieved, 3), "peak": PEAK_FP32_VALU_TFLOPS,
                     "unit": "TFLOP/s", "frac": round(achieved / PEAK_FP32_VALU_TFLOPS, 4), "traffic": None,
                     "avg_launch_ms": round(dom_ms, 4),
                     "note": "head dims 8 / 16: the two contractions run on the matrix cores in sub-head mode (1/8 to 1/2 "
                             "of each MFMA is useful work); the softmax's plain-ALU instructions bound the kernel, so the "
                             "algorithmic flops are set against the fp32 vector peak"},
    }
    if not args.no_cpu_baseline:
        import oracle
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            cores = os.cpu_count() or 1
        n_sample = 4
        t0 = time.perf_counter()
        if whole_model:
            oracle.gsit_model_forward(g["x"][:n_sample], m, seg, H, g["scale"], H, scale_intra)
        else:
            lay = [synth.layer_params(d, d_ff, w["seed"], l, dtype=dtype) for l in range(L)]
            oracle.gsit_encoder_forward(g["x"][:n_sample], lay, seg, masks[args.mask], H, g["scale"])
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": round(core * n_sample / Bsz / dt / 1e12, 6), "unit": "TFLOP/s", "cores": int(cores),
                               "kind": "oracle", "seconds": round(dt, 2),
                               "sample": f"first {n_sample} of {Bsz} batch elements of the same workload, dense fp64 numpy oracle forward"}
    print(json.dumps(out))


def bench_layer_train(args):
    """--config c4train: one encoder layer, training forward + backward, at the C4 shapes (bf16)."""
    import numpy as np
    import torch
    from paper_2505_01068_amd import binding as B, synth

    torch.cuda.set_device(0)
    masks = {"ifm_forward": B.IM_IFM_FORWARD, "ifm_backward": B.IM_IFM_BACKWARD, "iem": B.IM_IEM}
    lm = masks[args.mask]
    w = synth.workload("c4")
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

    def step():
        B.gsit_layer_fwd_train(shape, d_ff, x, p, saved, y=y, workspace=ws)
        B.gsit_layer_bwd(shape, d_ff, x, p, saved, dy, grads, dx=dx, workspace=ws)

    ms_step, per_step, launches, dom = timed_run(step, args, B, torch)
    P = live_pairs(seg, lm, Bsz, None, None)
    core = 14.0 * P * d
    other = 3.0 * (8.0 * d * d + 4.0 * d * d_ff) * Bsz * T     # projections + MLP, forward and the two backward products
    alg = {"attn_fwd": 4.0 * P * d, "attn_dkv": 8.0 * P * d, "attn_dq": 2.0 * P * d}
    achieved = alg[dom] / (per_step[dom] * 1e-3) / 1e12
    out = {
        "metric": "IM-attention fwd+bwd TFLOP/s on live blocks; % of ALU roofline",
        "value": round(core / (ms_step * 1e-3) / 1e12, 3), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"c4train: B={Bsz} L_t/L_v/L_a={'/'.join(map(str, seg))} d={d} H={H} d_ff={d_ff} bf16, one "
                               f"encoder layer training forward + backward, mask={args.mask}, padding=none",
                   "core_gflop_per_step": round(core / 1e9, 2), "proj_mlp_gflop_per_step": round(other / 1e9, 2)},
        "with_projection_mlp_tflops": round((core + other) / (ms_step * 1e-3) / 1e12, 3),
        "kernel_ms_per_step": {k: round(v, 4) for k, v in per_step.items()},
        "kernel_ms_note": "dominant attention family: HIP events over the timed steps; the other families: a separate pass after them with every family bracketed",
        "roofline": {"bound": "alu", "kernel": dom, "achieved": round(achieved, 3), "peak": PEAK_FP32_VALU_TFLOPS,
                     "unit": "TFLOP/s", "frac": round(achieved / PEAK_FP32_VALU_TFLOPS, 4), "traffic": None,
                     "avg_launch_ms": round(per_step[dom], 4),
                     "note": "head dim 8: the contractions run on the matrix cores in sub-head mode (1/8 to 1/2 of each MFMA "
                             "is useful work); the softmax's plain-ALU instructions bound the kernel, so the algorithmic "
                             "flops are set against the fp32 vector peak"},
    }
    if not args.no_cpu_baseline:
        import oracle
        try:
            from threadpoolctl import threadpool_info
            cores = max([q.get("num_threads", 1) for q in threadpool_info()] + [1])
        except Exception:
            cores = os.cpu_count() or 1
        n_sample = 4
        t0 = time.perf_counter()
        oracle.gsit_layer_backward(g["x"][:n_sample], pn, g["dy"][:n_sample], seg, lm, H, g["scale"])
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": round(core * n_sample / Bsz / dt / 1e12, 6), "unit": "TFLOP/s", "cores": int(cores),
                               "kind": "oracle", "seconds": round(dt, 2),
                               "sample": f"first {n_sample} of {Bsz} batch elements, dense fp64 numpy oracle layer forward + backward"}
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default="c5", choices=["c2", "c3", "c3p", "c3v", "c4", "c4train", "c5", "gsit"],
                    help="c3p: the C3 shape with the dataset's sequence-length statistics, packed rows; "
                         "c3v: the same lengths with padded rows and valid_len")
    ap.add_argument("--mask", default="ifm_forward", choices=["ifm_forward", "ifm_backward", "iem"])
    ap.add_argument("--graph", action="store_true",
                    help="attention configs: capture one forward+backward into a HIP graph and time its replays "
                         "(the per-kernel table and the roofline still come from eager passes)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run one 1 GiB device copy first (reference reading for rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2505_01068_amd import binding as B, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    if args.config in ("c4", "gsit"):
        return bench_encoder(args, args.config == "gsit")
    if args.config == "c4train":
        return bench_layer_train(args)
    torch.cuda.set_device(0)
    masks = {"ifm_forward": B.IM_IFM_FORWARD, "ifm_backward": B.IM_IFM_BACKWARD, "iem": B.IM_IEM}
    lm = masks[args.mask]

    lengths = None
    if args.config in ("c3p", "c3v"):
        # C3 shape; per-sample lengths with the mean and variance of the dataset table (App. "Datasets")
        w = synth.workload("c3", padding="none")
        g = synth.attention_inputs(**w)
        st = synth.MOSI_LENGTH_STATS
        lengths = synth.dataset_lengths(w["batch"], st["max"], st["mean"], st["var"], seed=w["seed"])
        g["valid_len"] = lengths
        w["padding"] = "packed rows" if args.config == "c3p" else "valid_len"
    else:
        w = synth.workload(args.config)
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

    def step():
        B.im_attention_fwd(shape, x, wq, wk, wv, wo, valid_len=vl, key_pad=kp, y=y, saved=saved, workspace=ws)
        B.im_attention_bwd(shape, x, wq, wk, wv, wo, saved, dy, dx, *dws, valid_len=vl, key_pad=kp, workspace=ws)

    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    ms_step, per_step, launches, dom = timed_run(step, args, B, torch)
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

    P = live_pairs(g["seg_len"], lm, Bsz, g["valid_len"], g["key_pad"])
    if lengths is not None:
        # only the rows inside the lengths are work that was asked for, as queries too
        n = len(g["seg_len"])
        P = int(sum(int(lengths[b, i]) * int(lengths[b, j]) for b in range(Bsz) for i in range(n) for j in range(n)
                    if (lm >> (i * n + j)) & 1))
    core_flops = 14.0 * P * d                         # 4 P d forward + 10 P d backward (summed over heads)
    proj_flops = 24.0 * rows * d * d                  # 8 fwd + 16 bwd, on the rows held in memory
    value = core_flops / (ms_step * 1e-3) / 1e12

    # ---- roofline of the dominant kernel (by accumulated event time) ----
    # algorithmic flops per launch: forward 4 P d (two products); dK/dV kernel 8 P d (S, dP, dV, dK);
    # dQ kernel 2 P d (the dQ product; its recomputed S and dP are not algorithmic work)
    alg = {"attn_fwd": 4.0 * P * d, "attn_dkv": 8.0 * P * d, "attn_dq": 2.0 * P * d,
           "proj_fwd": 8.0 * rows * d * d, "proj_bwd": 8.0 * rows * d * d, "wgrad": 8.0 * rows * d * d}
    attn_keys = [k for k in ("attn_fwd", "attn_dq", "attn_dkv") if k in per_step]
    dom_ms = per_step[dom]
    traffic = stored_traffic(args.config, dom) if args.mask == "ifm_forward" else None   # counters were taken with the default mask
    mfma_bound = dtype == "bf16" and d // H == 64
    if mfma_bound:
        achieved = alg[dom] / (dom_ms * 1e-3) / 1e12
        roof = {"bound": "mfma", "kernel": dom, "achieved": round(achieved, 2), "peak": PEAK_MFMA_BF16_TFLOPS,
                "unit": "TFLOP/s", "frac": round(achieved / PEAK_MFMA_BF16_TFLOPS, 4), "traffic": traffic,
                "avg_launch_ms": round(dom_ms, 4)}
    else:
        # small head dims: plain fp32 ALU work (FMAs of the two/five products; exp and softmax bookkeeping not counted)
        achieved = alg[dom] / (dom_ms * 1e-3) / 1e12
        roof = {"bound": "alu", "kernel": dom, "achieved": round(achieved, 3), "peak": PEAK_FP32_VALU_TFLOPS,
                "unit": "TFLOP/s", "frac": round(achieved / PEAK_FP32_VALU_TFLOPS, 4), "traffic": traffic,
                "avg_launch_ms": round(dom_ms, 4)}

    out = {
        "metric": "IM-attention fwd+bwd TFLOP/s on live blocks; % of HBM/MFMA roofline",
        "value": round(value, 3), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"{args.config}: B={Bsz} L_t/L_v/L_a={'/'.join(map(str, g['seg_len']))} d={d} H={H} "
                               f"{dtype} fwd+bwd, mask={args.mask}, padding={w['padding']}",
                   "rows_in_memory": rows, "live_pairs": P, "core_gflop_per_step": round(core_flops / 1e9, 2),
                   "proj_gflop_per_step": round(proj_flops / 1e9, 2)},
        "with_projection_tflops": round((core_flops + proj_flops) / (ms_step * 1e-3) / 1e12, 3),
        "kernel_ms_per_step": {k: round(v, 4) for k, v in per_step.items()},
        "kernel_ms_note": "dominant attention family: HIP events over the timed steps; the other families: a separate pass after them with every family bracketed",
        "attn_core_tflops": round(core_flops / (sum(per_step[k] for k in attn_keys) * 1e-3) / 1e12, 3),
        "roofline": roof,
    }
    if ms_eager is not None:
        out["config"]["launch"] = "HIP graph replay"
        out["ms_per_step_eager"] = round(ms_eager, 4)

    if not args.no_cpu_baseline:
        import oracle
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            cores = os.cpu_count() or 1
        n_sample = Bsz                                        # ~10-30 s of CPU work on the benchmark host
        sl = slice(0, n_sample)
        t0 = time.perf_counter()
        _, cache = oracle.forward(g["x"][sl], g["wq"], g["wk"], g["wv"], g["wo"], g["seg_len"], lm, H, g["scale"],
                                  valid_len=None if g["valid_len"] is None else g["valid_len"][sl],
                                  key_pad=None if g["key_pad"] is None else g["key_pad"][sl], return_cache=True)
        oracle.backward(cache, g["dy"][sl])
        dt = time.perf_counter() - t0
        P1 = live_pairs(g["seg_len"], lm, n_sample, None if g["valid_len"] is None else g["valid_len"][sl],
                        None if g["key_pad"] is None else g["key_pad"][sl])
        out["cpu_baseline"] = {"value": round(14.0 * P1 * d / dt / 1e12, 6), "unit": "TFLOP/s", "cores": int(cores),
                               "kind": "oracle", "seconds": round(dt, 2),
                               "sample": f"first {n_sample} of {Bsz} batch elements of the same workload, dense fp64 "
                                         "numpy oracle fwd+bwd (live-block flops counted, dense work done)"}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
