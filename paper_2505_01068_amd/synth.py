"""Seeded synthetic inputs for IM attention: shapes and padding structure of the
multimodal-sentiment workloads (three modality sequences of unequal length,
strongly varying valid lengths; dataset table of the paper's App. "Datasets").

This module only draws numbers.  It holds none of the method's arithmetic and is
the single piece of code that both the CPU oracle's tests and the GPU path's
tests / benchmark take their inputs from (as arrays).

Generator: a counter-based SplitMix64 hash of (seed, stream, index) -> uniform
(0, 1) -> Box-Muller for N(0, 1).  Values are float32; `to_bf16_grid` rounds to
the nearest bfloat16 (ties to even) while keeping float32 storage, so that the
oracle (which widens to fp64) and the GPU (which narrows to bf16 exactly) see
identical numbers.
"""
from __future__ import annotations

import numpy as np

_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)
_GOLD = np.uint64(0x9E3779B97F4A7C15)
_C1 = np.uint64(0xBF58476D1CE4E5B9)
_C2 = np.uint64(0x94D049BB133111EB)


def _mix(z):
    z = np.asarray(z, dtype=np.uint64)
    with np.errstate(over="ignore"):
        z = (z ^ (z >> np.uint64(30))) * _C1
        z = (z ^ (z >> np.uint64(27))) * _C2
        z = z ^ (z >> np.uint64(31))
    return z


def _bits(seed, stream, n):
    with np.errstate(over="ignore"):
        key = _mix(np.uint64(seed) + _GOLD * _mix(np.uint64(stream) + _GOLD))
        idx = np.arange(n, dtype=np.uint64)
        return _mix(key + (idx + np.uint64(1)) * _GOLD)


def uniform01(seed, stream, shape):
    n = int(np.prod(shape))
    u = ((_bits(seed, stream, n) >> np.uint64(11)).astype(np.float64) + 0.5) / float(1 << 53)
    return u.reshape(shape)


def normal(seed, stream, shape):
    n = int(np.prod(shape))
    u = uniform01(seed, stream, (2 * n,))
    z = np.sqrt(-2.0 * np.log(u[0::2])) * np.cos(2.0 * np.pi * u[1::2])
    return z.astype(np.float32).reshape(shape)


def xavier_uniform(seed, stream, d_in, d_out):
    bound = np.sqrt(6.0 / (d_in + d_out))
    return ((2.0 * uniform01(seed, stream, (d_in, d_out)) - 1.0) * bound).astype(np.float32)


def randint(seed, stream, lo, hi, shape):
    """Integers uniform in [lo, hi] (inclusive); lo/hi may be arrays broadcastable to shape."""
    u = uniform01(seed, stream, shape)
    lo = np.asarray(lo)
    hi = np.asarray(hi)
    return np.minimum(lo + np.floor(u * (hi - lo + 1)).astype(np.int64), hi).astype(np.int32)


def to_bf16_grid(a):
    """Round float32 to the nearest bfloat16 (ties to even), returned as float32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    with np.errstate(over="ignore"):
        v = (u + r) & np.uint32(0xFFFF0000)
    return v.view(np.float32).reshape(a.shape)


# Named workloads.  seg_len is in concatenation order (text, vision, audio).
# "c2".."c5" are the four benchmark shapes; "c1" is the tiny case.
WORKLOADS = {
    "c1": dict(batch=2, seg_len=(8, 8, 8), d_model=32, n_heads=4, dtype="fp32", padding="none"),
    "c2": dict(batch=64, seg_len=(50, 50, 50), d_model=40, n_heads=8, dtype="fp32", padding="key_pad"),
    "c3": dict(batch=32, seg_len=(50, 500, 375), d_model=40, n_heads=8, dtype="fp32", padding="valid_len"),
    "c4": dict(batch=32, seg_len=(50, 500, 375), d_model=64, n_heads=8, dtype="bf16", padding="none",
               n_layers=4, d_ff=256),
    "c5": dict(batch=8, seg_len=(512, 2048, 2048), d_model=512, n_heads=8, dtype="bf16", padding="none"),
}
BASE_SEED = 20250501


def attention_inputs(batch, seg_len, d_model, n_heads, dtype="fp32", padding="none",
                     seed=BASE_SEED, bias=False, with_dy=True, **_unused):
    """One IM-attention problem as a dict of numpy arrays.

    x ~ N(0,1); W_q, W_k, W_v, W_o Xavier-uniform [d, d]; dy ~ N(0,1).
    padding = "key_pad":   per sample and modality, a seeded random 10 % of the
                           positions get x = 0 and key_pad = 1;
              "valid_len": per sample and modality a valid length uniform in
                           [ceil(T/2), T]; x = 0 beyond it;
              "none".
    For dtype "bf16" every float array lies on the bfloat16 grid.
    """
    T = int(sum(seg_len))
    d = d_model
    g = {}
    g["x"] = normal(seed, 1, (batch, T, d))
    for n, s in (("wq", 2), ("wk", 3), ("wv", 4), ("wo", 5)):
        g[n] = xavier_uniform(seed, s, d, d)
    if bias:
        for n, s in (("bq", 6), ("bk", 7), ("bv", 8), ("bo", 9)):
            g[n] = (0.1 * normal(seed, s, (d,))).astype(np.float32)
    if with_dy:
        g["dy"] = normal(seed, 10, (batch, T, d))
    g["valid_len"] = None
    g["key_pad"] = None
    off = np.concatenate([[0], np.cumsum(seg_len)]).astype(int)
    if padding == "key_pad":
        kp = np.zeros((batch, T), dtype=np.uint8)
        u = uniform01(seed, 11, (batch, T))
        for s, n in enumerate(seg_len):
            n_pad = int(round(0.1 * n))
            if n_pad:
                order = np.argsort(u[:, off[s]:off[s + 1]], axis=1, kind="stable")
                rows = np.arange(batch)[:, None]
                kp[rows, off[s] + order[:, :n_pad]] = 1
        g["key_pad"] = kp
        g["x"] = g["x"] * (kp == 0)[:, :, None].astype(np.float32)
    elif padding == "valid_len":
        lo = np.array([(n + 1) // 2 for n in seg_len])
        hi = np.array(seg_len)
        vl = randint(seed, 12, lo[None, :], hi[None, :], (batch, len(seg_len)))
        g["valid_len"] = vl
        pos = np.concatenate([np.arange(n) for n in seg_len])
        seg = np.concatenate([np.full(n, s) for s, n in enumerate(seg_len)])
        keep = pos[None, :] < vl[:, seg]
        g["x"] = g["x"] * keep[:, :, None].astype(np.float32)
    elif padding != "none":
        raise ValueError(padding)
    if dtype == "bf16":
        for n in list(g):
            if isinstance(g[n], np.ndarray) and g[n].dtype == np.float32:
                g[n] = to_bf16_grid(g[n])
    g["seg_len"] = tuple(int(n) for n in seg_len)
    g["n_heads"] = int(n_heads)
    g["scale"] = float(1.0 / np.sqrt(d // n_heads))
    g["dtype"] = dtype
    return g


# Sequence-length statistics of the CMU-MOSI training split (dataset table of App. "Datasets": maximum,
# average length, length variance), in concatenation order (text, vision, audio).  The table lists
# 50/375/500, 14/42/38 and 66/927/805; its order is matched to the benchmark configuration's
# L_t/L_v/L_a = 50/500/375 through the maxima.
MOSI_LENGTH_STATS = dict(max=(50, 500, 375), mean=(14.0, 38.0, 42.0), var=(66.0, 805.0, 927.0))


def dataset_lengths(batch, seg_max, mean, var, seed=BASE_SEED, stream=13):
    """Per-sample, per-modality sequence lengths int32 [batch, n_seg]: a log-normal with the given mean and
    variance (the table gives no more than these two moments), rounded, clipped to 1..seg_max."""
    mean = np.asarray(mean, dtype=np.float64)
    var = np.asarray(var, dtype=np.float64)
    s2 = np.log1p(var / (mean * mean))
    mu = np.log(mean) - 0.5 * s2
    z = normal(seed, stream, (batch, len(seg_max))).astype(np.float64)
    n = np.rint(np.exp(mu[None, :] + np.sqrt(s2)[None, :] * z))
    return np.clip(n, 1, np.asarray(seg_max)[None, :]).astype(np.int32)


def row_offsets(lengths):
    """Packed-row offsets int32 [batch * n_seg + 1] of per-sample segment lengths [batch, n_seg]
    (sample-major, segments in concatenation order)."""
    return np.concatenate([[0], np.cumsum(np.asarray(lengths, dtype=np.int64).reshape(-1))]).astype(np.int32)


def pack_rows(a, lengths, seg_len):
    """[batch, T_m, ...] -> [total_rows, ...]: the first lengths[b, s] rows of every segment, in row_offsets order."""
    off = np.concatenate([[0], np.cumsum(seg_len)]).astype(int)
    parts = [a[b, off[s]:off[s] + int(lengths[b, s])] for b in range(a.shape[0]) for s in range(len(seg_len))]
    return np.ascontiguousarray(np.concatenate(parts, axis=0))


def unpack_rows(p, lengths, seg_len, fill=0.0):
    """Inverse of pack_rows; rows beyond the lengths are `fill`."""
    lengths = np.asarray(lengths)
    off = np.concatenate([[0], np.cumsum(seg_len)]).astype(int)
    out = np.full((lengths.shape[0], int(off[-1])) + p.shape[1:], fill, dtype=p.dtype)
    cu = row_offsets(lengths)
    for b in range(lengths.shape[0]):
        for s in range(len(seg_len)):
            i = b * len(seg_len) + s
            out[b, off[s]:off[s] + int(lengths[b, s])] = p[cu[i]:cu[i + 1]]
    return out


def layer_params(d_model, d_ff, seed, layer, dtype="bf16", bias=True):
    """Weights of one encoder layer: Xavier matrices, LN gain 1 + 0.1 N, LN bias 0.1 N."""
    d = d_model
    s0 = 100 * (layer + 1)
    p = {}
    for n, s in (("wq", 1), ("wk", 2), ("wv", 3), ("wo", 4)):
        p[n] = xavier_uniform(seed, s0 + s, d, d)
    p["w1"] = xavier_uniform(seed, s0 + 5, d, d_ff)
    p["w2"] = xavier_uniform(seed, s0 + 6, d_ff, d)
    p["ln1_g"] = (1.0 + 0.1 * normal(seed, s0 + 7, (d,))).astype(np.float32)
    p["ln1_b"] = (0.1 * normal(seed, s0 + 8, (d,))).astype(np.float32)
    p["ln2_g"] = (1.0 + 0.1 * normal(seed, s0 + 9, (d,))).astype(np.float32)
    p["ln2_b"] = (0.1 * normal(seed, s0 + 10, (d,))).astype(np.float32)
    names = (("bq", 11, d), ("bk", 12, d), ("bv", 13, d), ("bo", 14, d), ("b1", 15, d_ff), ("b2", 16, d))
    for n, s, m in names:
        p[n] = (0.1 * normal(seed, s0 + s, (m,))).astype(np.float32) if bias else None
    if dtype == "bf16":
        for n in list(p):
            if p[n] is not None:
                p[n] = to_bf16_grid(p[n])
    return p


def model_params(d_model, d_ff, d_ff_intra, n_layers, n_layers_intra, n_seg, n_out, seed, dtype="bf16", bias=True):
    """Weights of the whole model: two stacks of `n_layers` layers at width d (the two IFM encoders),
    one stack of `n_layers_intra` layers at width 2d (the IEM encoder), final linear [n_seg*2d, n_out]."""
    m = {
        "fwd_layers": [layer_params(d_model, d_ff, seed, l, dtype, bias) for l in range(n_layers)],
        "bwd_layers": [layer_params(d_model, d_ff, seed, 20 + l, dtype, bias) for l in range(n_layers)],
        "intra_layers": [layer_params(2 * d_model, d_ff_intra, seed, 40 + l, dtype, bias) for l in range(n_layers_intra)],
        "wf": xavier_uniform(seed, 9001, n_seg * 2 * d_model, n_out),
        "bf": (0.1 * normal(seed, 9002, (n_out,))).astype(np.float32) if bias else None,
    }
    if dtype == "bf16":
        m["wf"] = to_bf16_grid(m["wf"])
        if m["bf"] is not None:
            m["bf"] = to_bf16_grid(m["bf"])
    return m


def workload(name, **overrides):
    cfg = dict(WORKLOADS[name])
    cfg.update(overrides)
    k = int(name[1:]) if name[1:].isdigit() else 0
    cfg.setdefault("seed", BASE_SEED + k)
    return cfg
