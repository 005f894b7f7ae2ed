"""Pins for the forward attention oracle (CPU only).

Each test checks the oracle against something fixed by the paper or by plain
mathematics, never against the oracle itself:
  * scalar-loop brute force (no matrices, no numpy in the inner loops);
  * the 3x3 patterns the paper prints (tests/golden/im_patterns.txt);
  * the paper's equivalence claim (Sec. 4: the masked shared-weight pass equals
    the separately computed cross-modal / self attentions; Lemma 1);
  * Sec. "Information Disorder" under "Further Analysis": several live blocks in a row are
    normalised jointly;
  * row-stochastic / zero-block invariants (App. A softmax equation);
  * special cases that are textbook multi-head attention (library routine);
  * the live-pair count of App. B ("w/ Decomposition").
"""
import math

import numpy as np
import pytest
import torch

import oracle
from paper_2505_01068_amd import synth


def tiny(seed=7, B=2, seg=(3, 4, 2), d=8, H=2, bias=True, padding="none"):
    g = synth.attention_inputs(B, seg, d, H, "fp32", padding, seed=seed, bias=bias)
    return g


def brute_force(g, live_mask):
    """Attention written as scalar loops straight from the definition."""
    x = g["x"].astype(float).tolist()
    W = {n: g[n].astype(float).tolist() for n in ("wq", "wk", "wv", "wo")}
    bias = {n: (g[n].astype(float).tolist() if g.get(n) is not None else None) for n in ("bq", "bk", "bv", "bo")}
    seg_len, H, scale = g["seg_len"], g["n_heads"], g["scale"]
    B, T, d = len(x), len(x[0]), len(x[0][0])
    dh = d // H
    n_seg = len(seg_len)
    seg_of, pos_of = [], []
    for s, n in enumerate(seg_len):
        seg_of += [s] * n
        pos_of += list(range(n))
    y = [[[0.0] * d for _ in range(T)] for _ in range(B)]
    for b in range(B):
        def lin(r, w, bb):
            return [sum(x[b][r][i] * w[i][o] for i in range(d)) + (bb[o] if bb else 0.0) for o in range(d)]
        q = [lin(r, W["wq"], bias["bq"]) for r in range(T)]
        k = [lin(r, W["wk"], bias["bk"]) for r in range(T)]
        v = [lin(r, W["wv"], bias["bv"]) for r in range(T)]
        for r in range(T):
            o_row = [0.0] * d
            for h in range(H):
                keys, scores = [], []
                for c in range(T):
                    if not (live_mask >> (seg_of[r] * n_seg + seg_of[c])) & 1:
                        continue
                    if g["valid_len"] is not None and pos_of[c] >= g["valid_len"][b][seg_of[c]]:
                        continue
                    if g["key_pad"] is not None and g["key_pad"][b][c]:
                        continue
                    keys.append(c)
                    scores.append(scale * sum(q[r][h * dh + e] * k[c][h * dh + e] for e in range(dh)))
                if not keys:
                    continue
                m = max(scores)
                w = [math.exp(s - m) for s in scores]
                z = sum(w)
                for c, wc in zip(keys, w):
                    for e in range(dh):
                        o_row[h * dh + e] += wc / z * v[c][h * dh + e]
            for o in range(d):
                y[b][r][o] = sum(o_row[i] * W["wo"][i][o] for i in range(d)) + (bias["bo"][o] if bias["bo"] else 0.0)
    return np.array(y)


def run(g, live_mask, **kw):
    return oracle.forward(g["x"], g["wq"], g["wk"], g["wv"], g["wo"], g["seg_len"], live_mask,
                          g["n_heads"], g["scale"], bq=g.get("bq"), bk=g.get("bk"), bv=g.get("bv"),
                          bo=g.get("bo"), valid_len=g["valid_len"], key_pad=g["key_pad"], **kw)


@pytest.mark.parametrize("name", sorted(oracle.NAMED_PATTERNS))
@pytest.mark.parametrize("padding", ["none", "valid_len", "key_pad"])
def test_brute_force(name, padding):
    g = tiny(padding=padding, seg=(3, 10, 5))
    lm = oracle.NAMED_PATTERNS[name]
    np.testing.assert_allclose(run(g, lm), brute_force(g, lm), rtol=1e-12, atol=1e-13)


def test_brute_force_no_bias_asymmetric_heads():
    g = tiny(seed=3, B=1, seg=(2, 5, 3), d=12, H=3, bias=False)
    for lm in (oracle.IM_IFM_FORWARD, oracle.IM_IFM_BACKWARD):
        np.testing.assert_allclose(run(g, lm), brute_force(g, lm), rtol=1e-12, atol=1e-13)


def _parse_golden(golden_dir):
    pats, edges = {}, {}
    for line in open(f"{golden_dir}/im_patterns.txt"):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        if line.startswith("@edges"):
            name, e = line[len("@edges"):].split("|")
            edges[name.strip()] = e.split()
        else:
            name, _cite, rows = [f.strip() for f in line.split("|")]
            pats[name] = rows.split()
    return pats, edges


def test_patterns_match_paper(golden_dir):
    pats, edges = _parse_golden(golden_dir)
    assert set(pats) == set(oracle.NAMED_PATTERNS) - {"dense"}
    seg_len = (2, 3, 4)
    off = [0, 2, 5, 9]
    for name, rows in pats.items():
        lm = oracle.NAMED_PATTERNS[name]
        m = oracle.additive_mask(seg_len, lm)
        for i in range(3):
            for j in range(3):
                blk = m[off[i]:off[i + 1], off[j]:off[j + 1]]
                if rows[i][j] == "O":
                    assert np.all(blk == 0.0), (name, i, j)
                else:
                    assert np.all(np.isneginf(blk)), (name, i, j)
    for name, e in edges.items():
        assert oracle.live_mask_from_edges(e) == oracle.NAMED_PATTERNS[name], name
    assert oracle.IM_IFM_FORWARD == 0x062 and oracle.IM_IFM_BACKWARD == 0x08C and oracle.IM_IEM == 0x111


def test_ifm_pair_covers_all_cross_blocks_once():
    # Sec. 4: the two IFM graphs are opposing cycles that together realise all six
    # cross-modal pairings, each exactly once, and no intra-modal one.
    f, b = oracle.IM_IFM_FORWARD, oracle.IM_IFM_BACKWARD
    assert f & b == 0 and (f | b) == oracle.IM_DENSE ^ oracle.IM_IEM
    for a_, b_ in (("structure1_a", "structure1_b"), ("structure2_a", "structure2_b"),
                   ("structure3_a", "structure3_b")):
        x, y = oracle.NAMED_PATTERNS[a_], oracle.NAMED_PATTERNS[b_]
        assert x & y == 0 and (x | y) == oracle.IM_DENSE ^ oracle.IM_IEM


SINGLE_BLOCK_ROWS = [n for n, lm in oracle.NAMED_PATTERNS.items()
                     if all(bin((lm >> (3 * i)) & 7).count("1") == 1 for i in range(3))]


@pytest.mark.parametrize("name", SINGLE_BLOCK_ROWS)
@pytest.mark.parametrize("padding", ["none", "valid_len", "key_pad"])
def test_equivalence_with_mult_form(name, padding):
    """Sec. 4 / Lemma 1: masked shared-weight attention == separate CMA / MHSA with the same weights."""
    assert len(SINGLE_BLOCK_ROWS) >= 9
    g = synth.attention_inputs(3, (5, 17, 11), 16, 4, "fp32", padding, seed=11, bias=True)
    lm = oracle.NAMED_PATTERNS[name]
    y_dense = run(g, lm)
    y_mult = oracle.mult_blocks_forward(g["x"], g["wq"], g["wk"], g["wv"], g["wo"], g["seg_len"], lm,
                                        g["n_heads"], g["scale"], bq=g["bq"], bk=g["bk"], bv=g["bv"],
                                        bo=g["bo"], valid_len=g["valid_len"], key_pad=g["key_pad"])
    np.testing.assert_allclose(y_dense, y_mult, rtol=1e-11, atol=1e-12)


def _torch_mha(xq, xkv, g, kv_invalid=None):
    """Library multi-head attention in fp64 (torch.nn.functional), an independent third opinion."""
    d = xq.shape[-1]
    t = lambda a: torch.tensor(np.asarray(a), dtype=torch.float64)
    w_in = torch.cat([t(g["wq"]).T, t(g["wk"]).T, t(g["wv"]).T], 0)
    zeros = torch.zeros(d, dtype=torch.float64)
    b_in = torch.cat([t(g[n]) if g.get(n) is not None else zeros for n in ("bq", "bk", "bv")])
    out, _ = torch.nn.functional.multi_head_attention_forward(
        t(xq)[:, None, :], t(xkv)[:, None, :], t(xkv)[:, None, :], d, g["n_heads"], w_in, b_in,
        None, None, False, 0.0, t(g["wo"]).T, t(g["bo"]) if g.get("bo") is not None else zeros,
        training=False, need_weights=False,
        key_padding_mask=None if kv_invalid is None else torch.tensor(kv_invalid)[None, :])
    return out[:, 0, :].numpy()


def test_dense_pattern_is_textbook_mha():
    g = tiny(seed=5, B=2, seg=(4, 6, 5), d=16, H=4, bias=True, padding="key_pad")
    y = run(g, oracle.IM_DENSE)
    inv = oracle.key_invalid(g["seg_len"], 2, g["valid_len"], g["key_pad"])
    for b in range(2):
        np.testing.assert_allclose(y[b], _torch_mha(g["x"][b], g["x"][b], g, inv[b]), rtol=1e-10, atol=1e-12)


def test_iem_is_three_independent_mhas_and_ifm_is_three_cross_attentions():
    g = tiny(seed=9, B=1, seg=(4, 7, 5), d=16, H=2, bias=True)
    off = [0, 4, 11, 16]
    x = g["x"][0]
    y = run(g, oracle.IM_IEM)[0]
    for s in range(3):
        xs = x[off[s]:off[s + 1]]
        np.testing.assert_allclose(y[off[s]:off[s + 1]], _torch_mha(xs, xs, g), rtol=1e-10, atol=1e-12)
    y = run(g, oracle.IM_IFM_FORWARD)[0]
    for i, j in ((0, 1), (1, 2), (2, 0)):
        np.testing.assert_allclose(y[off[i]:off[i + 1]],
                                   _torch_mha(x[off[i]:off[i + 1]], x[off[j]:off[j + 1]], g),
                                   rtol=1e-10, atol=1e-12)


def test_information_disorder_joint_softmax():
    """Sec. "Information Disorder": with (t,v) and (t,a) both live, the t rows are one softmax over [V_v; V_a]
    and differ from the single-block result; v and a rows are unchanged."""
    g = tiny(seed=13, B=1, seg=(4, 6, 5), d=16, H=2, bias=False)
    off = [0, 4, 10, 15]
    x = g["x"][0]
    lm_mod = oracle.IM_IFM_FORWARD | (1 << (0 * 3 + 2))
    y0 = run(g, oracle.IM_IFM_FORWARD)[0]
    y1 = run(g, lm_mod)[0]
    joint = _torch_mha(x[:4], x[4:], g)           # keys = vision then audio, one normalisation
    np.testing.assert_allclose(y1[:4], joint, rtol=1e-10, atol=1e-12)
    assert np.max(np.abs(y1[:4] - y0[:4])) > 1e-3
    np.testing.assert_array_equal(y1[4:], y0[4:])
    # the (t,v) attention weights themselves change (G_d^{t,v} != G_d^{t,v'})
    _, c0 = run(g, oracle.IM_IFM_FORWARD, return_cache=True)
    _, c1 = run(g, lm_mod, return_cache=True)
    assert np.max(np.abs(c0["p"][0, :, :4, 4:10] - c1["p"][0, :, :4, 4:10])) > 1e-3
    np.testing.assert_allclose(c1["p"][0, :, :4, 4:].sum(-1), 1.0, rtol=1e-12)


@pytest.mark.parametrize("name", sorted(oracle.NAMED_PATTERNS))
def test_rows_are_stochastic_on_live_keys_and_zero_elsewhere(name):
    g = synth.attention_inputs(2, (6, 9, 7), 8, 2, "fp32", "valid_len", seed=21)
    lm = oracle.NAMED_PATTERNS[name]
    _, c = run(g, lm, return_cache=True)
    inv = oracle.key_invalid(g["seg_len"], 2, g["valid_len"], None)
    for b in range(2):
        live = np.isfinite(oracle.additive_mask(g["seg_len"], lm, inv[b]))
        p = c["p"][b]
        assert np.all(p[:, ~live] == 0.0)
        has_key = live.any(axis=1)
        np.testing.assert_allclose(p.sum(-1)[:, has_key], 1.0, rtol=1e-12)
        assert np.all(p.sum(-1)[:, ~has_key] == 0.0)
        assert np.all(p >= 0)


def test_dead_segment_contents_do_not_matter():
    """Worked block product of Sec. "Information Disorder": rows of modality i depend only on V_j of the live j."""
    g = tiny(seed=17, B=1, seg=(4, 6, 5), d=8, H=2, bias=True)
    y0 = run(g, oracle.IM_IFM_FORWARD)
    g2 = dict(g)
    x2 = g["x"].copy()
    x2[:, 10:15] = 1e3 * (1 + np.arange(5 * 8).reshape(5, 8))   # audio rows: dead for t-queries (t <- v only)
    g2["x"] = x2
    y1 = run(g2, oracle.IM_IFM_FORWARD)
    np.testing.assert_array_equal(y1[:, :4], y0[:, :4])          # t rows bit-identical
    assert np.max(np.abs(y1[:, 4:10] - y0[:, 4:10])) > 1.0       # v rows (v <- a) do change


def test_softmax_shift_and_key_permutation_invariance():
    g = tiny(seed=19, B=1, seg=(4, 6, 5), d=8, H=2, bias=True)
    y0 = run(g, oracle.IM_IFM_FORWARD)
    # a constant added to every key (via b_k) shifts every score of a row equally
    g2 = dict(g)
    # shifting K by a vector u adds q.u to the whole row: softmax unchanged
    g2["bk"] = g["bk"] + np.float32(3.0)
    np.testing.assert_allclose(run(g2, oracle.IM_IFM_FORWARD), y0, rtol=1e-9, atol=1e-11)
    # permuting the vision rows permutes vision outputs and leaves t rows (t <- v) unchanged
    perm = np.array([2, 0, 5, 1, 4, 3])
    g3 = dict(g)
    x3 = g["x"].copy()
    x3[:, 4:10] = g["x"][:, 4 + perm]
    g3["x"] = x3
    y3 = run(g3, oracle.IM_IFM_FORWARD)
    np.testing.assert_allclose(y3[:, :4], y0[:, :4], rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(y3[:, 4:10], y0[:, 4 + perm], rtol=1e-11, atol=1e-13)


def test_fully_masked_rows_give_bias_only_and_no_nan():
    g = tiny(seed=23, B=2, seg=(3, 4, 2), d=8, H=2, bias=True)
    g["valid_len"] = np.array([[3, 0, 2], [3, 4, 2]], dtype=np.int32)   # sample 0: no valid vision key
    y, c = run(g, oracle.IM_IFM_FORWARD, return_cache=True)
    assert np.all(np.isfinite(y))
    np.testing.assert_allclose(y[0, :3], np.broadcast_to(g["bo"], (3, 8)), rtol=0, atol=1e-15)
    assert np.all(np.isneginf(c["lse"][0, :, :3]))
    assert np.all(np.isfinite(c["lse"][1]))


def test_scale_and_head_split_matter():
    """Guards against a dropped scale or a wrong head partition (plausible slips)."""
    g = tiny(seed=29, B=1, seg=(3, 4, 2), d=8, H=2, bias=False)
    lm = oracle.IM_IFM_FORWARD
    g_half = dict(g, scale=g["scale"] * 0.5)
    assert np.max(np.abs(run(g, lm) - run(g_half, lm))) > 1e-3
    np.testing.assert_allclose(run(g_half, lm), brute_force(g_half, lm), rtol=1e-12, atol=1e-13)
    g_h4 = dict(g, n_heads=4, scale=0.5)
    assert np.max(np.abs(run(g_h4, lm) - run(dict(g, scale=0.5), lm))) > 1e-3
    np.testing.assert_allclose(run(g_h4, lm), brute_force(g_h4, lm), rtol=1e-12, atol=1e-13)


def test_live_pair_count_matches_complexity_appendix():
    """App. B, "Attention 1, w/ Decomposition": the cost factor is T_t T_v + T_t T_a + T_v T_a,
    equal to MulT's; the dense pass would touch T_m^2."""
    for seg in ((50, 375, 500), (50, 500, 500), (39, 400, 55), (30, 230, 480)):   # dataset table
        tt, tv, ta = seg
        cross = tt * tv + tt * ta + tv * ta
        assert oracle.live_pair_count(seg, oracle.IM_IFM_FORWARD, 1) == cross
        assert oracle.live_pair_count(seg, oracle.IM_IFM_BACKWARD, 1) == cross
        assert oracle.live_pair_count(seg, oracle.IM_IEM, 1) == tt * tt + tv * tv + ta * ta
        assert oracle.live_pair_count(seg, oracle.IM_DENSE, 1) == (tt + tv + ta) ** 2
    vl = np.array([[2, 3, 1]])
    assert oracle.live_pair_count((4, 5, 3), oracle.IM_IFM_FORWARD, 1, valid_len=vl) == 4 * 3 + 5 * 1 + 3 * 2
