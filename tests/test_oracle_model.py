"""Pins for the model-level oracle (CPU only): Sec. 5, Eq. "allmodalinone fusion"."""
import copy

import numpy as np

import oracle
from paper_2505_01068_amd import synth


def _problem(seed=61, B=3, seg=(3, 6, 4), d=8, H=2, d_ff=16, L=2, Li=1, n_out=5, padding="valid_len"):
    g = synth.attention_inputs(B, seg, d, H, "fp32", padding, seed=seed, with_dy=False)
    m = synth.model_params(d, d_ff, 2 * d_ff, L, Li, len(seg), n_out, seed, dtype="fp32")
    kw = dict(seg_len=g["seg_len"], n_heads=H, scale=g["scale"], n_heads_intra=H, scale_intra=1.0 / np.sqrt(2 * d / H),
              valid_len=g.get("valid_len"), key_pad=g.get("key_pad"))
    return g, m, kw


def test_last_steps_positions():
    a = np.arange(2 * 9 * 2, dtype=np.float64).reshape(2, 9, 2)
    z = oracle.last_steps(a, (2, 3, 4))
    np.testing.assert_array_equal(z[0], np.concatenate([a[0, 1], a[0, 4], a[0, 8]]))
    vl = np.array([[1, 3, 2], [2, 0, 4]])
    z = oracle.last_steps(a, (2, 3, 4), vl)
    np.testing.assert_array_equal(z[0], np.concatenate([a[0, 0], a[0, 4], a[0, 6]]))
    np.testing.assert_array_equal(z[1], np.concatenate([a[1, 1], a[1, 2], a[1, 8]]))   # valid length 0 -> position 0


def test_identity_encoders_closed_form():
    # output-side weights zero: every layer is the identity, so X = f(|| [x_last || x_last])
    g, m, kw = _problem()
    for layers in (m["fwd_layers"], m["bwd_layers"], m["intra_layers"]):
        for p in layers:
            for n in ("wo", "bo", "w2", "b2"):
                p[n] = np.zeros_like(p[n])
    out = oracle.gsit_model_forward(g["x"], m, **kw)
    x = g["x"].astype(np.float64)
    off = np.concatenate([[0], np.cumsum(g["seg_len"])])
    want = np.zeros((x.shape[0], m["wf"].shape[1]))
    for b in range(x.shape[0]):
        parts = []
        for s in range(3):
            pos = off[s] + max(min(int(g["valid_len"][b, s]), g["seg_len"][s]), 1) - 1
            parts += [x[b, pos], x[b, pos]]
        want[b] = np.concatenate(parts) @ m["wf"].astype(np.float64) + m["bf"]
    np.testing.assert_allclose(out, want, rtol=1e-13, atol=1e-13)


def _encoder_mult_form(x, layers, seg_len, live_mask, H, scale, eps, valid_len, key_pad):
    """Encoder in which every attention is evaluated as separate CMA / MHSA blocks (MulT form)."""
    x = np.asarray(x, np.float64)
    for p in layers:
        u = oracle.layer_norm(x, p["ln1_g"], p["ln1_b"], eps)
        att = oracle.mult_blocks_forward(u, p["wq"], p["wk"], p["wv"], p["wo"], seg_len, live_mask, H, scale,
                                         bq=p["bq"], bk=p["bk"], bv=p["bv"], bo=p["bo"], valid_len=valid_len, key_pad=key_pad)
        h = x + att
        v = oracle.layer_norm(h, p["ln2_g"], p["ln2_b"], eps)
        x = h + oracle.gelu(v @ p["w1"].astype(np.float64) + p["b1"]) @ p["w2"].astype(np.float64) + p["b2"]
    return x


def test_model_equals_block_separated_form():
    # Sec. 5: the interlaced-mask encoders equal the MulT-style separate cross-/self-attention blocks
    for padding in ("valid_len", "none"):
        g, m, kw = _problem(seed=62, padding=padding)
        out, parts = oracle.gsit_model_forward(g["x"], m, return_parts=True, **kw)
        eps = 1e-5
        a = (g["seg_len"],)
        F = _encoder_mult_form(g["x"], m["fwd_layers"], *a, oracle.IM_IFM_FORWARD, kw["n_heads"], kw["scale"], eps, kw["valid_len"], kw["key_pad"])
        Bk = _encoder_mult_form(g["x"], m["bwd_layers"], *a, oracle.IM_IFM_BACKWARD, kw["n_heads"], kw["scale"], eps, kw["valid_len"], kw["key_pad"])
        A = _encoder_mult_form(np.concatenate([F, Bk], -1), m["intra_layers"], *a, oracle.IM_IEM, kw["n_heads_intra"], kw["scale_intra"], eps, kw["valid_len"], kw["key_pad"])
        np.testing.assert_allclose(parts["F"], F, rtol=1e-11, atol=1e-12)
        np.testing.assert_allclose(parts["B"], Bk, rtol=1e-11, atol=1e-12)
        np.testing.assert_allclose(parts["A"], A, rtol=1e-11, atol=1e-12)
        z = oracle.last_steps(A, g["seg_len"], kw["valid_len"])
        np.testing.assert_allclose(out, z @ m["wf"].astype(np.float64) + m["bf"], rtol=1e-11, atol=1e-12)


def test_halves_come_from_their_own_encoders():
    # F fills columns [0, d), B columns [d, 2d) of the IEM encoder's input: changing only the backward
    # encoder's weights leaves F untouched, and vice versa; swapping the two stacks AND the two masks
    # swaps the halves.
    g, m, kw = _problem(seed=63)
    _, p0 = oracle.gsit_model_forward(g["x"], m, return_parts=True, **kw)
    m2 = copy.deepcopy(m)
    m2["bwd_layers"][0]["w1"] = m2["bwd_layers"][0]["w1"] * 1.5
    _, p1 = oracle.gsit_model_forward(g["x"], m2, return_parts=True, **kw)
    np.testing.assert_array_equal(p0["F"], p1["F"])
    assert np.max(np.abs(p0["B"] - p1["B"])) > 1e-6
    m3 = copy.deepcopy(m)
    m3["fwd_layers"], m3["bwd_layers"] = m["bwd_layers"], m["fwd_layers"]
    _, p3 = oracle.gsit_model_forward(g["x"], m3, return_parts=True, mask_fwd=oracle.IM_IFM_BACKWARD,
                                      mask_bwd=oracle.IM_IFM_FORWARD, **kw)
    np.testing.assert_array_equal(p3["F"], p0["B"])
    np.testing.assert_array_equal(p3["B"], p0["F"])


def test_modalities_do_not_mix_in_the_intra_encoder():
    # under the IEM a segment's rows of A depend only on that segment's rows of F || B: perturb the
    # text rows of x's image under the inter encoders by perturbing the intra input directly
    g, m, kw = _problem(seed=64, padding="none")
    _, p0 = oracle.gsit_model_forward(g["x"], m, return_parts=True, **kw)
    vbar = np.concatenate([p0["F"], p0["B"]], -1)
    vbar2 = vbar.copy()
    vbar2[:, :g["seg_len"][0]] += 0.3
    A0 = oracle.gsit_encoder_forward(vbar, m["intra_layers"], g["seg_len"], oracle.IM_IEM, kw["n_heads_intra"], kw["scale_intra"])
    A2 = oracle.gsit_encoder_forward(vbar2, m["intra_layers"], g["seg_len"], oracle.IM_IEM, kw["n_heads_intra"], kw["scale_intra"])
    t = g["seg_len"][0]
    np.testing.assert_array_equal(A0[:, t:], A2[:, t:])
    assert np.max(np.abs(A0[:, :t] - A2[:, :t])) > 1e-3
    np.testing.assert_allclose(A0, p0["A"], rtol=1e-13, atol=1e-13)
