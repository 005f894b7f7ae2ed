"""Pins for the encoder-layer backward oracle (CPU only): finite differences of the forward
oracle, LayerNorm-gradient invariants, GELU' closed form."""
import math

import numpy as np
import pytest

import oracle
from paper_2505_01068_amd import synth


def test_gelu_grad_closed_form_and_finite_difference():
    # Phi(1) = 0.8413447460685429, phi(1) = 0.24197072451914337
    np.testing.assert_allclose(oracle.gelu_grad(1.0), 0.8413447460685429 + 0.24197072451914337, rtol=1e-14)
    np.testing.assert_allclose(oracle.gelu_grad(0.0), 0.5, rtol=1e-15)
    x = np.linspace(-5, 5, 101)
    np.testing.assert_allclose(oracle.gelu_grad(x) + oracle.gelu_grad(-x), 1.0, rtol=1e-13)   # derivative of the odd-part identity
    h = 1e-5
    fd = (oracle.gelu(x + h) - oracle.gelu(x - h)) / (2 * h)
    np.testing.assert_allclose(oracle.gelu_grad(x), fd, rtol=1e-8, atol=1e-9)


def test_layer_norm_backward_invariants_and_fd():
    rng = np.random.default_rng(3)
    x = rng.normal(size=(5, 24)) * 2 + 1
    g, b = rng.normal(size=24), rng.normal(size=24)
    dy = rng.normal(size=(5, 24))
    eps = 1e-5
    dx, dg, db = oracle.layer_norm_backward(x, g, eps, dy)
    # LN is invariant to adding a constant to a row, and (for eps -> 0) to scaling the centred row:
    # dx is orthogonal to the ones vector, and nearly orthogonal to x - mean
    np.testing.assert_allclose(dx.sum(-1), 0.0, atol=1e-12)
    xc = x - x.mean(-1, keepdims=True)
    assert np.max(np.abs((dx * xc).sum(-1))) < 1e-4 * np.max(np.abs(dx)) * np.max(np.abs(xc)) * 24
    np.testing.assert_allclose(db, dy.sum(0), rtol=1e-14)
    f = lambda x_, g_, b_: float((oracle.layer_norm(x_, g_, b_, eps) * dy).sum())
    for arr, grad in ((x, dx), (g, dg), (b, db)):
        d = rng.normal(size=arr.shape)
        hh = 1e-6
        args = lambda t: [arr + t * d if a is arr else a for a in (x, g, b)]
        fd = (f(*args(hh)) - f(*args(-hh))) / (2 * hh)
        np.testing.assert_allclose((grad * d).sum(), fd, rtol=1e-7)


def _problem(seed, padding, bias=True, lm=oracle.IM_IFM_FORWARD, seg=(3, 6, 4), d=8, H=2, d_ff=12, B=2):
    g = synth.attention_inputs(B, seg, d, H, "fp32", padding, seed=seed)
    p = synth.layer_params(d, d_ff, seed, 0, dtype="fp32", bias=bias)
    kw = dict(seg_len=g["seg_len"], live_mask=lm, n_heads=H, scale=g["scale"], valid_len=g.get("valid_len"), key_pad=g.get("key_pad"))
    return g, p, kw


@pytest.mark.parametrize("padding,bias,lm", [("none", True, oracle.IM_IFM_FORWARD), ("valid_len", True, oracle.IM_IFM_BACKWARD),
                                             ("key_pad", False, oracle.IM_IEM), ("valid_len", True, oracle.NAMED_PATTERNS["self_only"])])
def test_layer_backward_matches_finite_differences(padding, bias, lm):
    g, p, kw = _problem(71, padding, bias, lm)
    x = g["x"].astype(np.float64)
    rng = np.random.default_rng(5)
    dy = rng.normal(size=x.shape)
    grads = oracle.gsit_layer_backward(x, p, dy, **kw)
    loss = lambda x_, p_: float((oracle.gsit_layer_forward(x_, p_, **kw) * dy).sum())
    hh = 1e-6
    # input
    dirx = rng.normal(size=x.shape)
    fd = (loss(x + hh * dirx, p) - loss(x - hh * dirx, p)) / (2 * hh)
    np.testing.assert_allclose((grads["dx"] * dirx).sum(), fd, rtol=2e-6, atol=1e-8)
    # every parameter
    for n, v in p.items():
        if v is None:
            assert "d" + n not in grads
            continue
        dirp = rng.normal(size=v.shape)
        pp, pm = dict(p), dict(p)
        pp[n] = v.astype(np.float64) + hh * dirp
        pm[n] = v.astype(np.float64) - hh * dirp
        fd = (loss(x, pp) - loss(x, pm)) / (2 * hh)
        np.testing.assert_allclose((grads["d" + n] * dirp).sum(), fd, rtol=5e-6, atol=1e-8, err_msg=n)


def test_layer_backward_identity_layer():
    # output-side weights zero: y = x, so dx = dy and the only non-zero parameter gradients are those
    # of wo, bo, w2, b2
    g, p, kw = _problem(72, "none")
    for n in ("wo", "bo", "w2", "b2"):
        p[n] = np.zeros_like(p[n])
    dy = np.random.default_rng(6).normal(size=g["x"].shape)
    grads = oracle.gsit_layer_backward(g["x"], p, dy, **kw)
    np.testing.assert_allclose(grads["dx"], dy, rtol=0, atol=1e-15)
    for n in ("ln1_g", "ln1_b", "wq", "wk", "wv", "bq", "bk", "bv", "ln2_g", "ln2_b", "w1", "b1"):
        assert np.max(np.abs(grads["d" + n])) < 1e-14, n
    np.testing.assert_allclose(grads["db2"], dy.sum((0, 1)), rtol=1e-13)
    np.testing.assert_allclose(grads["dbo"], dy.sum((0, 1)), rtol=1e-13)
