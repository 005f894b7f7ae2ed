"""Pins for the encoder-layer oracle (CPU only)."""
import math

import numpy as np

import oracle
from paper_2505_01068_amd import synth


def test_layer_norm_closed_form():
    rng = np.random.default_rng(1)
    x = rng.normal(size=(7, 64)) * 3 + 2
    eps = 1e-5
    y = oracle.layer_norm(x, np.ones(64), np.zeros(64), eps)
    var = x.var(axis=-1)                                     # biased
    np.testing.assert_allclose(y.mean(-1), 0.0, atol=1e-14)
    np.testing.assert_allclose(y.var(-1), var / (var + eps), rtol=1e-12)
    g, b = rng.normal(size=64), rng.normal(size=64)
    np.testing.assert_allclose(oracle.layer_norm(x, g, b, eps), y * g + b, rtol=1e-13, atol=1e-13)
    # hand-evaluated two-element row: (1,3) -> mean 2, var 1
    np.testing.assert_allclose(oracle.layer_norm(np.array([[1.0, 3.0]]), [2.0, 2.0], [0.5, 0.5], 0.0), [[-1.5, 2.5]])


def test_gelu_closed_forms():
    assert oracle.gelu(0.0) == 0.0
    x = np.linspace(-6, 6, 241)
    np.testing.assert_allclose(oracle.gelu(x) - oracle.gelu(-x), x, rtol=1e-14, atol=1e-15)
    # x * Phi(x) with tabulated Phi(1) = 0.8413447460685429, Phi(2) = 0.9772498680518208
    np.testing.assert_allclose(oracle.gelu(1.0), 0.8413447460685429, rtol=1e-14)
    np.testing.assert_allclose(oracle.gelu(2.0), 2 * 0.9772498680518208, rtol=1e-14)
    np.testing.assert_allclose(oracle.gelu(-1.0), -(1 - 0.8413447460685429), rtol=1e-13)
    np.testing.assert_allclose(oracle.gelu(x), [0.5 * v * (1 + math.erf(v / math.sqrt(2))) for v in x], rtol=1e-14, atol=1e-300)


def _layer_problem(seed=51, B=2, seg=(3, 6, 4), d=8, H=2, d_ff=32):
    g = synth.attention_inputs(B, seg, d, H, "fp32", "valid_len", seed=seed)
    p = synth.layer_params(d, d_ff, seed, 0, dtype="fp32")
    return g, p


def test_layer_is_identity_when_output_weights_vanish():
    g, p = _layer_problem()
    for n in ("wo", "bo", "w2", "b2"):
        p[n] = np.zeros_like(p[n])
    y = oracle.gsit_layer_forward(g["x"], p, g["seg_len"], oracle.IM_IFM_FORWARD, g["n_heads"], g["scale"],
                                  valid_len=g["valid_len"])
    np.testing.assert_array_equal(y, g["x"].astype(np.float64))


def test_layer_scalar_brute_force():
    g, p = _layer_problem()
    lm = oracle.IM_IFM_BACKWARD
    eps = 1e-5
    y = oracle.gsit_layer_forward(g["x"], p, g["seg_len"], lm, g["n_heads"], g["scale"], eps, valid_len=g["valid_len"])
    x = g["x"].astype(np.float64)
    B, T, d = x.shape

    def ln_row(r, gam, bet):
        mu = sum(r) / len(r)
        var = sum((v - mu) ** 2 for v in r) / len(r)
        return [(v - mu) / math.sqrt(var + eps) * ga + be for v, ga, be in zip(r, gam, bet)]

    u = np.array([[ln_row(x[b, t].tolist(), p["ln1_g"].tolist(), p["ln1_b"].tolist()) for t in range(T)] for b in range(B)])
    # attention on u: the forward oracle is pinned on its own (test_oracle_attention.py)
    att = oracle.forward(u, p["wq"], p["wk"], p["wv"], p["wo"], g["seg_len"], lm, g["n_heads"], g["scale"],
                         bq=p["bq"], bk=p["bk"], bv=p["bv"], bo=p["bo"], valid_len=g["valid_len"])
    h = x + att
    w1, w2 = p["w1"].astype(float).tolist(), p["w2"].astype(float).tolist()
    b1, b2 = p["b1"].astype(float).tolist(), p["b2"].astype(float).tolist()
    d_ff = len(b1)
    for b in range(B):
        for t in range(T):
            v = ln_row(h[b, t].tolist(), p["ln2_g"].tolist(), p["ln2_b"].tolist())
            z = [sum(v[i] * w1[i][j] for i in range(d)) + b1[j] for j in range(d_ff)]
            a = [0.5 * zz * (1 + math.erf(zz / math.sqrt(2))) for zz in z]
            f = [sum(a[j] * w2[j][o] for j in range(d_ff)) + b2[o] for o in range(d)]
            np.testing.assert_allclose(y[b, t], h[b, t] + np.array(f), rtol=1e-12, atol=1e-13)


def test_encoder_is_repeated_layer():
    g, _ = _layer_problem()
    layers = [synth.layer_params(8, 32, 51, l, dtype="fp32") for l in range(3)]
    lm = oracle.IM_IEM
    y = oracle.gsit_encoder_forward(g["x"], layers, g["seg_len"], lm, g["n_heads"], g["scale"], valid_len=g["valid_len"])
    z = g["x"]
    for p in layers:
        z = oracle.gsit_layer_forward(z, p, g["seg_len"], lm, g["n_heads"], g["scale"], valid_len=g["valid_len"])
    np.testing.assert_array_equal(y, z)
    assert np.abs(y - g["x"]).max() > 0.1
