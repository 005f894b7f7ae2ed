"""Dense fp64 definition of one GsiT encoder layer, a = MLP o MHSA_2 (Sec. 5,
Eq. "allmodalinone fusion"; MLP weights W_1 in R^{d^f x d^p}, W_2 in R^{d^p x d^f}
per App. B).

TEST INFRASTRUCTURE ONLY (see the package docstring).

The paper fixes only the composition "attention, then MLP".  The block
structure used here is the reading the benchmark configuration states: pre-
LayerNorm, residual connection around each of the two sub-blocks, exact (erf)
GELU, hidden width d_ff:

    u = LN(x; g1, beta1)      h = x + IMAttention(u)
    v = LN(h; g2, beta2)      y = h + GELU(v W_1 + b_1) W_2 + b_2

LayerNorm is over the feature axis with the biased variance.

Pins (tests/test_oracle_layer.py): LayerNorm output moments in closed form,
GELU against the normal CDF and its odd-part identity GELU(x) - GELU(-x) = x,
the layer reducing to the identity when W_o, b_o, W_2, b_2 vanish, and to the
attention oracle plus a hand-evaluated MLP on a scalar-loop brute force.

`gsit_layer_backward` is the calculus of that forward (the paper analyses no backward pass).  Its
pins (tests/test_oracle_layer_backward.py): central finite differences of the forward oracle along
random directions for the input and for every parameter; LayerNorm's input gradient being
orthogonal to the all-ones vector and to the normalised row; GELU' against the closed form
Phi(x) + x phi(x) at tabulated points.
"""
from __future__ import annotations

import math

import numpy as np
from scipy.special import erf as _erf  # library primitive: the error function

from . import im_attention as _att


def layer_norm(x, gamma, beta, eps):
    x = np.asarray(x, dtype=np.float64)
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps) * np.asarray(gamma, np.float64) + np.asarray(beta, np.float64)


def gelu(x):
    """Exact GELU: x * Phi(x) with Phi the standard normal CDF."""
    x = np.asarray(x, dtype=np.float64)
    return 0.5 * x * (1.0 + _erf(x / math.sqrt(2.0)))


def gsit_layer_forward(x, p, seg_len, live_mask, n_heads, scale, eps=1e-5,
                       valid_len=None, key_pad=None):
    """One encoder layer.  `p` is a dict with ln1_g, ln1_b, wq, wk, wv, wo,
    bq, bk, bv, bo (biases may be None), ln2_g, ln2_b, w1, b1, w2, b2."""
    x = np.asarray(x, dtype=np.float64)
    u = layer_norm(x, p["ln1_g"], p["ln1_b"], eps)
    h = x + _att.forward(u, p["wq"], p["wk"], p["wv"], p["wo"], seg_len, live_mask, n_heads, scale,
                         bq=p.get("bq"), bk=p.get("bk"), bv=p.get("bv"), bo=p.get("bo"),
                         valid_len=valid_len, key_pad=key_pad)
    v = layer_norm(h, p["ln2_g"], p["ln2_b"], eps)
    z = v @ np.asarray(p["w1"], np.float64)
    if p.get("b1") is not None:
        z = z + np.asarray(p["b1"], np.float64)
    f = gelu(z) @ np.asarray(p["w2"], np.float64)
    if p.get("b2") is not None:
        f = f + np.asarray(p["b2"], np.float64)
    return h + f


def gelu_grad(x):
    """d/dx [x Phi(x)] = Phi(x) + x phi(x)."""
    x = np.asarray(x, dtype=np.float64)
    return 0.5 * (1.0 + _erf(x / math.sqrt(2.0))) + x * np.exp(-0.5 * x * x) / math.sqrt(2.0 * math.pi)


def layer_norm_backward(x, gamma, eps, dy):
    """Gradients of y = LN(x; gamma, beta) given dy: (dx, dgamma, dbeta)."""
    x = np.asarray(x, dtype=np.float64)
    dy = np.asarray(dy, dtype=np.float64)
    gamma = np.asarray(gamma, np.float64)
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + eps)
    xhat = (x - mu) * rstd
    a = dy * gamma
    dx = rstd * (a - a.mean(axis=-1, keepdims=True) - xhat * (a * xhat).mean(axis=-1, keepdims=True))
    red = tuple(range(x.ndim - 1))
    return dx, (dy * xhat).sum(axis=red), dy.sum(axis=red)


def gsit_layer_backward(x, p, dy, seg_len, live_mask, n_heads, scale, eps=1e-5, valid_len=None, key_pad=None):
    """Gradients of gsit_layer_forward w.r.t. x and every parameter: dict with dx and
    d<name> for each entry of `p` that is not None."""
    x = np.asarray(x, dtype=np.float64)
    dy = np.asarray(dy, dtype=np.float64)
    f64 = lambda n: None if p.get(n) is None else np.asarray(p[n], np.float64)
    # forward, keeping what the backward needs
    u = layer_norm(x, p["ln1_g"], p["ln1_b"], eps)
    att, cache = _att.forward(u, p["wq"], p["wk"], p["wv"], p["wo"], seg_len, live_mask, n_heads, scale,
                              bq=p.get("bq"), bk=p.get("bk"), bv=p.get("bv"), bo=p.get("bo"),
                              valid_len=valid_len, key_pad=key_pad, return_cache=True)
    h = x + att
    v = layer_norm(h, p["ln2_g"], p["ln2_b"], eps)
    w1, w2 = f64("w1"), f64("w2")
    z = v @ w1 + (0.0 if p.get("b1") is None else f64("b1"))
    a = gelu(z)
    red = (0, 1)
    g = {}
    # y = h + a W2 + b2
    g["dw2"] = np.einsum("bti,btj->ij", a, dy)
    if p.get("b2") is not None:
        g["db2"] = dy.sum(axis=red)
    dz = (dy @ w2.T) * gelu_grad(z)
    g["dw1"] = np.einsum("bti,btj->ij", v, dz)
    if p.get("b1") is not None:
        g["db1"] = dz.sum(axis=red)
    dv = dz @ w1.T
    dh_ln, g["dln2_g"], g["dln2_b"] = layer_norm_backward(h, p["ln2_g"], eps, dv)
    dh = dy + dh_ln
    # h = x + IMAttention(u)
    ga = _att.backward(cache, dh)
    for n in ("wq", "wk", "wv", "wo"):
        g["d" + n] = ga["d" + n]
    for n in ("bq", "bk", "bv", "bo"):
        if p.get(n) is not None:
            g["d" + n] = ga["d" + n]
    dx_ln, g["dln1_g"], g["dln1_b"] = layer_norm_backward(x, p["ln1_g"], eps, ga["dx"])
    g["dx"] = dh + dx_ln
    g["attn_dk"] = ga["dk"]   # intermediate of the attention backward (what dbk sums), for error scales in tests
    return g


def gsit_encoder_forward(x, layers, seg_len, live_mask, n_heads, scale, eps=1e-5,
                         valid_len=None, key_pad=None):
    """A stack of layers with independent weights and one mask (an "encoder" of Sec. 5)."""
    for p in layers:
        x = gsit_layer_forward(x, p, seg_len, live_mask, n_heads, scale, eps, valid_len, key_pad)
    return x
