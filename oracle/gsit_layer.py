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


def gsit_encoder_forward(x, layers, seg_len, live_mask, n_heads, scale, eps=1e-5,
                         valid_len=None, key_pad=None):
    """A stack of layers with independent weights and one mask (an "encoder" of Sec. 5)."""
    for p in layers:
        x = gsit_layer_forward(x, p, seg_len, live_mask, n_heads, scale, eps, valid_len, key_pad)
    return x
