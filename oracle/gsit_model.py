"""Dense fp64 definition of the GsiT model around the encoder layers (Sec. 5,
Eq. "allmodalinone fusion"):

    F = a(G_inter^forward)       an encoder over the concatenated sequence V_m under the forward IFM
    B = a(G_inter^backward)      a second encoder (own weights) under the backward IFM
    Vbar = F || B                feature concatenation, width 2d
    A = a(G_intra)               a third encoder, width 2d, under the IEM
    X = f( || Split(A)[-1] )     last time step of every modality segment, concatenated, final linear f

TEST INFRASTRUCTURE ONLY (see the package docstring).

Readings (the paper gives the composition only):
  * each encoder is a stack of the layers of oracle.gsit_layer with independent weights;
  * "[-1]" of a segment is its last VALID step when per-sample valid lengths are given
    (position valid_len - 1, or 0 if the valid length is 0), else its last position;
  * f is one linear map R^{n_seg * 2d} -> R^{n_out} with optional bias.

Pins (tests/test_oracle_model.py): with all output-side weights of the layers zero the encoders
are identities and X has the closed form f(|| [x_last || x_last]); the encoders recomputed with
the block-separated (MulT-form) attention give the same X (the equivalence of Sec. 5 / App. A at
model level); F and B depend on disjoint parameter sets and enter A only through their halves.
"""
from __future__ import annotations

import numpy as np

from . import gsit_layer as _layer
from . import im_attention as _att


def last_steps(a, seg_len, valid_len=None):
    """[B, T_m, w] -> [B, n_seg * w]: the last (valid) step of every segment, concatenated."""
    a = np.asarray(a, dtype=np.float64)
    B = a.shape[0]
    off = np.concatenate([[0], np.cumsum(seg_len)])
    out = []
    for s, n in enumerate(seg_len):
        if valid_len is None:
            pos = np.full(B, n - 1)
        else:
            pos = np.maximum(np.minimum(np.asarray(valid_len)[:, s], n), 1) - 1
        out.append(a[np.arange(B), off[s] + pos])
    return np.concatenate(out, axis=-1)


def gsit_model_forward(x, model, seg_len, n_heads, scale, n_heads_intra, scale_intra, eps=1e-5,
                       valid_len=None, key_pad=None, mask_fwd=_att.IM_IFM_FORWARD,
                       mask_bwd=_att.IM_IFM_BACKWARD, mask_intra=_att.IM_IEM, return_parts=False):
    """`model`: dict with fwd_layers, bwd_layers, intra_layers (lists of layer dicts), wf, bf."""
    x = np.asarray(x, dtype=np.float64)
    F = _layer.gsit_encoder_forward(x, model["fwd_layers"], seg_len, mask_fwd, n_heads, scale, eps, valid_len, key_pad)
    Bk = _layer.gsit_encoder_forward(x, model["bwd_layers"], seg_len, mask_bwd, n_heads, scale, eps, valid_len, key_pad)
    vbar = np.concatenate([F, Bk], axis=-1)
    A = _layer.gsit_encoder_forward(vbar, model["intra_layers"], seg_len, mask_intra, n_heads_intra, scale_intra, eps,
                                    valid_len, key_pad)
    z = last_steps(A, seg_len, valid_len)
    out = z @ np.asarray(model["wf"], np.float64)
    if model.get("bf") is not None:
        out = out + np.asarray(model["bf"], np.float64)
    if return_parts:
        return out, dict(F=F, B=Bk, A=A, z=z)
    return out
