"""Dense fp64 definition of multi-head attention under the Interlaced Mask (IM).

TEST INFRASTRUCTURE ONLY (see the package docstring).

Notation follows the paper.  The three modality sequences are concatenated in
the order text, vision, audio into one vertex sequence V_m of length
T_m = T_t + T_v + T_a (Sec. 3, "Multimodal Transformers as Graphs"); one set of
projection weights W_q, W_k, W_v is applied to every row of V_m (Sec. 3; App. A,
Eq. "adjmat_all").  The block score matrix A = (V_m W_q)(V_m W_k)^T is a 3x3 grid
of blocks E^{i,j} with i the query modality and j the key/value modality
(App. A, "Graph Structure Construction").  The IM adds an all-zero block O or
an all-minus-infinity block J to each E^{i,j} before the row softmax
(Sec. 5, Eq. "ifm" and the IEM equation; Eq. "allmodalinone fusion").

The method computes exactly this dense result (it merely never touches blocks
whose softmax weight is exp(-inf) = 0), so the oracle is the dense definition.

Parity pins (tests/test_oracle_*.py): scalar-loop brute force on tiny inputs,
the equivalence with separately computed cross-modal / self attention of the
paper (Sec. 4 and Lemma 1), the joint-softmax behaviour of Sec. "Information Disorder"
("Information Disorder"), row-stochastic and zero-block invariants, the
special cases that reduce to textbook multi-head attention, the 3x3 patterns
printed in the paper (tests/golden/im_patterns.txt), the live-pair count of the
complexity appendix, and central finite differences for the backward pass.
The paper prints no numeric attention output, so agreement with "the paper's
numbers" is unpinned by necessity; nothing here is "parity unpinned" otherwise.

Conventions (each is a reading of a point the paper leaves open):
  * weights are [d_in, d_out] and applied as x @ W (Sec. 3 writes
    W in R^{d x d^f});
  * `scale` multiplies the scores before the softmax (App. B says "apply
    scaling and softmax"; the operator D of Eq. "softmax_staff");
  * a key is padding if key_pad[b, c] != 0 or its position inside its segment
    is >= valid_len[b, seg]; padded keys get -inf; padded query rows are
    computed like any other row;
  * a row whose every key is masked has attention output 0 (so y = b_o) and
    contributes nothing to any gradient;
  * rows with several live blocks share ONE softmax over all their live keys
    (the additive -inf definition; Sec. "Information Disorder").
"""
from __future__ import annotations

import numpy as np

# Segment order (t, v, a) = (0, 1, 2); bit (i * n_seg + j) set <=> block
# (query segment i, key segment j) is O (live).  Sec. 5, Eq. "ifm" / IEM.
IM_IFM_FORWARD = (1 << (0 * 3 + 1)) | (1 << (1 * 3 + 2)) | (1 << (2 * 3 + 0))
IM_IFM_BACKWARD = (1 << (0 * 3 + 2)) | (1 << (1 * 3 + 0)) | (1 << (2 * 3 + 1))
IM_IEM = (1 << 0) | (1 << 4) | (1 << 8)
IM_DENSE = (1 << 9) - 1


def live_mask_from_edges(edges, n_seg=3, names="tva"):
    """Bit mask from a list of information-flow edges 'j->i' (from V_j to V_i).

    The ablation section writes a structure as a set of fusion operations
    j -> i meaning "from V_j to V_i", i.e. query modality i, key modality j.
    """
    m = 0
    for e in edges:
        src, dst = e.split("->")
        j, i = names.index(src.strip()), names.index(dst.strip())
        m |= 1 << (i * n_seg + j)
    return m


# Patterns used in the paper.  The ablation structures follow the edge sets in
# the text of Sec. "Ablation Study" / App. "Graph Structures" (for Structure-1 the text, not the garbled
# matrix, see the design notes); Self-Only follows the printed matrix of App. "Graph Structures":
# J on the diagonal and O elsewhere (two live blocks per row, which is what
# makes it the information-disorder case).
NAMED_PATTERNS = {
    "ifm_forward": IM_IFM_FORWARD,
    "ifm_backward": IM_IFM_BACKWARD,
    "iem": IM_IEM,
    "dense": IM_DENSE,
    "structure1_a": live_mask_from_edges(["a->v", "v->a", "a->t"]),
    "structure1_b": live_mask_from_edges(["v->t", "t->v", "t->a"]),
    "structure2_a": live_mask_from_edges(["v->t", "t->v", "v->a"]),
    "structure2_b": live_mask_from_edges(["a->t", "t->a", "a->v"]),
    "structure3_a": live_mask_from_edges(["a->v", "v->a", "v->t"]),
    "structure3_b": live_mask_from_edges(["a->t", "t->a", "t->v"]),
    "self_only": IM_DENSE ^ IM_IEM,
}


def segment_of_rows(seg_len):
    """seg[r] = index of the modality segment row r of V_m belongs to; pos[r] = offset in it."""
    seg = np.concatenate([np.full(int(n), s, dtype=np.int64) for s, n in enumerate(seg_len)])
    pos = np.concatenate([np.arange(int(n), dtype=np.int64) for n in seg_len])
    return seg, pos


def key_invalid(seg_len, batch, valid_len=None, key_pad=None):
    """Boolean [B, T_m]: True where the key at that position is padding."""
    seg, pos = segment_of_rows(seg_len)
    inv = np.zeros((batch, seg.size), dtype=bool)
    if valid_len is not None:
        vl = np.asarray(valid_len).reshape(batch, len(seg_len))
        inv |= pos[None, :] >= vl[:, seg]
    if key_pad is not None:
        inv |= np.asarray(key_pad).reshape(batch, seg.size) != 0
    return inv


def additive_mask(seg_len, live_mask, invalid_b=None):
    """The IM as a dense [T_m, T_m] matrix of 0 / -inf blocks (Eq. "ifm", IEM).

    Entry (r, c) is 0 iff the block (segment of r, segment of c) is O, else
    -inf; columns of padded keys are -inf as well.
    """
    n_seg = len(seg_len)
    seg, _ = segment_of_rows(seg_len)
    blocks = np.array([[(int(live_mask) >> (i * n_seg + j)) & 1 for j in range(n_seg)]
                       for i in range(n_seg)], dtype=bool)
    live = blocks[seg[:, None], seg[None, :]]
    if invalid_b is not None:
        live = live & ~np.asarray(invalid_b, dtype=bool)[None, :]
    return np.where(live, 0.0, -np.inf)


def live_pair_count(seg_len, live_mask, batch, valid_len=None, key_pad=None):
    """Number of (query row, valid live key) pairs over the batch.

    With no padding and an IFM this is B (T_t T_v + T_t T_a + T_v T_a), the
    factor of the "w/ Decomposition" attention cost in App. B.
    """
    inv = key_invalid(seg_len, batch, valid_len, key_pad)
    return int(sum(np.isfinite(additive_mask(seg_len, live_mask, inv[b])).sum() for b in range(batch)))


def _f64(a):
    return None if a is None else np.asarray(a, dtype=np.float64)


def project_qkv(x, wq, wk, wv, bq=None, bk=None, bv=None):
    """Shared projection of every row of V_m (Sec. 3; App. A Eq. "adjmat_all")."""
    x = _f64(x)
    q = x @ _f64(wq)
    k = x @ _f64(wk)
    v = x @ _f64(wv)
    if bq is not None:
        q = q + _f64(bq)
    if bk is not None:
        k = k + _f64(bk)
    if bv is not None:
        v = v + _f64(bv)
    return q, k, v


def _softmax_rows(s):
    """Row softmax with exp(-inf) = 0; an all -inf row gives an all-zero row."""
    m = np.max(s, axis=-1, keepdims=True)
    m = np.where(np.isfinite(m), m, 0.0)
    e = np.exp(s - m)
    l = np.sum(e, axis=-1, keepdims=True)
    p = np.divide(e, l, out=np.zeros_like(e), where=l > 0)
    with np.errstate(divide="ignore"):
        lse = np.where(l > 0, m + np.log(l), -np.inf)
    return p, lse[..., 0]


def forward(x, wq, wk, wv, wo, seg_len, live_mask, n_heads, scale,
            bq=None, bk=None, bv=None, bo=None, valid_len=None, key_pad=None,
            return_cache=False):
    """IM attention: y[B, T_m, d].

    Per batch element and head l: S = scale * Q_l K_l^T + M, P = rowsoftmax(S),
    O_l = P V_l, heads concatenated along the feature axis (App. A, multi-head
    equation), then y = O W_o + b_o.
    """
    x = _f64(x)
    B, T, d = x.shape
    assert T == int(sum(seg_len)) and d % n_heads == 0
    dh = d // n_heads
    q, k, v = project_qkv(x, wq, wk, wv, bq, bk, bv)
    inv = key_invalid(seg_len, B, valid_len, key_pad)
    o = np.zeros((B, T, d))
    p_all = np.zeros((B, n_heads, T, T)) if return_cache else None
    lse_all = np.zeros((B, n_heads, T))
    for b in range(B):
        m = additive_mask(seg_len, live_mask, inv[b])
        for h in range(n_heads):
            c = slice(h * dh, (h + 1) * dh)
            s = scale * (q[b, :, c] @ k[b, :, c].T) + m
            p, lse = _softmax_rows(s)
            o[b, :, c] = p @ v[b, :, c]
            lse_all[b, h] = lse
            if return_cache:
                p_all[b, h] = p
    y = o @ _f64(wo)
    if bo is not None:
        y = y + _f64(bo)
    if return_cache:
        cache = dict(x=x, q=q, k=k, v=v, p=p_all, o=o, lse=lse_all, wq=_f64(wq), wk=_f64(wk),
                     wv=_f64(wv), wo=_f64(wo), n_heads=n_heads, scale=float(scale),
                     has_bias=(bq is not None, bk is not None, bv is not None, bo is not None))
        return y, cache
    return y


def backward(cache, dy):
    """Gradient of `forward` w.r.t. x and every weight / bias, by the chain rule.

    The paper gives no backward pass; this is the calculus of the forward
    definition (softmax Jacobian dS = P * (dP - rowsum(P * dP))), pinned by
    central finite differences in the tests.
    """
    x, q, k, v, p, o = (cache[n] for n in ("x", "q", "k", "v", "p", "o"))
    wq, wk, wv, wo = (cache[n] for n in ("wq", "wk", "wv", "wo"))
    H, scale = cache["n_heads"], cache["scale"]
    dy = _f64(dy)
    B, T, d = x.shape
    dh = d // H
    d_o = dy @ wo.T
    dwo = np.einsum("bti,btj->ij", o, dy)
    dbo = dy.sum(axis=(0, 1))
    dq = np.zeros_like(q)
    dk = np.zeros_like(k)
    dv = np.zeros_like(v)
    for b in range(B):
        for h in range(H):
            c = slice(h * dh, (h + 1) * dh)
            pb = p[b, h]
            dv[b, :, c] = pb.T @ d_o[b, :, c]
            dp = d_o[b, :, c] @ v[b, :, c].T
            ds = pb * (dp - np.sum(pb * dp, axis=-1, keepdims=True))
            dq[b, :, c] = scale * (ds @ k[b, :, c])
            dk[b, :, c] = scale * (ds.T @ q[b, :, c])
    g = dict(
        dx=dq @ wq.T + dk @ wk.T + dv @ wv.T,
        dwq=np.einsum("bti,btj->ij", x, dq),
        dwk=np.einsum("bti,btj->ij", x, dk),
        dwv=np.einsum("bti,btj->ij", x, dv),
        dwo=dwo,
        dbq=dq.sum(axis=(0, 1)), dbk=dk.sum(axis=(0, 1)), dbv=dv.sum(axis=(0, 1)), dbo=dbo,
        dq=dq, dk=dk, dv=dv, d_o=d_o,
    )
    return g


def _plain_mha(xq, xkv, wq, wk, wv, n_heads, scale, bq, bk, bv, kv_invalid):
    """Ordinary multi-head attention, queries from xq, keys/values from xkv (no out-projection)."""
    q = xq @ wq + (0.0 if bq is None else bq)
    k = xkv @ wk + (0.0 if bk is None else bk)
    v = xkv @ wv + (0.0 if bv is None else bv)
    d = q.shape[-1]
    dh = d // n_heads
    out = np.zeros((xq.shape[0], d))
    for h in range(n_heads):
        c = slice(h * dh, (h + 1) * dh)
        s = scale * (q[:, c] @ k[:, c].T)
        s = np.where(kv_invalid[None, :], -np.inf, s)
        p, _ = _softmax_rows(s)
        out[:, c] = p @ v[:, c]
    return out


def mult_blocks_forward(x, wq, wk, wv, wo, seg_len, live_mask, n_heads, scale,
                        bq=None, bk=None, bv=None, bo=None, valid_len=None, key_pad=None):
    """The same result in the MulT form (Sec. 3.2, Eq. "g_1"; Lemma 1).

    For every live block (i, j): cross-modal attention CMA(V_i, V_j) when
    i != j, self-attention MHSA(V_i) when i == j, with the SAME weights, written
    into the rows of segment i.  Only defined when every query segment has
    exactly one live block (all the paper's masks); the test of the paper's
    equivalence claim compares this with `forward`.
    """
    x = _f64(x)
    B, T, d = x.shape
    n_seg = len(seg_len)
    off = np.concatenate([[0], np.cumsum(seg_len)]).astype(int)
    inv = key_invalid(seg_len, B, valid_len, key_pad)
    wq, wk, wv, wo = _f64(wq), _f64(wk), _f64(wv), _f64(wo)
    bq, bk, bv = _f64(bq), _f64(bk), _f64(bv)
    o = np.zeros((B, T, d))
    for i in range(n_seg):
        js = [j for j in range(n_seg) if (int(live_mask) >> (i * n_seg + j)) & 1]
        if len(js) > 1:
            raise ValueError("MulT form needs at most one live block per query segment")
        for j in js:
            for b in range(B):
                o[b, off[i]:off[i + 1]] = _plain_mha(
                    x[b, off[i]:off[i + 1]], x[b, off[j]:off[j + 1]], wq, wk, wv,
                    n_heads, scale, bq, bk, bv, inv[b, off[j]:off[j + 1]])
    y = o @ wo
    if bo is not None:
        y = y + _f64(bo)
    return y
