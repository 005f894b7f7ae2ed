"""Host-only checks of the C ABI: the library loads, exports every declared symbol,
rejects bad arguments before touching a GPU, and its schedule enumerates exactly the live blocks."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import oracle
from paper_2505_01068_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_every_declared_symbol_is_exported():
    hdr = open(os.path.join(ROOT, "include", "imattn.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = re.findall(r"^\s*(?:const\s+char\s*\*|int)\s+(\w+)\s*\(", hdr, flags=re.M)
    assert set(names) >= {"im_attention_fwd", "im_attention_bwd", "gsit_layer_fwd", "im_attention_sizes",
                          "gsit_layer_sizes", "gsit_model_sizes", "gsit_model_fwd", "im_schedule_build", "im_last_error",
                          "im_version", "im_attention_fwd_noalloc", "im_noalloc_init"}
    L = B.lib()
    for n in names:
        assert hasattr(L, n), n
    assert b"gfx950" in L.im_version()


def test_named_constants_agree_with_header_and_oracle():
    hdr = open(os.path.join(ROOT, "include", "imattn.h")).read()
    vals = {m.group(1): int(m.group(2), 16) for m in re.finditer(r"#define (IM_\w+) (0x[0-9A-Fa-f]+)ull", hdr)}
    assert vals["IM_IFM_FORWARD"] == oracle.IM_IFM_FORWARD == B.IM_IFM_FORWARD
    assert vals["IM_IFM_BACKWARD"] == oracle.IM_IFM_BACKWARD == B.IM_IFM_BACKWARD
    assert vals["IM_IEM"] == oracle.IM_IEM == B.IM_IEM
    assert vals["IM_DENSE3"] == oracle.IM_DENSE == B.IM_DENSE
    # every named pattern of the ablation: header constant == binding table == the oracle's (which the golden
    # file pins to the printed matrices and edge lists)
    assert set(B.NAMED_MASKS) == set(oracle.NAMED_PATTERNS)
    for name, bits in oracle.NAMED_PATTERNS.items():
        assert B.NAMED_MASKS[name] == bits, name
        assert vals["IM_DENSE3" if name == "dense" else "IM_" + name.upper()] == bits, name


def test_batch_limit_and_alignment_are_checked_on_the_host():
    L = B.lib()
    with pytest.raises(B.ImAttnError) as e:
        B.im_attention_sizes(shape(batch=65536))
    assert e.value.code == -1
    s = shape(seg_len=(64, 64, 64), d_model=128, n_heads=2, dtype="bf16")   # matrix-core path
    sb, wb = B.im_attention_sizes(s)
    ok, odd = C.c_void_p(256), C.c_void_p(264)   # never dereferenced: validation fails first
    rc = L.im_attention_fwd(C.byref(s), odd, ok, ok, ok, ok, None, None, None, None, None, None, ok, ok, ok, wb, None)
    assert rc == -1 and b"16-byte aligned" in L.im_last_error()
    rc = L.im_attention_bwd(C.byref(s), ok, ok, ok, ok, ok, None, None, ok, ok, odd, ok, ok, ok, ok, None, None, None, None, ok, wb, None)
    assert rc == -1 and b"16-byte aligned" in L.im_last_error()


def shape(**kw):
    a = dict(batch=2, seg_len=(8, 8, 8), d_model=32, n_heads=4, live_mask=B.IM_IFM_FORWARD, scale=0.35, dtype="fp32")
    a.update(kw)
    return B.make_shape(**a)


@pytest.mark.parametrize("kw,code", [
    (dict(batch=0), -1), (dict(seg_len=()), -1), (dict(seg_len=(8, 0, 8)), -1), (dict(d_model=30), -1),
    (dict(n_heads=0), -1), (dict(live_mask=1 << 9), -1), (dict(scale=float("nan")), -1),
    (dict(d_model=32 * 4, n_heads=4, dtype="fp32"), -2),       # head dim 32 in fp32: no kernel
    (dict(d_model=96, n_heads=4, dtype="bf16"), -2),           # head dim 24 in bf16: no kernel
])
def test_invalid_shapes_are_rejected(kw, code):
    s = shape(**kw)
    with pytest.raises(B.ImAttnError) as e:
        B.im_attention_sizes(s)
    assert e.value.code == code and str(e.value)


def test_bad_dtype_code():
    s = shape()
    s.dtype = 7
    with pytest.raises(B.ImAttnError) as e:
        B.im_attention_sizes(s)
    assert e.value.code == -1


def test_null_pointers_and_small_workspace_fail_before_any_launch():
    L = B.lib()
    s = shape()
    sb, wb = B.im_attention_sizes(s)
    assert sb > 0 and wb >= sb
    one = C.c_void_p(256)   # never dereferenced: validation fails first
    rc = L.im_attention_fwd(C.byref(s), None, one, one, one, one, None, None, None, None, None, None, one, one, one, wb, None)
    assert rc == -1 and b"NULL" in L.im_last_error()
    rc = L.im_attention_fwd(C.byref(s), one, one, one, one, one, None, None, None, None, None, None, one, None, one, 16, None)
    assert rc == -3 and b"workspace" in L.im_last_error()
    rc = L.im_attention_bwd(C.byref(s), one, one, one, one, one, None, None, None, one, one, one, one, one, one, None, None, None, None, one, wb, None)
    assert rc == -1
    rc = L.im_attention_bwd(C.byref(s), one, one, one, one, one, None, None, one, one, one, one, one, one, one, None, None, None, None, one, 8, None)
    assert rc == -3
    rc = L.gsit_layer_fwd(C.byref(s), 64, one, None, one, one, one, one, one, None, None, None, None, one, one, one, None, one, None,
                          1e-5, None, None, one, one, 1 << 30, None)
    assert rc == -1
    rc = L.gsit_layer_fwd(C.byref(s), 0, *([one] * 17), 1e-5, None, None, one, one, 1 << 30, None)
    assert rc == -1


def test_model_entry_rejects_bad_arguments_on_the_host():
    L = B.lib()
    s = shape()
    one = C.c_void_p(256)
    lay = (B.GsitLayerParams * 1)()
    m = B.GsitModel()
    m.n_layers_inter = m.n_layers_intra = 1
    m.d_ff_inter, m.d_ff_intra, m.n_heads_intra, m.n_out = 64, 128, 4, 3
    m.scale_intra, m.ln_eps = 0.25, 1e-5
    m.mask_fwd, m.mask_bwd, m.mask_intra = B.IM_IFM_FORWARD, B.IM_IFM_BACKWARD, B.IM_IEM
    m.fwd_layers = m.bwd_layers = m.intra_layers = lay
    m.wf = 256
    n = C.c_size_t(0)
    assert L.gsit_model_sizes(C.byref(s), C.byref(m), C.byref(n)) == 0 and n.value > 0
    assert L.gsit_model_fwd(C.byref(s), C.byref(m), one, None, None, one, one, 16, None) == -3
    assert L.gsit_model_fwd(C.byref(s), C.byref(m), None, None, None, one, one, n.value, None) == -1
    m.n_heads_intra = 5                       # does not divide 2d = 64
    assert L.gsit_model_sizes(C.byref(s), C.byref(m), C.byref(n)) == -1 and b"n_heads_intra" in L.im_last_error()
    m.n_heads_intra, m.n_layers_intra = 4, 0
    assert L.gsit_model_sizes(C.byref(s), C.byref(m), C.byref(n)) == -1
    m.n_layers_intra, m.mask_intra = 1, 1 << 9   # bit outside the 3 x 3 pattern
    assert L.gsit_model_sizes(C.byref(s), C.byref(m), C.byref(n)) == -1


@pytest.mark.parametrize("seg", [(50, 375, 500), (50, 500, 500), (39, 400, 55), (30, 230, 480), (8, 8, 8), (512, 2048, 2048)])
@pytest.mark.parametrize("name", sorted(oracle.NAMED_PATTERNS))
@pytest.mark.parametrize("tile", [64, 128])
def test_schedule_covers_exactly_the_live_blocks(seg, name, tile):
    """Sec. 6 / App. B: with Decomposition the pairs visited are sum over live (i,j) of T_i T_j -- no more
    (Delta C = O(0) against MulT), and no item names a masked block."""
    lm = oracle.NAMED_PATTERNS[name]
    s = shape(seg_len=seg, live_mask=lm)
    items, pairs = B.im_schedule_build(s, tile)
    assert pairs == oracle.live_pair_count(seg, lm, 1)
    covered = {}
    for it in items:
        assert 0 < it.q_rows <= tile and it.q_start % tile == 0 and it.q_start + it.q_rows <= seg[it.q_seg]
        js = [it.key_seg[k] for k in range(it.n_key_seg)]
        assert js and all((lm >> (it.q_seg * 3 + j)) & 1 for j in js)
        assert js == [j for j in range(3) if (lm >> (it.q_seg * 3 + j)) & 1]
        assert it.pairs == it.q_rows * sum(seg[j] for j in js)
        covered.setdefault(it.q_seg, []).append((it.q_start, it.q_rows))
    for i in range(3):
        if (lm >> (3 * i)) & 7:
            rows = sorted(covered[i])
            assert rows[0][0] == 0 and sum(r for _, r in rows) == seg[i]
        else:
            assert i not in covered
    # heaviest segments first
    per_row = [it.pairs // it.q_rows for it in items]
    assert per_row == sorted(per_row, reverse=True)
