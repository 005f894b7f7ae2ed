"""GPU parity with packed rows (no padding rows in memory; per-sample segment offsets): HIP kernels
through the C ABI vs the fp64 oracle on the padded problem with the same lengths."""
import numpy as np
import pytest
import torch

import oracle
from paper_2505_01068_amd import binding as B
from paper_2505_01068_amd import synth
from tests.gpu_util import PackedProblem, Problem

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)


def lengths_for(batch, seg, seed, lo_frac=0.0):
    """lengths uniform in [lo_frac * T, T] per sample and segment, with the extremes planted: one sample at
    full length, one with a zero-length segment (when lo_frac == 0)."""
    lo = np.array([int(lo_frac * n) for n in seg])
    L = synth.randint(seed, 21, lo[None, :], np.array(seg)[None, :], (batch, len(seg))).astype(np.int32)
    L[0, :] = seg
    if lo_frac == 0.0 and batch > 1:
        L[1, seed % len(seg)] = 0
    return L


@pytest.mark.parametrize("name", ["ifm_forward", "ifm_backward", "iem", "dense", "self_only", "structure1_a"])
def test_packed_fp32_rowlane(name):
    say(f"[case] packed fp32 pattern={name}")
    seg = (37, 201, 130)
    g = synth.attention_inputs(4, seg, 40, 8, "fp32", "none", seed=301, bias=True)
    PackedProblem(g, oracle.NAMED_PATTERNS[name], lengths_for(4, seg, 301)).check(what=f"packed/fp32/{name}")


@pytest.mark.parametrize("name", ["ifm_forward", "iem", "dense"])
def test_packed_bf16_matrix_cores(name):
    # head dim 64; several 128- and 256-row tiles per segment, tiles past a sample's length exit early
    say(f"[case] packed bf16 dh=64 pattern={name}")
    seg = (70, 300, 520)
    g = synth.attention_inputs(3, seg, 128, 2, "bf16", "none", seed=302, bias=True)
    PackedProblem(g, oracle.NAMED_PATTERNS[name], lengths_for(3, seg, 302)).check(what=f"packed/bf16/{name}")


@pytest.mark.parametrize("dtype,d,H", [("fp32", 40, 8), ("bf16", 128, 2), ("bf16", 64, 8)])
def test_packed_with_key_pad(dtype, d, H):
    # key_pad over the packed rows: 10 % of the positions are padding keys on top of the per-sample lengths
    say(f"[case] packed + key_pad {dtype} d={d} H={H}")
    seg = (40, 210, 150)
    g = synth.attention_inputs(3, seg, d, H, dtype, "key_pad", seed=308, bias=True)
    PackedProblem(g, oracle.IM_IFM_BACKWARD, lengths_for(3, seg, 308, lo_frac=0.3)).check(what=f"packed/key_pad/{dtype}")


@pytest.mark.parametrize("dh", [8, 16])
def test_packed_bf16_subhead(dh):
    say(f"[case] packed bf16 sub-head dh={dh}")
    seg = (50, 200, 150)
    g = synth.attention_inputs(3, seg, 64, 64 // dh, "bf16", "none", seed=303, bias=True)
    PackedProblem(g, oracle.IM_IFM_FORWARD, lengths_for(3, seg, 303)).check(what=f"packed/subhead{dh}")


def test_packed_dead_segment_rows_are_zero():
    # a query segment without live keys: its packed output rows are exactly the output bias, its dQ rows zero
    say("[case] packed, segment without live block")
    seg = (20, 90, 40)
    lm = oracle.IM_IFM_FORWARD & ~(1 << (0 * 3 + 1))   # text queries lose their only key segment
    for dtype, d, H in (("fp32", 40, 8), ("bf16", 128, 2)):
        g = synth.attention_inputs(3, seg, d, H, dtype, "none", seed=304, bias=True)
        PackedProblem(g, lm, lengths_for(3, seg, 304)).check(what=f"packed/dead/{dtype}")


def test_packed_equals_padded_at_full_length():
    # all lengths at their maxima: packed rows are the padded rows; results must agree bit for bit
    say("[case] packed == padded at full lengths")
    seg = (33, 140, 97)
    for dtype, d, H in (("fp32", 40, 8), ("bf16", 128, 2)):
        g = synth.attention_inputs(2, seg, d, H, dtype, "none", seed=305, bias=True)
        full = np.tile(np.array(seg, dtype=np.int32), (2, 1))
        pp, pd = PackedProblem(g, oracle.IM_IFM_FORWARD, full), Problem(g, oracle.IM_IFM_FORWARD)
        yp, yd = pp.fwd(), pd.fwd()
        gp, gd = pp.bwd(), pd.bwd()
        torch.cuda.synchronize()
        assert torch.equal(yp.reshape(-1), yd.reshape(-1))
        for n in gp:
            if gp[n] is not None:
                assert torch.equal(gp[n].reshape(-1), gd[n].reshape(-1)), n


def test_packed_dataset_lengths_c3_shape():
    # the benchmark's packed workload: C3 shape, lengths with the dataset's mean and variance
    say("[case] packed C3 with dataset length statistics")
    st = synth.MOSI_LENGTH_STATS
    w = synth.workload("c3", padding="none")
    g = synth.attention_inputs(**w)
    L = synth.dataset_lengths(w["batch"], st["max"], st["mean"], st["var"], seed=w["seed"])
    errs = PackedProblem(g, oracle.IM_IFM_FORWARD, L).check(what="packed/c3")
    say("    errors: " + " ".join(f"{k}={v:.1e}" for k, v in errs.items()))


def test_packed_host_errors():
    seg = (8, 8, 8)
    g = synth.attention_inputs(2, seg, 32, 4, "fp32", "none", seed=306)
    L = np.array([[8, 3, 5], [1, 8, 2]], dtype=np.int32)
    p = PackedProblem(g, oracle.IM_IFM_FORWARD, L)
    vl = torch.from_numpy(L).cuda()
    with pytest.raises(B.ImAttnError) as e:   # lengths come from cu_rows, not valid_len
        B.im_attention_fwd(p.shape, p.t["x"], p.t["wq"], p.t["wk"], p.t["wv"], p.t["wo"], valid_len=vl,
                           saved=p.saved, workspace=p.ws)
    assert e.value.code == B.IM_ERR_INVALID
    bad = B.make_shape(2, seg, 32, 4, oracle.IM_IFM_FORWARD, g["scale"], "fp32", cu_rows=p.cu, total_rows=2 * 24 + 1)
    with pytest.raises(B.ImAttnError) as e:
        B.im_attention_sizes(bad)
    assert e.value.code == B.IM_ERR_INVALID


@pytest.mark.parametrize("dtype,d,H,d_ff", [("fp32", 40, 8, 100), ("bf16", 64, 8, 256), ("bf16", 128, 2, 256)])
def test_packed_layer_forward_backward(dtype, d, H, d_ff):
    # one encoder layer (training forward, inference forward, backward) on packed rows
    from tests.gpu_util import assert_close, to_dev, TOL
    say(f"[case] packed layer fwd+bwd {dtype} d={d} H={H}")
    seg, lm = (50, 200, 130), oracle.IM_IFM_FORWARD
    g = synth.attention_inputs(3, seg, d, H, dtype, "none", seed=307)
    p = synth.layer_params(d, d_ff, 307, 0, dtype=dtype)
    L = lengths_for(3, seg, 307, lo_frac=0.2)
    cu = synth.row_offsets(L)
    cu_d = torch.from_numpy(cu).cuda()
    shape = B.make_shape(3, seg, d, H, lm, g["scale"], dtype, cu_rows=cu_d, total_rows=int(cu[-1]))
    pack = lambda a: synth.pack_rows(a, L, seg)
    sb, wb = B.gsit_layer_train_sizes(shape, d_ff)
    saved = torch.empty(sb, dtype=torch.uint8, device="cuda")
    ws = torch.empty(wb, dtype=torch.uint8, device="cuda")
    xd, dyd = to_dev(pack(g["x"]), dtype), to_dev(pack(g["dy"]), dtype)
    pd = {k: to_dev(v, dtype) for k, v in p.items()}
    y = B.gsit_layer_fwd_train(shape, d_ff, xd, pd, saved, workspace=ws)
    y_inf = B.gsit_layer_fwd(shape, d_ff, xd, pd,
                             workspace=torch.empty(B.gsit_layer_sizes(shape, d_ff), dtype=torch.uint8, device="cuda"))
    grads = {k: torch.full(v.shape, float("nan"), dtype=torch.float32, device="cuda") for k, v in p.items() if v is not None}
    dx = B.gsit_layer_bwd(shape, d_ff, xd, pd, saved, dyd, grads, workspace=ws)
    torch.cuda.synchronize()

    kw = dict(seg_len=seg, live_mask=lm, n_heads=H, scale=g["scale"], valid_len=L, key_pad=None)
    tol = TOL[dtype]
    y_ref = pack(oracle.gsit_layer_forward(g["x"], p, **kw))
    assert_close(y, y_ref, tol, "packed layer y")
    assert_close(y_inf, y_ref, tol, "packed layer y (inference)")
    dy0 = synth.unpack_rows(pack(g["dy"]), L, seg)   # zero beyond the lengths
    ref = oracle.gsit_layer_backward(g["x"], p, dy0, **kw)
    ulp = 2.0 ** -8 if dtype == "bf16" else 2.0 ** -23
    floor = ulp * max(float(np.max(np.abs(v))) for v in ref.values())
    assert_close(dx, pack(ref["dx"]), tol, "packed layer dx")
    for n, v in grads.items():
        r = ref["d" + n]
        scale = max(float(np.max(np.abs(r))), floor)
        if n == "bk":
            scale = max(scale, float(np.max(np.abs(ref["dwk"]))))
        assert_close(v, r, tol, "packed layer d" + n, scale)


def test_packed_model_call_is_refused():
    from tests.test_gpu_model import dev_model
    seg = (8, 8, 8)
    cu = torch.zeros(2 * 3 + 1, dtype=torch.int32, device="cuda")
    shape = B.make_shape(2, seg, 32, 4, 0, 0.35, "fp32", cu_rows=cu, total_rows=10)
    m = synth.model_params(32, 64, 128, 1, 1, 3, 1, seed=1, dtype="fp32")
    model = B.make_model(dev_model(m, "fp32"), 64, 128, 4, 0.25)
    with pytest.raises(B.ImAttnError) as e:
        B.gsit_model_sizes(shape, model)
    assert e.value.code == B.IM_ERR_UNSUPPORTED
