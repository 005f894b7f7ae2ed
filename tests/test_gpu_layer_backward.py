"""GPU parity of gsit_layer_fwd_train / gsit_layer_bwd (one encoder layer, forward that saves and
backward) vs the fp64 layer oracle: dx and the gradient of every parameter."""
import numpy as np
import pytest
import torch

import oracle
from paper_2505_01068_amd import binding as B, synth
from tests.gpu_util import assert_close, grad_scale, to_dev, TOL

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)


def run(g, p, lm, dtype, d_ff):
    x = g["x"]
    shape = B.make_shape(x.shape[0], g["seg_len"], x.shape[2], g["n_heads"], lm, g["scale"], dtype)
    sb, wb = B.gsit_layer_train_sizes(shape, d_ff)
    saved = torch.empty(sb, dtype=torch.uint8, device="cuda")
    ws = torch.empty(wb, dtype=torch.uint8, device="cuda")
    xd, dyd = to_dev(x, dtype), to_dev(g["dy"], dtype)
    pd = {k: to_dev(v, dtype) for k, v in p.items()}
    vl, kp = to_dev(g.get("valid_len"), dtype), to_dev(g.get("key_pad"), dtype)
    y = B.gsit_layer_fwd_train(shape, d_ff, xd, pd, saved, valid_len=vl, key_pad=kp, workspace=ws)
    y_inf = B.gsit_layer_fwd(shape, d_ff, xd, pd, valid_len=vl, key_pad=kp,
                             workspace=torch.empty(B.gsit_layer_sizes(shape, d_ff), dtype=torch.uint8, device="cuda"))
    grads = {k: torch.full(v.shape, float("nan"), dtype=torch.float32, device="cuda") for k, v in p.items() if v is not None}
    dx = B.gsit_layer_bwd(shape, d_ff, xd, pd, saved, dyd, grads, valid_len=vl, key_pad=kp, workspace=ws)
    torch.cuda.synchronize()
    return y, y_inf, dx, grads


def check(g, p, lm, dtype, d_ff, what):
    y, y_inf, dx, grads = run(g, p, lm, dtype, d_ff)
    kw = dict(seg_len=g["seg_len"], live_mask=lm, n_heads=g["n_heads"], scale=g["scale"], valid_len=g.get("valid_len"),
              key_pad=g.get("key_pad"))
    tol = TOL[dtype]
    y_ref = oracle.gsit_layer_forward(g["x"], p, **kw)
    errs = {"y": assert_close(y, y_ref, tol, what + " y"), "y_inf": assert_close(y_inf, y_ref, tol, what + " y (inference)")}
    ref = oracle.gsit_layer_backward(g["x"], p, g["dy"], **kw)
    ulp = 2.0 ** -8 if dtype == "bf16" else 2.0 ** -23
    floor = ulp * max(float(np.max(np.abs(v))) for k, v in ref.items() if k != "attn_dk")
    errs["dx"] = assert_close(dx, ref["dx"], tol, what + " dx")
    dk_sum = np.max(np.sum(np.abs(ref["attn_dk"]), axis=(0, 1)))
    for n, v in grads.items():
        r = ref["d" + n]
        errs["d" + n] = assert_close(v, r, tol, what + " d" + n, grad_scale(n, r, floor, dk_sum))
    return errs


@pytest.mark.parametrize("name", ["ifm_forward", "ifm_backward", "iem", "self_only"])
@pytest.mark.parametrize("padding", ["valid_len", "key_pad"])
def test_layer_backward_fp32(name, padding):
    say(f"[case] layer bwd fp32 pattern={name} padding={padding}")
    d, H, d_ff, seg = 40, 8, 100, (37, 130, 75)
    g = synth.attention_inputs(3, seg, d, H, "fp32", padding, seed=501)
    p = synth.layer_params(d, d_ff, 501, 0, dtype="fp32")
    errs = check(g, p, oracle.NAMED_PATTERNS[name], "fp32", d_ff, f"layer-bwd/fp32/{name}/{padding}")
    say("    " + " ".join(f"{k}={v:.1e}" for k, v in errs.items()))


@pytest.mark.parametrize("d,H,d_ff", [(40, 8, 100), (64, 8, 128)])
def test_layer_tall_fp32(d, H, d_ff):
    """More than 1024 rows in fp32: the layer's narrow GEMMs (output projection and second MLP layer with their
    residuals, the input-gradient products with transposed weights; K = 100 is not a multiple of 8) run on the
    fp32 matrix-instruction kernel."""
    say(f"[case] layer fwd+bwd fp32, tall input, d={d} d_ff={d_ff}")
    seg = (37, 201, 150)
    g = synth.attention_inputs(3, seg, d, H, "fp32", "valid_len", seed=507)
    p = synth.layer_params(d, d_ff, 507, 0, dtype="fp32")
    errs = check(g, p, oracle.IM_IFM_FORWARD, "fp32", d_ff, f"layer-bwd/fp32/tall/d={d}")
    say("    " + " ".join(f"{k}={v:.1e}" for k, v in errs.items()))


@pytest.mark.parametrize("bias", [True, False])
def test_layer_backward_bf16_small_heads(bias):
    say(f"[case] layer bwd bf16 d=64 (sub-head matrix-core attention) bias={bias}")
    d, H, d_ff, seg = 64, 8, 256, (50, 200, 130)
    g = synth.attention_inputs(3, seg, d, H, "bf16", "valid_len", seed=502)
    p = synth.layer_params(d, d_ff, 502, 0, dtype="bf16", bias=bias)
    errs = check(g, p, oracle.IM_IFM_FORWARD, "bf16", d_ff, "layer-bwd/bf16/d64")
    say("    " + " ".join(f"{k}={v:.1e}" for k, v in errs.items()))


def test_layer_backward_bf16_narrow_widths():
    # d = 40 (head dim 5: row-per-lane attention), d_ff = 104: multiples of 8 but not of 64, so the
    # matrix-core GEMMs run with partial k-tiles and the split data gradient stays on the ALU GEMM
    say("[case] layer bwd bf16 d=40 d_ff=104")
    d, H, d_ff, seg = 40, 8, 104, (50, 200, 130)
    g = synth.attention_inputs(3, seg, d, H, "bf16", "key_pad", seed=505)
    p = synth.layer_params(d, d_ff, 505, 0, dtype="bf16")
    errs = check(g, p, oracle.IM_IFM_FORWARD, "bf16", d_ff, "layer-bwd/bf16/d40")
    say("    " + " ".join(f"{k}={v:.1e}" for k, v in errs.items()))


def test_layer_backward_bf16_matrix_core_attention():
    say("[case] layer bwd bf16 d=128, head dim 64 (MFMA attention)")
    d, H, d_ff, seg = 128, 2, 256, (70, 200, 130)
    g = synth.attention_inputs(2, seg, d, H, "bf16", "valid_len", seed=503)
    p = synth.layer_params(d, d_ff, 503, 0, dtype="bf16")
    errs = check(g, p, oracle.IM_IFM_BACKWARD, "bf16", d_ff, "layer-bwd/bf16/d128")
    say("    " + " ".join(f"{k}={v:.1e}" for k, v in errs.items()))


def test_layer_backward_bitwise_reproducible():
    say("[case] layer bwd reproducible")
    d, H, d_ff, seg = 64, 8, 128, (50, 120, 90)
    g = synth.attention_inputs(2, seg, d, H, "bf16", "valid_len", seed=504)
    p = synth.layer_params(d, d_ff, 504, 0, dtype="bf16")
    a = run(g, p, oracle.IM_IFM_FORWARD, "bf16", d_ff)
    b = run(g, p, oracle.IM_IFM_FORWARD, "bf16", d_ff)
    assert torch.equal(a[2], b[2])
    for n in a[3]:
        assert torch.equal(a[3][n], b[3][n]), n


def test_layer_backward_bf16_wide_model_large_tile_epilogues():
    # d = 256, d_ff = 512: the projections and both MLP GEMMs run on the 256 x 256 large-tile kernel, including its
    # GELU and residual epilogues; 1136 rows = 4 row tiles + a ragged one
    say("[case] layer fwd+bwd bf16 d=256 (large-tile GEMM with GELU / residual epilogues)")
    d, H, d_ff, seg = 256, 4, 512, (72, 296, 200)
    g = synth.attention_inputs(2, seg, d, H, "bf16", "valid_len", seed=506)
    p = synth.layer_params(d, d_ff, 506, 0, dtype="bf16")
    errs = check(g, p, oracle.IM_IFM_FORWARD, "bf16", d_ff, "layer-bwd/bf16/d256")
    say("    " + " ".join(f"{k}={v:.1e}" for k, v in errs.items()))


def test_layer_backward_at_the_benchmark_shape():
    """The shape `bench.py --config c4train` times (B = 32, 50/500/375, d = 64, 8 heads, d_ff = 256, bf16), whole
    batch on the GPU in one call; the dense oracle walks the batch four elements at a time (elements are
    independent in y and dx) and its parameter-gradient contributions are summed."""
    say("[case] layer fwd+bwd bf16 at the c4train benchmark shape")
    w = synth.workload("c4")
    g = synth.attention_inputs(**w)
    d, H, d_ff, seg, lm = w["d_model"], w["n_heads"], w["d_ff"], g["seg_len"], oracle.IM_IFM_FORWARD
    p = synth.layer_params(d, d_ff, w["seed"], 0, dtype="bf16")
    y, y_inf, dx, grads = run(g, p, lm, "bf16", d_ff)
    y, y_inf, dx = (t.float().cpu().numpy() for t in (y, y_inf, dx))
    tol, acc, dk_sum = TOL["bf16"], {}, 0.0
    for b0 in range(0, g["x"].shape[0], 4):
        sl = slice(b0, b0 + 4)
        kw = dict(seg_len=seg, live_mask=lm, n_heads=H, scale=g["scale"])
        y_ref = oracle.gsit_layer_forward(g["x"][sl], p, **kw)
        ref = oracle.gsit_layer_backward(g["x"][sl], p, g["dy"][sl], **kw)
        e = (assert_close(y[sl], y_ref, tol, f"c4train[{b0}:] y"), assert_close(y_inf[sl], y_ref, tol, f"c4train[{b0}:] y (inference)"),
             assert_close(dx[sl], ref["dx"], tol, f"c4train[{b0}:] dx"))
        say(f"    elements {b0}..{b0 + 3}: y={e[0]:.1e} y_inf={e[1]:.1e} dx={e[2]:.1e}")
        dk_sum = dk_sum + np.sum(np.abs(ref["attn_dk"]), axis=(0, 1))
        for n in grads:
            acc[n] = acc.get(n, 0) + ref["d" + n]
    floor = 2.0 ** -8 * max(float(np.max(np.abs(v))) for v in acc.values())
    errs = {n: assert_close(v, acc[n], tol, f"c4train d{n}", grad_scale(n, acc[n], floor, np.max(dk_sum))) for n, v in grads.items()}
    say("    " + " ".join(f"d{k}={v:.1e}" for k, v in errs.items()))
