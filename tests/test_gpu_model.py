"""GPU parity of gsit_model_fwd (Sec. 5, Eq. "allmodalinone fusion": two IFM encoders, feature
concatenation, IEM encoder at width 2d, last step of every segment, final linear) vs the fp64 oracle."""
import numpy as np
import pytest
import torch

import oracle
from paper_2505_01068_amd import binding as B, synth
from tests.gpu_util import assert_close, to_dev, TOL

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)


def dev_model(m, dtype):
    conv = lambda layers: [{k: to_dev(v, dtype) for k, v in p.items()} for p in layers]
    return {"fwd_layers": conv(m["fwd_layers"]), "bwd_layers": conv(m["bwd_layers"]), "intra_layers": conv(m["intra_layers"]),
            "wf": to_dev(m["wf"], dtype), "bf": to_dev(m["bf"], dtype)}


def run_model(g, m, dtype, d_ff, d_ff_intra, H_intra, masks=None):
    x = g["x"]
    d = x.shape[2]
    shape = B.make_shape(x.shape[0], g["seg_len"], d, g["n_heads"], 0, g["scale"], dtype)
    scale_intra = 1.0 / np.sqrt(2 * d / H_intra)
    md = dev_model(m, dtype)
    kw = {} if masks is None else dict(mask_fwd=masks[0], mask_bwd=masks[1], mask_intra=masks[2])
    model = B.make_model(md, d_ff, d_ff_intra, H_intra, scale_intra, **kw)
    ws = torch.empty(B.gsit_model_sizes(shape, model), dtype=torch.uint8, device="cuda")
    out = B.gsit_model_fwd(shape, model, to_dev(x, dtype), valid_len=to_dev(g.get("valid_len"), dtype),
                           key_pad=to_dev(g.get("key_pad"), dtype), workspace=ws)
    torch.cuda.synchronize()
    okw = {} if masks is None else dict(mask_fwd=masks[0], mask_bwd=masks[1], mask_intra=masks[2])
    ref = oracle.gsit_model_forward(x, m, g["seg_len"], g["n_heads"], g["scale"], H_intra, scale_intra,
                                    valid_len=g.get("valid_len"), key_pad=g.get("key_pad"), **okw)
    return out, ref


@pytest.mark.parametrize("dtype,d,H,Hi", [("fp32", 40, 8, 8), ("bf16", 64, 8, 8)])
@pytest.mark.parametrize("padding", ["valid_len", "none", "key_pad"])
def test_model_small_heads(dtype, d, H, Hi, padding):
    # row-per-lane path at both widths (head dims 5 / 10 and 8 / 16)
    say(f"[case] model dtype={dtype} d={d} padding={padding}")
    seg, d_ff, L, Li, n_out = (37, 130, 75), 2 * d, 2, 2, 3
    g = synth.attention_inputs(3, seg, d, H, dtype, padding, seed=401, with_dy=False)
    m = synth.model_params(d, d_ff, 2 * d_ff, L, Li, 3, n_out, 401, dtype=dtype)
    out, ref = run_model(g, m, dtype, d_ff, 2 * d_ff, Hi)
    e = assert_close(out, ref, TOL[dtype], f"model/{dtype}/{padding}")
    say(f"    error {e:.2e}")


def test_model_matrix_core_path():
    # head dimension 64 at both widths: d = 128 with 2 heads, 2d = 256 with 4 heads
    say("[case] model bf16 d=128 (MFMA kernels)")
    d, H, Hi, seg, d_ff, n_out = 128, 2, 4, (70, 200, 130), 256, 7
    g = synth.attention_inputs(2, seg, d, H, "bf16", "valid_len", seed=402, with_dy=False)
    m = synth.model_params(d, d_ff, 2 * d_ff, 2, 1, 3, n_out, 402, dtype="bf16")
    out, ref = run_model(g, m, "bf16", d_ff, 2 * d_ff, Hi)
    e = assert_close(out, ref, TOL["bf16"], "model/mfma")
    say(f"    error {e:.2e}")


def test_model_identity_encoders_closed_form():
    # all output-side weights zero: X = f(|| [x_last || x_last]) exactly representable steps
    say("[case] model identity encoders")
    d, H, seg, d_ff = 40, 8, (20, 33, 9), 80
    g = synth.attention_inputs(2, seg, d, H, "fp32", "valid_len", seed=403, with_dy=False)
    m = synth.model_params(d, d_ff, 2 * d_ff, 1, 1, 3, 4, 403, dtype="fp32")
    for layers in (m["fwd_layers"], m["bwd_layers"], m["intra_layers"]):
        for p in layers:
            for n in ("wo", "bo", "w2", "b2"):
                p[n] = np.zeros_like(p[n])
    out, ref = run_model(g, m, "fp32", d_ff, 2 * d_ff, H)
    assert_close(out, ref, TOL["fp32"], "model/identity")


def test_model_other_masks_two_segments():
    # masks are arguments: a two-segment model with cross masks (0 <-> 1) and a dense "intra" mask
    say("[case] model n_seg=2 custom masks")
    d, H, seg, d_ff = 40, 8, (50, 70), 80
    g = synth.attention_inputs(2, seg, d, H, "fp32", "valid_len", seed=404, with_dy=False)
    m = synth.model_params(d, d_ff, 2 * d_ff, 1, 1, 2, 2, 404, dtype="fp32")
    masks = (0b0110, 0b1001, 0b1111)
    out, ref = run_model(g, m, "fp32", d_ff, 2 * d_ff, H, masks)
    assert_close(out, ref, TOL["fp32"], "model/2seg")


@pytest.mark.parametrize("padding", ["none", "valid_len"])
def test_model_at_the_benchmark_shape_and_depth(padding):
    """The configuration `bench.py --config gsit` times: B = 32, 50/500/375, d = 64, 8 heads, 4 + 4 IFM layers and
    4 IEM layers at width 128, bf16 -- twelve layers of bf16 rounding against the 2e-2 bar.  The whole batch runs
    on the GPU in one call; batch elements are independent, so the dense oracle evaluates a slice of four (the
    first two and the last two) and those outputs are compared."""
    say(f"[case] model bf16 at the gsit benchmark shape, 4+4+4 layers, padding={padding}")
    w = synth.workload("c4", padding=padding)
    g = synth.attention_inputs(**{**w, "with_dy": False})
    d, H, d_ff, L, seg = w["d_model"], w["n_heads"], w["d_ff"], w["n_layers"], g["seg_len"]
    m = synth.model_params(d, d_ff, 2 * d_ff, L, L, len(seg), 1, w["seed"], dtype="bf16")
    shape = B.make_shape(g["x"].shape[0], seg, d, H, 0, g["scale"], "bf16")
    scale_intra = 1.0 / np.sqrt(2 * d / H)
    model = B.make_model(dev_model(m, "bf16"), d_ff, 2 * d_ff, H, scale_intra)
    ws = torch.empty(B.gsit_model_sizes(shape, model), dtype=torch.uint8, device="cuda")
    out = B.gsit_model_fwd(shape, model, to_dev(g["x"], "bf16"), valid_len=to_dev(g.get("valid_len"), "bf16"), workspace=ws)
    torch.cuda.synchronize()
    pick = [0, 1, g["x"].shape[0] - 2, g["x"].shape[0] - 1]
    vl = None if g.get("valid_len") is None else g["valid_len"][pick]
    ref = oracle.gsit_model_forward(g["x"][pick], m, seg, H, g["scale"], H, scale_intra, valid_len=vl)
    e = assert_close(out[pick], ref, TOL["bf16"], f"model at benchmark shape/{padding}")
    say(f"    error {e:.2e} on batch elements {pick}")
