"""GPU parity of gsit_layer_fwd (one pre-LayerNorm encoder layer) and of the 4-layer encoder stack."""
import numpy as np
import pytest
import torch

import oracle
from paper_2505_01068_amd import binding as B, synth
from tests.gpu_util import assert_close, to_dev, TOL

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)


def run_layers(g, layers, lm, dtype, d_ff, in_place=False):
    x = g["x"]
    shape = B.make_shape(x.shape[0], g["seg_len"], x.shape[2], g["n_heads"], lm, g["scale"], dtype)
    ws = torch.empty(B.gsit_layer_sizes(shape, d_ff), dtype=torch.uint8, device="cuda")
    h = to_dev(x, dtype)
    vl, kp = to_dev(g.get("valid_len"), dtype), to_dev(g.get("key_pad"), dtype)
    for p in layers:
        pd = {k: to_dev(v, dtype) for k, v in p.items()}
        h = B.gsit_layer_fwd(shape, d_ff, h, pd, valid_len=vl, key_pad=kp, y=h if in_place else None, workspace=ws)
    torch.cuda.synchronize()
    return h


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("name", ["ifm_forward", "ifm_backward", "iem", "self_only"])
@pytest.mark.parametrize("bias", [True, False])
def test_single_layer(dtype, name, bias):
    say(f"[case] layer dtype={dtype} pattern={name} bias={bias}")
    d, H, d_ff, seg = 64, 8, 256, (37, 201, 130)
    g = synth.attention_inputs(3, seg, d, H, dtype, "valid_len", seed=301, with_dy=False)
    p = synth.layer_params(d, d_ff, 301, 0, dtype=dtype, bias=bias)
    lm = oracle.NAMED_PATTERNS[name]
    y = run_layers(g, [p], lm, dtype, d_ff)
    ref = oracle.gsit_layer_forward(g["x"], p, seg, lm, H, g["scale"], valid_len=g["valid_len"])
    assert_close(y, ref, TOL[dtype], f"layer/{dtype}/{name}")


def test_layer_odd_widths_fp32():
    say("[case] layer fp32 d=40 d_ff=100")
    d, H, d_ff, seg = 40, 8, 100, (20, 70, 33)
    g = synth.attention_inputs(2, seg, d, H, "fp32", "key_pad", seed=302, with_dy=False)
    p = synth.layer_params(d, d_ff, 302, 0, dtype="fp32")
    y = run_layers(g, [p], oracle.IM_IFM_FORWARD, "fp32", d_ff)
    ref = oracle.gsit_layer_forward(g["x"], p, seg, oracle.IM_IFM_FORWARD, H, g["scale"], key_pad=g["key_pad"])
    assert_close(y, ref, TOL["fp32"], "layer odd widths")


@pytest.mark.parametrize("d_ff", [200, 64, 320])
def test_layer_bf16_width_64_hidden_widths(d_ff):
    # d = 64: the LayerNorms run inside the GEMMs; a hidden width that is a multiple of 64 takes the fused
    # layer tail (one chunk, five chunks), any other the separate MLP GEMMs with the fused LayerNorm
    say(f"[case] layer bf16 d=64 d_ff={d_ff}")
    d, H, seg = 64, 8, (33, 140, 97)
    g = synth.attention_inputs(2, seg, d, H, "bf16", "key_pad", seed=306, with_dy=False)
    p = synth.layer_params(d, d_ff, 306, 0, dtype="bf16")
    y = run_layers(g, [p], oracle.IM_IEM, "bf16", d_ff)
    ref = oracle.gsit_layer_forward(g["x"], p, seg, oracle.IM_IEM, H, g["scale"], key_pad=g["key_pad"])
    assert_close(y, ref, TOL["bf16"], f"layer d=64 d_ff={d_ff}")


@pytest.mark.parametrize("d_ff", [512, 192, 200])
def test_layer_bf16_width_128(d_ff):
    # d = 128 (head dim 16): hidden widths that are multiples of 64 take the fused layer tail (two 64-deep
    # chunks of the output projection, 8 resp. 3 hidden chunks), 200 the separate kernels
    say(f"[case] layer bf16 d=128 d_ff={d_ff}")
    d, H, seg = 128, 8, (33, 140, 97)
    g = synth.attention_inputs(2, seg, d, H, "bf16", "valid_len", seed=308, with_dy=False)
    p = synth.layer_params(d, d_ff, 308, 0, dtype="bf16")
    y = run_layers(g, [p], oracle.IM_IFM_FORWARD, "bf16", d_ff)
    ref = oracle.gsit_layer_forward(g["x"], p, seg, oracle.IM_IFM_FORWARD, H, g["scale"], valid_len=g["valid_len"])
    assert_close(y, ref, TOL["bf16"], f"layer d=128 d_ff={d_ff}")


def test_layer_bf16_width_64_in_place_and_ragged_rows():
    # 2 * 93 = 186 rows: the last 64-row tile of the fused tail holds 58 rows; y written over x
    say("[case] layer bf16 d=64 in place, ragged last tile")
    d, H, d_ff, seg = 64, 8, 128, (20, 40, 33)
    g = synth.attention_inputs(2, seg, d, H, "bf16", "valid_len", seed=307, with_dy=False)
    p = synth.layer_params(d, d_ff, 307, 0, dtype="bf16", bias=False)
    y = run_layers(g, [p], oracle.IM_IFM_BACKWARD, "bf16", d_ff, in_place=True)
    ref = oracle.gsit_layer_forward(g["x"], p, seg, oracle.IM_IFM_BACKWARD, H, g["scale"], valid_len=g["valid_len"])
    assert_close(y, ref, TOL["bf16"], "layer d=64 in place")


def test_layer_identity_when_output_weights_vanish():
    say("[case] layer identity")
    d, H, d_ff, seg = 64, 8, 256, (20, 70, 33)
    g = synth.attention_inputs(2, seg, d, H, "bf16", "none", seed=303, with_dy=False)
    p = synth.layer_params(d, d_ff, 303, 0, dtype="bf16")
    for n in ("wo", "bo", "w2", "b2"):
        p[n] = np.zeros_like(p[n])
    y = run_layers(g, [p], oracle.IM_IFM_FORWARD, "bf16", d_ff)
    assert torch.equal(y.float().cpu(), torch.from_numpy(g["x"]))


@pytest.mark.parametrize("name,padding", [("ifm_forward", "none"), ("iem", "none"), ("ifm_forward", "valid_len"),
                                          ("ifm_backward", "valid_len")])
def test_c4_four_layer_encoder_full_size(name, padding):
    # padding = "valid_len": the variant `bench.py --config c4v` times (per-sample valid lengths as in C3)
    say(f"[case] c4 full size 4 layers pattern={name} padding={padding}")
    w = synth.workload("c4", padding=padding)
    g = synth.attention_inputs(**{**w, "with_dy": False})
    layers = [synth.layer_params(w["d_model"], w["d_ff"], w["seed"], l, dtype="bf16") for l in range(w["n_layers"])]
    lm = oracle.NAMED_PATTERNS[name]
    y = run_layers(g, layers, lm, "bf16", w["d_ff"], in_place=False)
    ref = oracle.gsit_encoder_forward(g["x"], layers, g["seg_len"], lm, g["n_heads"], g["scale"], valid_len=g.get("valid_len"))
    e = assert_close(y, ref, TOL["bf16"], f"c4/{name}/{padding}")
    say(f"    y={e:.1e}")
    y2 = run_layers(g, layers, lm, "bf16", w["d_ff"], in_place=True)     # y aliasing x
    assert torch.equal(y, y2)
