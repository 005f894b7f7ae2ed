"""GPU parity, bf16 paths (MFMA kernels at head dim 64; row-per-lane kernels at small head dims)
vs the fp64 oracle evaluated on the same bf16-rounded inputs.  Bar: 2e-2 relative, per tensor."""
import numpy as np
import pytest
import torch

import oracle
from paper_2505_01068_amd import synth
from tests.gpu_util import Problem, assert_close, rel_err, TOL

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)


@pytest.mark.parametrize("name", ["ifm_forward", "ifm_backward", "iem", "self_only", "dense", "structure2_b"])
@pytest.mark.parametrize("padding", ["none", "valid_len", "key_pad"])
def test_mfma_ragged_fwd_bwd(name, padding):
    # head dim 64; segments span several 64-key tiles and 128/256-row query tiles with ragged tails,
    # lengths that are not multiples of 8 (padded transposed layout), biases
    say(f"[case] mfma ragged pattern={name} padding={padding}")
    g = synth.attention_inputs(2, (70, 300, 129), 128, 2, "bf16", padding, seed=201, bias=True)
    errs = Problem(g, oracle.NAMED_PATTERNS[name]).check(what=f"mfma/{name}/{padding}")
    say("    " + " ".join(f"{k}={v:.1e}" for k, v in errs.items()))


@pytest.mark.parametrize("seg,H", [((1, 1, 1), 1), ((64, 128, 256), 1), ((7,), 2), ((33, 90), 1), ((5, 9, 70, 11), 1),
                                   ((257, 3, 64), 2), ((8, 520, 8), 1)])
def test_mfma_shapes_and_segment_counts(seg, H):
    say(f"[case] mfma shape seg={seg} H={H}")
    n = len(seg)
    g = synth.attention_inputs(2, seg, 64 * H, H, "bf16", "valid_len", seed=17, bias=True)
    masks = [(1 << (n * n)) - 1, sum(1 << (i * n + (i + 1) % n) for i in range(n)), sum(1 << (i * n + i) for i in range(n))]
    for lm in masks:
        Problem(g, lm).check(what=f"mfma seg={seg} lm={lm:#x}")


def test_mfma_wide_model_weight_gradient_kernel():
    # d = 320 (5 heads), 2048 token rows: the weight gradients take the asynchronous 256 x 256 GEMM
    # kernel with ragged row / column tiles (320 = 256 + 64, 960 = 3 * 256 + 192) and split-K
    say("[case] mfma d=320 R=2048 (large-tile weight-gradient GEMM)")
    g = synth.attention_inputs(2, (300, 420, 304), 320, 5, "bf16", "valid_len", seed=41, bias=True)
    errs = Problem(g, oracle.IM_IFM_BACKWARD).check(what="mfma d=320")
    say("    " + " ".join(f"{k}={v:.1e}" for k, v in errs.items()))


def test_mfma_projection_large_tile_ragged_rows():
    # d = 256, 2 x 1092 = 2184 token rows (a multiple of 8, not of 256): the QKV and output projections
    # take the asynchronous 256 x 256 GEMM kernel with a ragged last row tile (2184 = 8 * 256 + 136) and,
    # for N = 768 / 256, full column tiles; biases go through its staged epilogue
    say("[case] mfma d=256 R=2184 (large-tile projection GEMM, ragged rows)")
    g = synth.attention_inputs(2, (300, 488, 304), 256, 4, "bf16", "valid_len", seed=43, bias=True)
    errs = Problem(g, oracle.IM_IFM_FORWARD).check(what="mfma d=256")
    say("    " + " ".join(f"{k}={v:.1e}" for k, v in errs.items()))


def test_mfma_projection_288_row_tiles_ragged():
    """409 samples x (24 + 32 + 32) rows = 35 992 token rows, d = 320 (5 heads): 256-row tiles would need three rounds
    of the 256 CUs for the QKV projection (141 x 4 tiles), 288-row tiles two (125 x 4) -- the launcher takes the
    twelve-wave 288 x 256 kernel, here with a ragged last row tile (35 992 = 124 x 288 + 280), ragged column tiles
    (960 = 3 x 256 + 192, 320 = 256 + 64), biases, and, in the backward, the data gradients on transposed weights."""
    say("[case] mfma d=320 R=35992 (288-row projection tiles, ragged rows and columns)")
    g = synth.attention_inputs(409, (24, 32, 32), 320, 5, "bf16", "valid_len", seed=47, bias=True)
    errs = Problem(g, oracle.IM_IFM_FORWARD).check(what="mfma d=320 R=35992")
    say("    " + " ".join(f"{k}={v:.1e}" for k, v in errs.items()))


def test_mfma_dead_segments_and_fully_masked_rows():
    say("[case] mfma dead segments / fully masked rows")
    g = synth.attention_inputs(2, (9, 70, 33), 64, 1, "bf16", "none", seed=9, bias=True)
    Problem(g, 1 << 1).check(what="mfma single block")
    g["valid_len"] = np.array([[9, 0, 33], [4, 70, 1]], dtype=np.int32)
    for lm in (oracle.IM_IFM_FORWARD, oracle.IM_IFM_BACKWARD, oracle.NAMED_PATTERNS["self_only"], 0):
        Problem(g, lm).check(what=f"mfma zero-valid lm={lm:#x}")


def test_mfma_bitwise_reproducible_and_inference_path():
    say("[case] mfma determinism / saved=NULL")
    g = synth.attention_inputs(2, (70, 300, 129), 128, 2, "bf16", "valid_len", seed=5)
    p = Problem(g, oracle.IM_IFM_FORWARD)
    y0 = p.fwd().clone()
    g0 = {k: v.clone() for k, v in p.bwd().items() if v is not None}
    y1 = p.fwd().clone()
    g1 = p.bwd()
    y2 = p.fwd(save=False)
    torch.cuda.synchronize()
    assert torch.equal(y0, y1) and torch.equal(y0, y2)
    for k in g0:
        assert torch.equal(g0[k], g1[k]), k


def test_mfma_dead_block_contents_do_not_matter_bitwise():
    say("[case] mfma dead block poison")
    g = synth.attention_inputs(1, (64, 200, 136), 64, 1, "bf16", "none", seed=13)
    y0 = Problem(g, oracle.IM_IFM_FORWARD).fwd()
    g2 = dict(g)
    x2 = g["x"].copy()
    x2[:, 264:] = 3e4                      # audio rows are dead for text queries (t <- v only)
    g2["x"] = x2
    y1 = Problem(g2, oracle.IM_IFM_FORWARD).fwd()
    torch.cuda.synchronize()
    assert torch.equal(y0[:, :64], y1[:, :64])


@pytest.mark.parametrize("name", ["ifm_forward", "iem"])
def test_subhead_bf16_small_heads_fwd_bwd(name):
    # the encoder-layer shape: d = 64, 8 heads of dimension 8, bf16 storage: matrix-core kernels in
    # sub-head mode, forward and backward
    say(f"[case] sub-head bf16 fwd+bwd pattern={name}")
    g = synth.attention_inputs(4, (50, 500, 375), 64, 8, "bf16", "valid_len", seed=23, bias=True)
    errs = Problem(g, oracle.NAMED_PATTERNS[name]).check(what=f"subhead-bf16/{name}")
    say("    " + " ".join(f"{k}={v:.1e}" for k, v in errs.items()))


@pytest.mark.parametrize("d,H", [(128, 8), (128, 16), (192, 12)])
@pytest.mark.parametrize("name,padding", [("self_only", "key_pad"), ("ifm_backward", "valid_len"), ("dense", "none")])
def test_subhead_bf16_other_widths_fwd_bwd(d, H, name, padding):
    # head dims 16 / 8 with two and three 64-column groups; multi-live-block rows; all padding modes
    say(f"[case] sub-head bf16 fwd+bwd d={d} H={H} pattern={name} padding={padding}")
    g = synth.attention_inputs(2, (37, 201, 130), d, H, "bf16", padding, seed=31, bias=True)
    Problem(g, oracle.NAMED_PATTERNS[name]).check(what=f"subhead-bf16/{d}/{H}/{name}")


@pytest.mark.parametrize("d,H", [(48, 6), (40, 8), (96, 6)])
def test_rowlane_bf16_widths_off_the_matrix_cores(d, H):
    # bf16 storage with d % 64 != 0 (head dims 8, 5, 16): the row-per-lane kernels
    say(f"[case] rowlane bf16 d={d} H={H}")
    g = synth.attention_inputs(3, (50, 200, 130), d, H, "bf16", "valid_len", seed=24, bias=True)
    errs = Problem(g, oracle.IM_IFM_FORWARD).check(what=f"rowlane-bf16/{d}")
    say("    " + " ".join(f"{k}={v:.1e}" for k, v in errs.items()))


# ---- the scaled-up benchmark shape at full size, in the launch configuration bench.py times ----
_c5_inputs = {}


@pytest.fixture(scope="module", params=["ifm_forward", "ifm_backward", "iem"])
def c5_full(request):
    """One forward + backward of the whole C5 batch on the GPU under the mask `request.param`, and the dense
    oracle on every batch element (elements are independent in y and dx; a few seconds of CPU each), with its
    weight-gradient contributions summed.  Returns the per-element errors and the weight-gradient pairs; the
    tests below only assert on them, so neither depends on the other having run."""
    name = request.param
    lm = oracle.NAMED_PATTERNS[name]
    if "g" not in _c5_inputs:
        _c5_inputs["g"] = synth.attention_inputs(**synth.workload("c5"))
    g = _c5_inputs["g"]
    say(f"[case] c5 full size, mask={name}: GPU forward + backward")
    p = Problem(g, lm)
    y = p.fwd()
    grads = p.bwd()
    torch.cuda.synchronize()
    y = y.float().cpu().numpy()
    grads = {k: v.float().cpu().numpy() for k, v in grads.items() if v is not None}
    del p
    torch.cuda.empty_cache()
    acc, rows = {}, []
    for b in range(g["x"].shape[0]):
        sl = slice(b, b + 1)
        y_ref, cache = oracle.forward(g["x"][sl], g["wq"], g["wk"], g["wv"], g["wo"], g["seg_len"], lm, g["n_heads"],
                                      g["scale"], return_cache=True)
        ref = oracle.backward(cache, g["dy"][sl])
        rows.append((b, rel_err(y[sl], y_ref), rel_err(grads["dx"][sl], ref["dx"])))
        for n in ("dwq", "dwk", "dwv", "dwo"):
            acc[n] = acc.get(n, 0) + ref[n]
        say(f"    mask={name} batch element {b}: y={rows[-1][1]:.1e} dx={rows[-1][2]:.1e}")
    return {"name": name, "rows": rows, "dw": {n: (grads[n], acc[n]) for n in acc}}


def test_c5_full_size_outputs_and_input_gradients(c5_full):
    for b, e_y, e_dx in c5_full["rows"]:
        assert e_y <= TOL["bf16"], f"c5/{c5_full['name']}[{b}] y: relative error {e_y:.3e}"
        assert e_dx <= TOL["bf16"], f"c5/{c5_full['name']}[{b}] dx: relative error {e_dx:.3e}"
    assert len(c5_full["rows"]) == 8


def test_c5_full_size_weight_gradients(c5_full):
    assert sorted(c5_full["dw"]) == ["dwk", "dwo", "dwq", "dwv"]
    for n, (gpu, ref) in c5_full["dw"].items():
        e = assert_close(gpu, ref, TOL["bf16"], f"c5/{c5_full['name']} {n}")
        say(f"    mask={c5_full['name']} {n}={e:.1e}")


def test_mfma_zero_scale_and_large_scores():
    """scale = 0 gives uniform attention over valid keys (no NaN from -inf * 0); large, growing scores
    exercise the lazily updated softmax reference (tile maxima far above the running one)."""
    say("[case] mfma scale=0 / growing scores")
    g = synth.attention_inputs(2, (70, 300, 129), 64, 1, "bf16", "valid_len", seed=31, bias=False)
    g0 = dict(g, scale=0.0)
    Problem(g0, oracle.IM_IFM_FORWARD).check(what="mfma scale=0")
    g1 = dict(g)
    x = g["x"].copy()
    ramp = np.linspace(0.3, 2.2, x.shape[1], dtype=np.float32)[None, :, None]
    g1["x"] = synth.to_bf16_grid(x * ramp)       # later keys have larger scores: row maxima keep growing
    g1["scale"] = 0.35                           # exponent range well beyond the 2^8 rescale threshold
    # forward only: with softmax this peaked the bf16 rounding of Q and K alone moves the gradients by
    # more than the bar (conditioning of the problem, not of the kernel)
    for lm in (oracle.IM_IFM_FORWARD, oracle.IM_DENSE):
        Problem(g1, lm).check(backward=False, what=f"mfma growing scores lm={lm:#x}")


@pytest.mark.parametrize("name", [n for n in sorted(oracle.NAMED_PATTERNS) if n.startswith(("structure", "self_only"))])
def test_mfma_pattern_variants_fwd_bwd(name):
    # Structures 1-3 and Self-Only (Sec. "Ablation Study", App. "Graph Structures") on the
    # matrix-core path: the tile ring runs through several live key segments per query row
    say(f"[case] mfma pattern variant {name} fwd+bwd")
    g = synth.attention_inputs(2, (70, 200, 130), 128, 2, "bf16", "valid_len", seed=20250512, bias=True)
    Problem(g, oracle.NAMED_PATTERNS[name]).check(what=f"mfma-variant/{name}")


@pytest.mark.parametrize("d,H", [(64, 8), (128, 8), (128, 16), (192, 12)])
@pytest.mark.parametrize("name", ["ifm_forward", "iem", "self_only", "dense"])
@pytest.mark.parametrize("padding", ["none", "valid_len", "key_pad"])
def test_subhead_inference_forward(d, H, name, padding):
    # inference (nothing saved) at head dims 8 / 16: the matrix-core forward in its sub-head mode,
    # several heads per 64-column group, ragged segments and tails
    say(f"[case] sub-head inference d={d} H={H} pattern={name} padding={padding}")
    g = synth.attention_inputs(2, (37, 201, 130), d, H, "bf16", padding, seed=29, bias=True, with_dy=False)
    p = Problem(g, oracle.NAMED_PATTERNS[name])
    y = p.fwd(save=False)
    torch.cuda.synchronize()
    assert_close(y, p.oracle_fwd(), TOL["bf16"], f"subhead/{d}/{H}/{name}/{padding}")
    y_train = p.fwd(save=True)       # same kernels with the tensors for the backward saved: identical output
    torch.cuda.synchronize()
    assert torch.equal(y, y_train)
