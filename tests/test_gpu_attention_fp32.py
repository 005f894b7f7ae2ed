"""GPU parity, fp32 path: HIP kernels through the C ABI vs the fp64 oracle, element by element."""
import numpy as np
import pytest
import torch

import oracle
from paper_2505_01068_amd import synth
from tests.gpu_util import Problem, assert_close, TOL

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)


@pytest.mark.parametrize("name", sorted(oracle.NAMED_PATTERNS))
def test_c1_all_patterns_forward(name):
    say(f"[case] c1 fwd pattern={name}")
    g = synth.attention_inputs(**synth.workload("c1"))
    Problem(g, oracle.NAMED_PATTERNS[name]).check(backward=False, what=f"c1/{name}")


@pytest.mark.parametrize("name", ["ifm_forward", "ifm_backward", "iem", "self_only", "dense", "structure1_a"])
@pytest.mark.parametrize("padding", ["none", "valid_len", "key_pad"])
def test_ragged_multi_tile_fwd_bwd(name, padding):
    # several 64-row tiles per segment, ragged tails, LDS chunks of 128 keys with a tail, biases
    say(f"[case] ragged fwd+bwd pattern={name} padding={padding}")
    g = synth.attention_inputs(3, (37, 201, 130), 40, 8, "fp32", padding, seed=101, bias=True)
    Problem(g, oracle.NAMED_PATTERNS[name]).check(what=f"ragged/{name}/{padding}")


@pytest.mark.parametrize("cfg", ["c2", "c3"])
@pytest.mark.parametrize("name", ["ifm_forward", "ifm_backward", "iem"])
def test_full_size_configs(cfg, name):
    say(f"[case] {cfg} full size fwd+bwd pattern={name}")
    g = synth.attention_inputs(**synth.workload(cfg))
    errs = Problem(g, oracle.NAMED_PATTERNS[name]).check(what=f"{cfg}/{name}")
    say(f"    errors: " + " ".join(f"{k}={v:.1e}" for k, v in errs.items()))


def test_very_tall_weight_gradients_fp32():
    """132 000 rows at d = 40 (11 000 batch elements of 12 rows): the weight-gradient kernels take more than 128 rows
    per workgroup (their partial results are capped at 1024 per gradient) and the last workgroup is ragged."""
    say("[case] very tall fp32 weight gradients d=40 H=8 B=11000")
    g = synth.attention_inputs(11000, (3, 5, 4), 40, 8, "fp32", "valid_len", seed=313, bias=True)
    Problem(g, oracle.IM_IFM_FORWARD).check(what="very tall/d=40")


@pytest.mark.parametrize("d,H", [(40, 8), (36, 6), (48, 4), (20, 4), (64, 8), (42, 7), (33, 3)])
def test_tall_projections_ragged_rows(d, H):
    """More than 1024 rows, not a multiple of 32: the fp32 projections of a tall input run on the matrix-instruction
    GEMM (32-row blocks, widths padded to 32 columns, K padded to 8; d = 42 cannot store four columns at a time and
    stays on the ALU GEMM)."""
    say(f"[case] tall fp32 projections d={d} H={H}")
    g = synth.attention_inputs(3, (37, 201, 150), d, H, "fp32", "valid_len", seed=311, bias=True)
    p = Problem(g, oracle.IM_IFM_FORWARD)
    p.check(what=f"tall/d={d}")
    if d != 40:
        return
    # the two weight gradients share a launch when both are asked for; either one alone must give the same bits
    from paper_2505_01068_amd import binding as B
    full, t = p.bwd(), p.t
    f32 = dict(dtype=torch.float32, device="cuda")
    for which in ("dwo", "dwk"):
        out = torch.empty(d, d, **f32)
        args = [out if n == which else None for n in ("dwq", "dwk", "dwv", "dwo")]
        B.im_attention_bwd(p.shape, t["x"], t["wq"], t["wk"], t["wv"], t["wo"], p.saved, t["dy"], None, *args,
                           None, None, None, None, t["valid_len"], t["key_pad"], workspace=p.ws)
        torch.cuda.synchronize()
        assert torch.equal(out, full[which]), which


def test_c2_trailing_padding_through_valid_len():
    say("[case] c2 trailing-5 valid_len variant")
    w = synth.workload("c2", padding="none")
    g = synth.attention_inputs(**w)
    g["valid_len"] = np.full((w["batch"], 3), 45, dtype=np.int32)
    Problem(g, oracle.IM_IFM_FORWARD).check(what="c2/valid45")


@pytest.mark.parametrize("seg,H,d", [((1, 1, 1), 1, 4), ((1, 65, 64), 2, 32), ((64, 128, 192), 4, 32),
                                     ((7,), 2, 16), ((33, 90), 2, 24), ((5, 9, 70, 11), 4, 64), ((129, 3, 64), 3, 48)])
def test_shapes_and_segment_counts(seg, H, d):
    say(f"[case] shape seg={seg} H={H} d={d}")
    n = len(seg)
    g = synth.attention_inputs(2, seg, d, H, "fp32", "valid_len", seed=7, bias=True)
    masks = [(1 << (n * n)) - 1, sum(1 << (i * n + (i + 1) % n) for i in range(n)), sum(1 << (i * n + i) for i in range(n))]
    for lm in masks:
        Problem(g, lm).check(what=f"seg={seg} lm={lm:#x}")


def test_dead_segments_and_fully_masked_rows():
    say("[case] dead segments / fully masked rows")
    g = synth.attention_inputs(2, (9, 70, 33), 16, 2, "fp32", "none", seed=9, bias=True)
    # only block (t <- v) live: v, a queries dead; t, a never keys
    p = Problem(g, 1 << 1)
    p.check(what="single block")
    y = p.fwd()
    torch.cuda.synchronize()
    bo = g["bo"]
    np.testing.assert_allclose(y[:, 9:].cpu().numpy(), np.broadcast_to(bo, (2, 103, 16)), rtol=1e-6, atol=1e-7)
    # a segment with zero valid keys for one sample
    g["valid_len"] = np.array([[9, 0, 33], [4, 70, 1]], dtype=np.int32)
    for lm in (oracle.IM_IFM_FORWARD, oracle.IM_IFM_BACKWARD, oracle.NAMED_PATTERNS["self_only"]):
        Problem(g, lm).check(what=f"zero-valid lm={lm:#x}")
    # nothing live at all
    p = Problem(g, 0)
    p.check(what="empty mask")


def test_dead_block_contents_do_not_matter_bitwise():
    say("[case] dead block poison")
    g = synth.attention_inputs(2, (20, 100, 70), 40, 8, "fp32", "none", seed=13)
    y0 = Problem(g, oracle.IM_IFM_FORWARD).fwd()
    g2 = dict(g)
    x2 = g["x"].copy()
    x2[:, 120:] = 1e4                      # audio rows are dead for text queries (t <- v only)
    g2["x"] = x2
    y1 = Problem(g2, oracle.IM_IFM_FORWARD).fwd()
    torch.cuda.synchronize()
    assert torch.equal(y0[:, :20], y1[:, :20])


def test_bitwise_reproducible():
    say("[case] determinism")
    g = synth.attention_inputs(**synth.workload("c3", batch=4))
    p = Problem(g, oracle.IM_IFM_FORWARD)
    y0 = p.fwd().clone()
    g0 = {k: v.clone() for k, v in p.bwd().items() if v is not None}
    y1 = p.fwd()
    g1 = p.bwd()
    torch.cuda.synchronize()
    assert torch.equal(y0, y1)
    for k in g0:
        assert torch.equal(g0[k], g1[k]), k


def test_inference_without_saved_matches():
    say("[case] saved=NULL inference")
    g = synth.attention_inputs(2, (37, 201, 130), 40, 8, "fp32", "valid_len", seed=3)
    p = Problem(g, oracle.IM_IFM_BACKWARD)
    y0 = p.fwd(save=True).clone()
    y1 = p.fwd(save=False)
    torch.cuda.synchronize()
    assert torch.equal(y0, y1)


# Maximum sequence lengths (text, vision, audio) of the other three datasets in the paper's dataset
# table (Appendix E): CMU-MOSEI, CH-SIMS, MIntRec.  Synthetic N(0,1) features of those shapes with
# per-sample valid lengths stand in for the datasets.
DATASET_SHAPES = {"mosei": (50, 500, 500), "sims": (39, 400, 55), "mintrec": (30, 230, 480)}


@pytest.mark.parametrize("ds", sorted(DATASET_SHAPES))
@pytest.mark.parametrize("name", ["ifm_forward", "ifm_backward", "iem"])
def test_other_dataset_shapes(ds, name):
    say(f"[case] dataset shape {ds} pattern={name}")
    g = synth.attention_inputs(4, DATASET_SHAPES[ds], 40, 8, "fp32", "valid_len", seed=20250510, bias=False)
    Problem(g, oracle.NAMED_PATTERNS[name]).check(what=f"{ds}/{name}")


@pytest.mark.parametrize("name", [n for n in sorted(oracle.NAMED_PATTERNS) if n.startswith(("structure", "self_only"))])
def test_pattern_variants_fwd_bwd(name):
    # Structures 1-3 and Self-Only (Sec. "Ablation Study", App. "Graph Structures"; Self-Only is also the multi-live-block case of the information-disorder discussion): rows
    # with several live blocks share ONE softmax across segments (Sec. "Information Disorder")
    say(f"[case] pattern variant {name} fwd+bwd")
    g = synth.attention_inputs(2, (50, 200, 150), 40, 8, "fp32", "valid_len", seed=20250511, bias=True)
    Problem(g, oracle.NAMED_PATTERNS[name]).check(what=f"variant/{name}")


@pytest.mark.parametrize("dtype,d,H", [("fp32", 40, 8), ("bf16", 128, 2)])
def test_optional_gradient_outputs(dtype, d, H):
    # every gradient output may be NULL; the ones that are asked for do not depend on which others are
    say(f"[case] optional gradient outputs {dtype}")
    from paper_2505_01068_amd import binding as B
    g = synth.attention_inputs(2, (33, 140, 97), d, H, dtype, "valid_len", seed=77, bias=True)
    p = Problem(g, oracle.IM_IFM_FORWARD)
    p.fwd()
    full = p.bwd()
    t = p.t
    f32 = dict(dtype=torch.float32, device="cuda")
    dx = torch.empty_like(t["x"])
    dwq, dwo = torch.empty(d, d, **f32), torch.empty(d, d, **f32)
    dbq, dbv = torch.empty(d, **f32), torch.empty(d, **f32)
    B.im_attention_bwd(p.shape, t["x"], t["wq"], t["wk"], t["wv"], t["wo"], p.saved, t["dy"], dx, dwq, None, None, dwo,
                       dbq, None, dbv, None, t["valid_len"], t["key_pad"], workspace=p.ws)
    torch.cuda.synchronize()
    for name, v in (("dx", dx), ("dwq", dwq), ("dwo", dwo), ("dbq", dbq), ("dbv", dbv)):
        assert torch.equal(v, full[name]), name
    B.im_attention_bwd(p.shape, t["x"], t["wq"], t["wk"], t["wv"], t["wo"], p.saved, t["dy"], None, None, None, None, None,
                       None, None, None, None, t["valid_len"], t["key_pad"], workspace=p.ws)   # nothing asked for
    torch.cuda.synchronize()
