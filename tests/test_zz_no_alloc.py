"""The allocation-free forward (im_attention_fwd_noalloc) against im_attention_fwd with a caller
workspace: same inputs, same output (the parity bar of the forward, and in fact bitwise), on two calls
in a row of which the second is smaller -- the built-in scratch buffer then still holds the first
call's tensors -- for the row-per-lane (fp32) and the matrix-core (bf16) paths.  Collected last."""
import ctypes as C

import numpy as np
import pytest
import torch

import oracle
from paper_2505_01068_amd import binding as B, synth
from tests.gpu_util import Problem, TOL, assert_close, rel_err


def say(msg):
    print(msg, flush=True)


def _noalloc(p):
    t = p.t
    y = torch.full_like(t["x"], float("nan"))
    B.im_attention_fwd_noalloc(p.shape, t["x"], t["wq"], t["wk"], t["wv"], t["wo"], t["bq"], t["bk"], t["bv"], t["bo"],
                               t["valid_len"], t["key_pad"], y=y)
    return y


@pytest.mark.gpu
@pytest.mark.parametrize("dtype,d,H,segs", [
    ("fp32", 40, 8, [(50, 300, 170), (20, 90, 70)]),
    ("bf16", 128, 2, [(70, 300, 129), (33, 64, 9)]),
    ("bf16", 64, 8, [(50, 260, 131), (8, 70, 40)]),
])
def test_noalloc_forward_matches_workspace_forward_twice(dtype, d, H, segs):
    B.im_noalloc_init()
    for call, seg in enumerate(segs):      # the second call is the smaller one
        say(f"[case] noalloc {dtype} d={d} H={H} seg={seg} call={call}")
        g = synth.attention_inputs(3 - call, seg, d, H, dtype, "valid_len", seed=70 + call, bias=True, with_dy=False)
        p = Problem(g, oracle.IM_IFM_FORWARD if call == 0 else oracle.NAMED_PATTERNS["self_only"])
        y_ws = p.fwd(save=False)
        y_na = _noalloc(p)
        torch.cuda.synchronize()
        assert torch.equal(y_na, y_ws), f"differs from the workspace forward: {rel_err(y_na, y_ws.float().cpu().numpy()):.3e}"
        assert_close(y_na, p.oracle_fwd(), TOL[dtype], f"noalloc {dtype} call {call} vs oracle")


def test_noalloc_rejects_shapes_beyond_the_builtin_buffer_on_the_host():
    L = B.lib()
    one = C.c_void_p(256)   # never dereferenced: the size check comes first
    s = B.make_shape(8, (512, 2048, 2048), 512, 8, B.IM_IFM_FORWARD, 0.125, "bf16")
    _, wb = B.im_attention_sizes(s)
    assert wb > B.IM_NOALLOC_MAX_BYTES
    rc = L.im_attention_fwd_noalloc(C.byref(s), one, one, one, one, one, None, None, None, None, None, None, one, None)
    assert rc == B.IM_ERR_WORKSPACE and b"IM_NOALLOC_MAX_BYTES" in L.im_last_error()
    rc = L.im_attention_fwd_noalloc(C.byref(s), None, one, one, one, one, None, None, None, None, None, None, one, None)
    assert rc == B.IM_ERR_INVALID
