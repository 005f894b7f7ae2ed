"""The entry points allocate nothing, record no memsets and launch on the caller's stream only, so a
forward + backward can be captured into a HIP graph.  Every replay must reproduce the eager result bit
for bit, with eager work and synchronisations between the replays."""
import pytest
import torch

import oracle
from paper_2505_01068_amd import synth
from tests.gpu_util import Problem

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)


@pytest.mark.parametrize("dtype,seg,d,H", [("fp32", (37, 130, 75), 40, 8), ("bf16", (70, 300, 200), 128, 2),
                                           ("bf16", (50, 200, 130), 64, 8)])
def test_forward_backward_graph_replay(dtype, seg, d, H):
    say(f"[case] graph capture fwd+bwd {dtype} seg={seg} d={d} H={H}")
    g = synth.attention_inputs(2, seg, d, H, dtype, "valid_len", seed=601, bias=True)
    p = Problem(g, oracle.IM_IFM_FORWARD)
    y_ref = p.fwd().clone()
    gr_ref = {k: v.clone() for k, v in p.bwd().items() if v is not None}
    torch.cuda.synchronize()

    # static output buffers for the captured calls
    y = torch.empty_like(y_ref)
    out = {k: torch.empty_like(v) for k, v in gr_ref.items()}
    t = p.t
    from paper_2505_01068_amd import binding as B

    def run():
        B.im_attention_fwd(p.shape, t["x"], t["wq"], t["wk"], t["wv"], t["wo"], t["bq"], t["bk"], t["bv"], t["bo"],
                           t["valid_len"], t["key_pad"], y=y, saved=p.saved, workspace=p.ws)
        B.im_attention_bwd(p.shape, t["x"], t["wq"], t["wk"], t["wv"], t["wo"], p.saved, t["dy"], out["dx"],
                           out["dwq"], out["dwk"], out["dwv"], out["dwo"], out["dbq"], out["dbk"], out["dbv"],
                           out["dbo"], t["valid_len"], t["key_pad"], workspace=p.ws)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run()                                   # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        run()
    for rep in range(3):
        y.fill_(float("nan"))                   # eager work between the replays
        for v in out.values():
            v.fill_(float("nan"))
        p.ws.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y, y_ref), f"replay {rep}: y"
        for k, v in out.items():
            assert torch.equal(v, gr_ref[k]), f"replay {rep}: {k}"
