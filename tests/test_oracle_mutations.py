"""The pins must bite: plant one plausible slip at a time into a private copy of the
oracle's source (on the CPU, never in the GPU path) and check that a pin fails."""
import importlib.util
import os
import sys
import types

import numpy as np
import pytest

import oracle
from paper_2505_01068_amd import synth
from tests import test_oracle_attention as ta
from tests import test_oracle_backward as tb

SRC = os.path.join(os.path.dirname(oracle.__file__), "im_attention.py")

MUTATIONS = [
    ("dropped scale in scores", "s = scale * (q[b, :, c] @ k[b, :, c].T) + m", "s = (q[b, :, c] @ k[b, :, c].T) + m"),
    ("transposed weight", "q = x @ _f64(wq)", "q = x @ _f64(wq).T"),
    ("k and v weights swapped", "k = x @ _f64(wk)\n    v = x @ _f64(wv)", "k = x @ _f64(wv)\n    v = x @ _f64(wk)"),
    ("query/key role of the block index swapped", "(i * n_seg + j)) & 1 for j in range(n_seg)]\n                       for i",
     "(j * n_seg + i)) & 1 for j in range(n_seg)]\n                       for i"),
    ("padding applied to queries instead of keys", "live & ~np.asarray(invalid_b, dtype=bool)[None, :]",
     "live & ~np.asarray(invalid_b, dtype=bool)[:, None]"),
    ("dropped softmax-Jacobian term", "ds = pb * (dp - np.sum(pb * dp, axis=-1, keepdims=True))", "ds = pb * dp"),
    ("dropped scale in dK", "dk[b, :, c] = scale * (ds.T @ q[b, :, c])", "dk[b, :, c] = (ds.T @ q[b, :, c])"),
    ("dV not transposed", "dv[b, :, c] = pb.T @ d_o[b, :, c]", "dv[b, :, c] = pb @ d_o[b, :, c]"),
    ("missing dK term of dx", "dx=dq @ wq.T + dk @ wk.T + dv @ wv.T", "dx=dq @ wq.T + dv @ wv.T"),
    ("wrong sign of the mask", "np.where(live, 0.0, -np.inf)", "np.where(live, -np.inf, 0.0)"),
    ("valid_len off by one", "pos[None, :] >= vl[:, seg]", "pos[None, :] > vl[:, seg]"),
]


def _mutant(old, new):
    src = open(SRC).read()
    assert src.count(old) == 1, old
    mod = types.ModuleType("oracle_mutant")
    mod.__file__ = SRC
    exec(compile(src.replace(old, new), SRC, "exec"), mod.__dict__)
    return mod


def _pins(mod, monkeypatch):
    """Run a representative subset of the pins against `mod` in place of the oracle."""
    for n in ("forward", "backward", "additive_mask", "key_invalid", "mult_blocks_forward", "live_pair_count"):
        monkeypatch.setattr(oracle, n, getattr(mod, n))
    ta.test_brute_force("ifm_forward", "valid_len")
    ta.test_brute_force("self_only", "key_pad")
    ta.test_patterns_match_paper(os.path.join(os.path.dirname(__file__), "golden"))
    ta.test_live_pair_count_matches_complexity_appendix()
    tb.test_finite_differences("ifm_forward", "valid_len")
    tb.test_against_library_autograd("ifm_backward", "key_pad")


def test_unmutated_source_passes(monkeypatch):
    src = open(SRC).read()
    mod = types.ModuleType("oracle_copy")
    exec(compile(src, SRC, "exec"), mod.__dict__)
    _pins(mod, monkeypatch)


@pytest.mark.parametrize("what,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_pins_catch(what, old, new, monkeypatch):
    mod = _mutant(old, new)
    with pytest.raises((AssertionError, ValueError, FloatingPointError, IndexError)):
        _pins(mod, monkeypatch)
