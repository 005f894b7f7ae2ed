"""The input generator: determinism, distribution, padding recipe, bf16 grid."""
import numpy as np
import torch

from paper_2505_01068_amd import synth


def test_deterministic_and_stream_separated():
    a = synth.normal(5, 1, (64,))
    np.testing.assert_array_equal(a, synth.normal(5, 1, (64,)))
    assert not np.array_equal(a, synth.normal(5, 2, (64,)))
    assert not np.array_equal(a, synth.normal(6, 1, (64,)))


def test_moments():
    z = synth.normal(1, 1, (400000,)).astype(np.float64)
    assert abs(z.mean()) < 5e-3 and abs(z.std() - 1) < 5e-3
    w = synth.xavier_uniform(1, 2, 40, 40)
    bound = np.sqrt(6 / 80)
    assert np.abs(w).max() <= bound and np.abs(w).max() > 0.95 * bound


def test_bf16_grid_matches_torch_rounding():
    a = synth.normal(3, 1, (4096,)) * 7
    np.testing.assert_array_equal(synth.to_bf16_grid(a), torch.tensor(a).bfloat16().float().numpy())


def test_padding_recipes():
    g = synth.attention_inputs(**synth.workload("c2", batch=4))
    assert g["key_pad"].shape == (4, 150)
    for s in range(3):
        assert np.all(g["key_pad"][:, 50 * s:50 * (s + 1)].sum(1) == 5)
    assert np.all(g["x"][g["key_pad"] == 1] == 0)
    g = synth.attention_inputs(**synth.workload("c3", batch=8))
    vl = g["valid_len"]
    assert vl.shape == (8, 3) and np.all(vl[:, 0] >= 25) and np.all(vl[:, 0] <= 50)
    assert np.all(vl[:, 1] >= 250) and np.all(vl[:, 1] <= 500) and np.all(vl[:, 2] >= 188) and np.all(vl[:, 2] <= 375)
    assert np.all(g["x"][0, vl[0, 0]:50] == 0) and np.all(g["x"][0, 50 + vl[0, 1]:550] == 0)
