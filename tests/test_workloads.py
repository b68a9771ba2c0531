"""Host-side checks of the seeded input generators (no method arithmetic here)."""
import numpy as np
import pytest
import torch

from paper_2304_03946_amd import workloads as W


def test_bf16_rounding_matches_torch():
    rng = np.random.default_rng(0)
    a = (rng.standard_normal(100000) * np.exp(rng.uniform(-20, 20, 100000))).astype(np.float32)
    bits = W.f32_to_bf16_bits(a)
    ref = torch.from_numpy(a).to(torch.bfloat16)
    assert np.array_equal(bits.view(np.int16), ref.view(torch.int16).numpy())
    assert np.array_equal(W.bf16_bits_to_f32(bits), ref.float().numpy())


def test_inputs_are_seeded_and_shaped():
    cfg = W.scaled(W.CONFIGS["gpt_m"], N=64, d=32, f=64, E=8, V=12)
    a, b = W.make_layer_inputs(cfg), W.make_layer_inputs(cfg)
    assert np.array_equal(a.x.bits, b.x.bits) and np.array_equal(a.w1.bits, b.w1.bits)
    assert a.x.shape == (64, 32) and a.wg.shape == (32, 8) and a.w1.shape == (8, 32, 64) and a.w2.shape == (8, 64, 32)
    assert a.dy.shape == (64, 32)
    assert np.all(W.decode(a.x)[:, -1] == 1.0)                      # the bias feature
    c = W.make_layer_inputs(cfg, seed=a.seed + 1)
    assert not np.array_equal(a.x.bits, c.x.bits)


def test_tiny_config_is_fp32_identity_placement():
    cfg = W.CONFIGS["tiny"]
    inp = W.make_layer_inputs(cfg)
    assert inp.x.dtype == np.float32 and inp.dy is None
    off, ids = W.config_placement(cfg)
    assert off.tolist() == [0, 1, 2, 3, 4] and ids.tolist() == [0, 1, 2, 3]
    assert abs(float(np.std(inp.w1)) - 0.02) < 1e-3


@pytest.mark.parametrize("name", ["bert", "gpt_m", "swin", "gpt_xl"])
def test_config_placements_are_valid(name):
    cfg = W.CONFIGS[name]
    for shuffle in (None, 5):
        off, ids = W.config_placement(cfg, shuffle_seed=shuffle)
        assert off[0] == 0 and off[-1] == cfg.V and np.all(np.diff(off) >= 1)
        assert np.max(np.diff(off)) <= cfg.max_rep
        assert sorted(ids.tolist()) == list(range(cfg.V))


def test_bert_placement_replicates_two_hottest():
    off, ids = W.config_placement(W.CONFIGS["bert"])
    assert ids[off[0]:off[1]].tolist() == [0, 16] and ids[off[1]:off[2]].tolist() == [1, 17]
    assert np.all(np.diff(off)[2:] == 1)


def test_placement_from_loads_follows_capacity_rule():
    # loads 100, 10, 10: spare slots go to the expert with the largest load per replica
    off, ids = W.placement_from_loads([100, 10, 10], 6, 8)
    assert np.diff(off).tolist() == [4, 1, 1] and ids.tolist() == [0, 3, 4, 5, 1, 2]
    off, ids = W.placement_from_loads([100, 60, 10], 5, 2)
    assert np.diff(off).tolist() == [2, 2, 1]


def test_gpt_xl_skew_resembles_paper_load_trace():
    # Observation 2 of the paper: 10 of 64 experts take about 3/4 of the tokens.
    cfg = W.CONFIGS["gpt_xl"]
    idx = W.sample_topk_idx(W.scaled(cfg, N=8192), seed=1)
    cnt = np.sort(np.bincount(idx.reshape(-1), minlength=cfg.E))[::-1]
    share = cnt[:10].sum() / cnt.sum()
    assert 0.6 < share < 0.9
    assert all(len(set(r)) == cfg.k for r in idx[:200].tolist())


def test_drift_rotates_hot_set():
    cfg = W.CONFIGS["gpt_xl"]
    b0, b1 = W.expert_bias(cfg, 1, 0), W.expert_bias(cfg, 1, 1)
    assert np.argmax(b0) != np.argmax(b1) and np.allclose(np.sort(b0), np.sort(b1))
