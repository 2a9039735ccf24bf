"""The synthetic workloads have the shapes and statistics their recipe states (CPU only)."""
import numpy as np
import torch

from oracle import fp_formats as ff
from oracle import moe_layer as om
from workloads import CONFIGS, make_inputs, make_expert_weights


def _bits(x):
    return x.view(torch.int16).numpy().view(np.uint16)


def test_config_table_matches_the_five_workloads():
    shapes = [(c.T, c.d, c.E, c.k, c.F) for c in CONFIGS]
    assert shapes == [(64, 128, 8, 2, 256), (256, 4096, 64, 6, 1408), (4096, 5120, 128, 8, 1536),
                      (4096, 5120, 128, 8, 1536), (32768, 7168, 256, 8, 2048)]
    for c in CONFIGS:
        assert c.d % 128 == 0 and c.F % 128 == 0 and c.k <= c.E


def test_generation_is_seeded_and_expertwise_reproducible():
    a = make_inputs(CONFIGS[0])
    b = make_inputs(CONFIGS[0])
    for key in ("x", "W_r", "W1q", "W3q", "W2q", "s1", "s3", "s2"):
        assert torch.equal(a[key], b[key]), key
    sub = make_expert_weights(CONFIGS[0], experts=[5, 2])
    assert torch.equal(sub["W2q"][0], a["W2q"][5]) and torch.equal(sub["s1"][1], a["s1"][2])
    c = make_inputs(CONFIGS[0], seed=99)
    assert not torch.equal(a["x"], c["x"])


def test_weight_codes_are_block_quantised_e4m3():
    """Every 128x128 block uses the full e4m3 range and has no NaN code; std matches N(0,1/d)."""
    w = make_expert_weights(CONFIGS[1], experts=[0])
    q = w["W1q"][0].numpy()
    assert not np.any((q & 0x7F) == 0x7F)
    dec = np.abs(ff.e4m3_decode(q)).reshape(11, 128, 32, 128)
    assert np.all(dec.max(axis=(1, 3)) == 448.0)
    deq = ff.e4m3_decode(q) * np.kron(w["s1"][0].numpy().astype(np.float64), np.ones((128, 128)))
    assert abs(deq.std() * np.sqrt(4096) - 1.0) < 0.02


def test_config2_bias_balances_load():
    inp = make_inputs(CONFIGS[2], with_experts=False)
    idx, _, _ = om.route(_bits(inp["x"]), inp["W_r"].numpy(), 8, inp["sel_bias"].numpy())
    load = np.bincount(idx.reshape(-1), minlength=128)
    assert np.abs(load - 256).max() / 256 <= 0.03
    idx0, _, _ = om.route(_bits(inp["x"]), inp["W_r"].numpy(), 8, None)
    assert np.abs(np.bincount(idx0.reshape(-1), minlength=128) - 256).max() / 256 > 0.08


def test_config3_log_is_zipf_with_three_percent_mismatch():
    inp = make_inputs(CONFIGS[3], with_experts=False)
    idx, _, _ = om.route(_bits(inp["x"]), inp["W_r"].numpy(), 8, None)
    log = inp["logged_idx"].numpy()
    same = np.array([set(a) == set(b) for a, b in zip(idx.tolist(), log.tolist())])
    assert 0.02 < 1 - same.mean() < 0.04
    assert np.array_equal(~same, inp["differs"].numpy())
    assert all(len(set(r)) == 8 for r in log.tolist())
    load = np.bincount(log.reshape(-1), minlength=128)
    assert load[0] > 0.9 * 4096 and load[0] > load[1] > load[2] and np.median(load) < 150
    assert np.allclose(inp["logged_w"].numpy().sum(1), 1.0, atol=1e-5)


def test_config4_outliers():
    import dataclasses
    small = dataclasses.replace(CONFIGS[4], T=2048)
    x = make_inputs(small, with_experts=False)["x"].float()
    frac = (x.abs() == 20.0).float().mean().item()
    assert 5e-4 < frac < 2e-3
