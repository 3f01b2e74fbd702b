"""The seeded generator: deterministic, block-addressable, and with the stated distributions."""
import numpy as np
import torch

import osscar_inputs as inp


def test_blocks_are_addressable_and_deterministic():
    cfg = inp.scaled(inp.CONFIGS["cfg3"], p=96, m=16, n=300)
    full = inp.gen_X(cfg)
    assert full.dtype == torch.bfloat16 and full.shape == (300, 96)
    part = inp.gen_X(cfg, row0=100, nrows=50, cols=torch.tensor([5, 17, 95]))
    assert torch.equal(part, full[100:150][:, [5, 17, 95]])
    assert torch.equal(inp.gen_X(cfg), full)
    assert not torch.equal(inp.gen_X(cfg.replace(seed=cfg.seed + 1)), full)
    mixed = inp.gen_X(cfg.replace(mix=0.5))
    pm = inp.gen_X(cfg.replace(mix=0.5), row0=7, nrows=9, cols=torch.tensor([95, 0]))
    assert torch.equal(pm, mixed[7:16][:, [95, 0]])


def test_standard_normal_moments():
    z = inp.std_normal(123, 9, torch.arange(400), torch.arange(500)).double().numpy()
    assert abs(z.mean()) < 0.01 and abs(z.std() - 1) < 0.01
    assert abs(np.mean(z ** 4) - 3) < 0.1


def test_ar1_covariance():
    cfg = inp.CONFIGS["cfg1"].replace(n=20000)
    X = inp.gen_X(cfg).double().numpy()
    C = X.T @ X / X.shape[0]
    for lag in (0, 1, 2, 4):
        want = 0.6 ** lag
        got = np.mean([C[i, i + lag] for i in range(10, 50)])
        assert abs(got - want) < 0.03


def test_recipes_shapes_and_structure():
    c2 = inp.scaled(inp.CONFIGS["cfg2"], p=8, m=4, n=64)
    X2 = inp.gen_X(c2)
    assert X2.dtype == torch.float32 and X2.shape == (64, 72) and (X2 >= 0).all()
    s2 = inp.column_scales(c2)
    assert np.all(s2.reshape(8, 9) == s2.reshape(8, 9)[:, :1])      # one scale per channel
    c4 = inp.scaled(inp.CONFIGS["cfg4"], p=4, m=4, n=64)
    X4 = inp.gen_X(c4)
    assert X4.shape == (64, 256) and (X4 < 0).any()
    c3 = inp.CONFIGS["cfg3"]
    s3 = inp.column_scales(c3)
    assert np.sum(s3 > 20 * np.exp(-3)) >= 8 and s3.shape == (8192,)
    W = inp.gen_W(inp.scaled(c3, p=512, m=256, n=8))
    assert W.dtype == torch.bfloat16 and abs(W.float().std().item() - 0.02) < 0.002
