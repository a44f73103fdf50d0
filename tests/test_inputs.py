"""Sanity of the seeded input generators (statistical, not parity)."""
import numpy as np
import torch

import fs_inputs


def test_c1_shape_and_coverage():
    cfg = fs_inputs.CONFIGS["c1"]
    b = fs_inputs.make_batch(cfg)
    assert b["n"] == 8192 and b["offsets"][-1] == 8192 and int(b["ids"].max()) < cfg.E
    pl = fs_inputs.make_placement(cfg, b["perms"]).numpy().view(np.uint32)
    tiers = np.bincount(pl >> 30, minlength=3)
    assert tiers.tolist() == [1000, 0, 99000]
    assert np.all((pl & 0x3FFFFFFF)[pl >> 30 == 2] == np.arange(cfg.E)[pl >> 30 == 2] % cfg.U)
    share = (pl[b["ids"].numpy()] >> 30 == 0).mean()
    assert 0.62 < share < 0.75            # analytic H(1000, 1.05) / H(100000, 1.05) = 0.688
    b2 = fs_inputs.make_batch(cfg)
    assert torch.equal(b["ids"], b2["ids"])   # seeded


def test_length_laws():
    for name, lo, hi, mean in (("c2", 1, 256, 128.5), ("c3", 1, 1024, 120.0), ("c4", 1, 2048, 274.8), ("c5", 1, 512, 256.5)):
        cfg = fs_inputs.CONFIGS[name].scaled(B=2048, T=2)
        ln = fs_inputs.make_lengths(cfg).double()
        assert ln.min() >= lo and ln.max() <= hi
        assert abs(ln.mean().item() - mean) / mean < 0.08, (name, ln.mean().item())


def test_three_tier_placement_and_dtype_bits():
    cfg = fs_inputs.CONFIGS["c3"].scaled(E=50_000, B=16, T=2)
    b = fs_inputs.make_batch(cfg)
    pl = fs_inputs.make_placement(cfg, b["perms"]).numpy().view(np.uint32)
    assert np.bincount(pl >> 30, minlength=3).tolist() == [200, 2000, 97800]
    assert (pl & 0x3FFFFFFF)[pl >> 30 == 1].max() < cfg.W
    w = fs_inputs.make_table(cfg, rows=64)
    assert w.dtype == torch.bfloat16 and fs_inputs.as_numpy_bits(w).dtype == np.uint16
    assert abs(w.float().std().item() - 0.1) < 0.01
