"""The seeded input generator: reproducible, right shapes and laws."""
import numpy as np
import pytest

import workloads


def test_same_seed_same_bits_and_bf16_representable():
    a = workloads.make(64, 32, 100, "bf16", ignore=("iid", 0.3), seed=5)
    b = workloads.make(64, 32, 100, "bf16", ignore=("iid", 0.3), seed=5)
    c = workloads.make(64, 32, 100, "bf16", ignore=("iid", 0.3), seed=6)
    assert np.array_equal(a.X, b.X) and np.array_equal(a.W, b.W)
    assert np.array_equal(a.targets, b.targets)
    assert not np.array_equal(a.X, c.X)
    assert not (a.X.view(np.uint32) & 0xFFFF).any()
    bits = workloads.bf16_bits(a.W)
    assert np.array_equal(workloads.bf16_bits_to_f32(bits), a.W)


def test_bf16_rounding_is_nearest_even():
    import torch
    g = np.random.default_rng(0)
    x = g.standard_normal(100000).astype(np.float32)
    x[:4] = np.array([1.00390625, 1.01171875, 3.0e-39, -0.0], dtype=np.float32)
    ref = torch.from_numpy(x.copy()).to(torch.bfloat16).to(torch.float32).numpy()
    got = workloads.round_to_bf16(x.copy())
    assert np.array_equal(got.view(np.uint32), ref.view(np.uint32))


def test_distributions_of_the_small_config():
    w = workloads.make_config(1)
    assert (w.BT, w.H, w.V, w.dtype) == (256, 512, 4096, "f32")
    assert abs(w.X.std() - 1.0) < 0.02 and abs(w.W.std() - 0.02) < 2e-4
    assert w.n_valid == 256 and w.targets.min() >= 0 and w.targets.max() < 4096


@pytest.mark.parametrize("law,frac", [(("iid", 0.3), 0.3), (("pad", 2048, 819), 0.2)])
def test_ignore_laws(law, frac):
    w = workloads.make(16384, 8, 50, "bf16", ignore=law, seed=9)
    ign = (w.targets == workloads.IGNORE_INDEX)
    assert abs(ign.mean() - frac) < 0.08
    if law[0] == "pad":
        for s in range(0, 16384, 2048):
            seq = ign[s:s + 2048]
            n = seq.sum()
            assert n <= 819 and seq[2048 - n:].all() and not seq[:2048 - n].any()


def test_zipf_targets_are_head_heavy():
    w = workloads.make(20000, 8, 128256, "bf16", targets="zipf", seed=3)
    t = w.targets
    assert t.min() >= 0 and t.max() < 128256
    assert (t == 0).mean() > 0.05 and (t < 100).mean() > 0.3 and (t > 10000).mean() > 0.05
