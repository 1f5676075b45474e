"""The synthetic-input recipe: shapes, determinism, distribution."""
import numpy as np

from paper_2201_05500_amd import workloads as WL


def test_tiny_batch_shape_and_determinism():
    w = WL.WORKLOADS["tiny"]
    a = WL.as_numpy(WL.make_batch(w, 0))
    b = WL.as_numpy(WL.make_batch(w, 0))
    c = WL.as_numpy(WL.make_batch(w, 1))
    G = w.batch * w.slots
    assert a["offsets"].shape == (G + 1,) and a["offsets"][0] == 0
    counts = np.diff(a["offsets"].astype(np.int64))
    assert counts.min() >= 1 and counts.max() <= 8 and abs(counts.mean() - 4.5) < 0.1
    assert a["keys"].shape == (a["offsets"][-1],) and a["keys"].dtype == np.uint64
    assert a["grad"].shape == (G, w.dim) and abs(a["grad"].std() - 1) < 0.02
    for f in a:
        assert np.array_equal(a[f], b[f])
    assert not np.array_equal(a["keys"][:100], c["keys"][:100])
    assert not np.any(a["keys"] == np.uint64(2 ** 64 - 1))


def test_key_mix_is_a_bijection_on_the_id_width():
    import torch
    for bits in (16, 40, 48):
        r = torch.arange(0, 1 << 16, dtype=torch.int64)
        k = WL._mix_rank_to_key(r, bits).numpy()
        assert k.min() >= 0 and k.max() < (1 << bits)
        assert np.unique(k).size == r.numel()
    k64 = WL._mix_rank_to_key(torch.arange(0, 1 << 16, dtype=torch.int64), 64).numpy()
    assert np.unique(k64).size == 1 << 16


def test_zipf_is_heavy_tailed_and_bounded():
    import torch
    g = torch.Generator().manual_seed(1)
    U = 1 << 20
    r = WL.zipf_ranks(400000, 1.0, U, g, "cpu").numpy()
    assert r.min() >= 1 and r.max() <= U
    # P(rank = 1) = log(2)/log(U) for the continuous bounded law with s = 1
    assert abs((r == 1).mean() - np.log(2) / np.log(U)) < 0.004
    r = WL.zipf_ranks(400000, 1.1, 10 ** 6, g, "cpu").numpy()
    assert r.min() >= 1 and r.max() <= 10 ** 6 and (r == 1).mean() > 0.05


def test_poisson_configs():
    w = WL.scaled(WL.WORKLOADS["mid"], batch=64)
    c = np.diff(WL.as_numpy(WL.make_batch(w, 0, with_grad=False))["offsets"].astype(np.int64))
    assert c.min() >= 1 and abs(c.mean() - 3.05) < 0.1
    w = WL.scaled(WL.WORKLOADS["large"], batch=32)
    b = WL.as_numpy(WL.make_batch(w, 0, with_grad=False))
    c = np.diff(b["offsets"].astype(np.int64))
    assert c.min() == 0 and abs(c.mean() - 4.0) < 0.1
    assert b["keys"].max() < np.uint64(1 << 48)
