"""Prediction path on the GPU: lookup-only pooling (no insert) and the tower's forward pass, against the oracles."""
import numpy as np
import pytest

from oracle import ctr_oracle as O
from oracle import mlp_oracle as M
from paper_2201_05500_amd import workloads as WL
from tests.parity_util import assert_close, compare_tables, pooled_tolerance, run_step, to_device

pytestmark = pytest.mark.gpu


def _trained_pair(w, steps=3, **kw):
    from paper_2201_05500_amd.binding import CtrTable
    gt = CtrTable(w.capacity_rows, w.dim, init_seed=8, init_std=0.05, **kw)
    ot = O.OracleTable(w.capacity_rows, w.dim, init_seed=8, init_std=0.05, **kw)
    for s in range(steps):
        bn = WL.as_numpy(WL.make_batch(w, s))
        run_step(gt, ot, to_device(bn), bn, what="training step %d" % s)
    return gt, ot


@pytest.mark.parametrize("dim", [8, 64])
def test_lookup_pool_matches_the_oracle_and_changes_nothing(dim):
    import torch
    from paper_2201_05500_amd import binding as B
    w = WL.scaled(WL.WORKLOADS["large"], capacity_rows=1 << 15, zipf_universe=40000, batch=48, slots=20, dim=dim)
    gt, ot = _trained_pair(w)
    before = gt.table_export(0)
    n_rows = gt.n_rows
    bn = WL.as_numpy(WL.make_batch(w, 50))                       # a later batch: part of its keys were never seen
    bt = to_device(bn)
    st, pooled = gt.lookup_pool(0, bt["keys"], bt["offsets"])
    ost, opooled = ot.lookup_pool(0, bn["keys"], bn["offsets"])
    assert st == B.CTR_OK and ost == O.OK and gt.last_status() == B.CTR_OK
    absent = np.array([ot.lookup(int(k)) < 0 for k in bn["keys"][:2000]])
    assert 0.02 < absent.mean() < 0.9                             # the case is not vacuous
    # tolerance: the parameter bound summed over the rows that are present
    ox = ot.table_export(0)["x"]
    rows = np.array([ot.lookup(int(k)) for k in bn["keys"]])
    per = np.where(rows[:, None] >= 0, 1e-6 + 1e-5 * np.abs(ox[np.maximum(rows, 0)].astype(np.float64)), 0.0)
    c = np.concatenate([np.zeros((1, dim)), np.cumsum(per, axis=0)])
    off = bn["offsets"].astype(np.int64)
    assert_close(pooled.cpu().numpy(), opooled, "lookup pooled", np.maximum(c[off[1:]] - c[off[:-1]], 1e-6))
    st, p16 = gt.lookup_pool(0, bt["keys"], bt["offsets"], bf16=True)
    assert st == B.CTR_OK and torch.equal(p16, pooled.to(torch.bfloat16))
    assert gt.n_rows == n_rows == ot.n_rows
    after = gt.table_export(0)
    for f in ("keys", "x", "m", "v"):
        assert np.array_equal(before[f], after[f]), f
    # training goes on as if nothing had happened
    bn2 = WL.as_numpy(WL.make_batch(w, 3))
    run_step(gt, ot, to_device(bn2), bn2, what="step after lookups")
    compare_tables(gt, ot, what="after lookups")


def test_lookup_errors_are_deferred_like_a_pull():
    import torch
    from paper_2201_05500_amd import binding as B
    w = WL.scaled(WL.WORKLOADS["tiny"], capacity_rows=4096, zipf_universe=3000, batch=16)
    gt, ot = _trained_pair(w, steps=1)
    keys = torch.tensor([5, -1, 7], dtype=torch.int64, device="cuda")         # -1 is the reserved key 2^64 - 1
    offs = torch.tensor([0, 1, 3], dtype=torch.int32, device="cuda")
    st, _ = gt.lookup_pool(0, keys, offs)
    assert st == B.CTR_OK and gt.last_status() == B.CTR_E_BADKEY and gt.last_status() == B.CTR_OK
    bad_offs = torch.tensor([0, 2, 1, 3], dtype=torch.int32, device="cuda")
    st, _ = gt.lookup_pool(0, keys.abs(), bad_offs)
    assert st == B.CTR_OK and gt.last_status() == B.CTR_E_INVAL
    assert gt.lookup_pool(3, keys, offs)[0] == B.CTR_E_INVAL
    st, p = gt.lookup_pool(0, keys[:0], torch.tensor([0, 0], dtype=torch.int32, device="cuda"))
    assert st == B.CTR_OK and not p.any() and gt.last_status() == B.CTR_OK
    # a live batch whose workspace the lookup reuses goes stale; one with another workspace would not
    bt = to_device(WL.as_numpy(WL.make_batch(w, 5)))
    st, h, _ = gt.pull_pool(0, bt["keys"], bt["offsets"])
    assert st == B.CTR_OK
    assert gt.lookup_pool(0, bt["keys"], bt["offsets"])[0] == B.CTR_OK
    assert gt.push_adam(0, h, bt["grad"]) == B.CTR_E_STATE


def test_prediction_chain_lookup_then_forward():
    """lookup (bf16) -> tower forward: logits against the two oracles chained the same way."""
    import torch
    from paper_2201_05500_amd.binding import CTR_OK
    from paper_2201_05500_amd.binding_mlp import CtrMlp
    from tests.test_gpu_mlp import close_rows
    w = WL.scaled(WL.WORKLOADS["large"], capacity_rows=1 << 15, zipf_universe=20000, batch=64, slots=12, dim=16)
    gt, ot = _trained_pair(w, steps=2)
    in_dim = w.slots * w.dim
    gm = CtrMlp(in_dim, [64, 32], init_seed=6)
    om = M.MlpOracle(in_dim, [64, 32], init_seed=6)
    bn = WL.as_numpy(WL.make_batch(w, 9))
    bt = to_device(bn)
    st, p16 = gt.lookup_pool(0, bt["keys"], bt["offsets"], bf16=True)
    assert st == CTR_OK
    st, logits = gm.forward(0, p16.view(w.batch, in_dim))
    assert st == CTR_OK
    # the tower's oracle is fed what the GPU lookup produced (checked above against the table oracle)
    ologits = om.forward(0, p16.float().cpu().numpy().reshape(w.batch, in_dim))
    close_rows(logits.cpu().numpy(), ologits, "prediction logits", 1)
