"""The full training step at reduced size: pull -> dense tower -> push (Algorithm 1's three
per-mini-batch calls).  The tower's outputs are compared with its oracle at bf16 tolerance; the sparse
path is compared tightly with the table oracle fed the very gradient the GPU tower produced."""
import numpy as np
import pytest

from oracle import ctr_oracle as O
from oracle import mlp_oracle as M
from paper_2201_05500_amd import workloads as WL
from tests.parity_util import assert_close, compare_tables, pooled_tolerance
from tests.test_gpu_mlp import close_enough, close_rows

pytestmark = pytest.mark.gpu


def test_pull_tower_push_chain():
    import torch
    from paper_2201_05500_amd.binding import CTR_OK, CtrTable
    from paper_2201_05500_amd.binding_mlp import CtrMlp
    w = WL.scaled(WL.WORKLOADS["large"], capacity_rows=1 << 15, zipf_universe=20000, batch=64, slots=12, dim=16)
    in_dim = w.slots * w.dim
    hidden = [64, 32, 16]
    gt = CtrTable(w.capacity_rows, w.dim, init_seed=2, init_std=0.05)
    ot = O.OracleTable(w.capacity_rows, w.dim, init_seed=2, init_std=0.05)
    gm = CtrMlp(in_dim, hidden, init_seed=6)
    om = M.MlpOracle(in_dim, hidden, init_seed=6)
    rng = np.random.default_rng(1)
    for step in range(3):
        bn = WL.as_numpy(WL.make_batch(w, step, with_grad=False))
        keys = torch.from_numpy(bn["keys"].view(np.int64)).cuda()
        offs = torch.from_numpy(bn["offsets"].view(np.int32)).cuda()
        labels = (rng.random(w.batch) < 0.05).astype(np.float32)
        st, gb, pooled16, pooled = gt.pull_pool_bf16(0, keys, offs, want_f32=True)
        assert st == CTR_OK and gt.last_status() == CTR_OK
        assert torch.equal(pooled16, pooled.to(torch.bfloat16))
        ost, opooled = ot.pull_pool(0, bn["keys"], bn["offsets"])
        assert ost == 0
        _, orows, oinv = ot.batch_export(bn["keys"].size)
        assert_close(pooled.cpu().numpy(), opooled, "pooled step %d" % step,
                     pooled_tolerance(ot.table_export(0)["x"], orows, oinv, bn["offsets"]))
        x = pooled16.view(w.batch, in_dim)                     # [B, S*D]: slots concatenated per sample
        st, loss, gp = gm.step(0, x, torch.from_numpy(labels).cuda())
        assert st == CTR_OK
        oloss, ogp = om.step(0, pooled.cpu().numpy().reshape(w.batch, in_dim), labels)   # same input as the GPU tower
        assert abs(float(loss.cpu()[0]) - float(oloss)) <= 1e-4 * max(1.0, float(oloss))
        close_rows(gp.cpu().numpy(), ogp, "grad of pooled step %d" % step, in_dim)
        grad = gp.view(w.n_segments, w.dim)
        assert gt.push_adam(0, gb, grad) == CTR_OK
        assert ot.push_adam(0, grad.cpu().numpy()) == 0        # the oracle gets the GPU tower's gradient
        compare_tables(gt, ot, what="table after step %d" % step)
    close_enough(gm.export()["params"], om.params[0], "tower parameters", rtol=1e-3, norm_tol=1e-3)


def test_pull_tower_push_chain_in_bf16():
    """The same chain with both hand-overs in bf16: pooled embeddings out of the pull, the gradient of the
    pooled embeddings out of the tower and into ctr_push_adam_bf16.  The sparse oracle is fed the GPU tower's
    bf16 gradient widened to fp32 (exact), so the table bar stays the tight one."""
    import torch
    from paper_2201_05500_amd.binding import CTR_OK, CtrTable
    from paper_2201_05500_amd.binding_mlp import CtrMlp
    w = WL.scaled(WL.WORKLOADS["large"], capacity_rows=1 << 15, zipf_universe=20000, batch=64, slots=12, dim=16)
    in_dim = w.slots * w.dim
    hidden = [64, 32, 16]
    gt = CtrTable(w.capacity_rows, w.dim, init_seed=2, init_std=0.05)
    ot = O.OracleTable(w.capacity_rows, w.dim, init_seed=2, init_std=0.05)
    gm = CtrMlp(in_dim, hidden, init_seed=6)
    om = M.MlpOracle(in_dim, hidden, init_seed=6)
    rng = np.random.default_rng(1)
    g16 = torch.empty((w.batch, in_dim), dtype=torch.bfloat16, device="cuda")
    for step in range(3):
        bn = WL.as_numpy(WL.make_batch(w, step, with_grad=False))
        keys = torch.from_numpy(bn["keys"].view(np.int64)).cuda()
        offs = torch.from_numpy(bn["offsets"].view(np.int32)).cuda()
        labels = (rng.random(w.batch) < 0.05).astype(np.float32)
        st, gb, pooled16, pooled = gt.pull_pool_bf16(0, keys, offs, want_f32=True)
        assert st == CTR_OK and gt.last_status() == CTR_OK
        ost, _ = ot.pull_pool(0, bn["keys"], bn["offsets"])
        assert ost == 0
        st, loss, gp = gm.step(0, pooled16.view(w.batch, in_dim), torch.from_numpy(labels).cuda(), grad_pooled=g16)
        assert st == CTR_OK and gp.dtype == torch.bfloat16
        oloss, ogp = om.step(0, pooled.cpu().numpy().reshape(w.batch, in_dim), labels, grad_bf16=True)
        assert abs(float(loss.cpu()[0]) - float(oloss)) <= 1e-4 * max(1.0, float(oloss))
        close_rows(gp.to(torch.float32).cpu().numpy(), ogp, "bf16 grad of pooled step %d" % step, in_dim)
        grad = gp.view(w.n_segments, w.dim)
        assert gt.push_adam(0, gb, grad) == CTR_OK
        assert ot.push_adam(0, grad.to(torch.float32).cpu().numpy()) == 0
        compare_tables(gt, ot, what="table after step %d" % step)
    close_enough(gm.export()["params"], om.params[0], "tower parameters", rtol=1e-3, norm_tol=1e-3)
