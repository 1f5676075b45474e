"""The hot calls only enqueue kernels (no allocation, copy, memset or synchronisation), so a pull + push pair
can be recorded into a HIP graph and replayed: each replay is one more training step on the recorded batch.
Checked against the same steps issued eagerly on a second table, after every replay, with eager work and
synchronisations in between."""
import numpy as np
import pytest

from paper_2201_05500_amd import workloads as WL
from tests.parity_util import to_device

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("variant", ["single", "kstep", "bias_corrected", "ordered_spans", "ordered_spans_own_launch"])
def test_captured_pull_push_replays_like_eager_steps(variant):
    # bias_corrected: the step count and its correction factors live on the device, so every replay is a new step t
    # ordered_spans*: the graphed table's push computes and follows an execution order of its spans (the launches
    # a large gradient array adds), the eager one keeps the list order: same bits
    kstep = variant == "kstep"
    import torch
    from paper_2201_05500_amd.binding import CTR_OK, CTR_STEP_LOCAL, CTR_STEP_MERGE_PENDING, CtrTable
    w = WL.scaled(WL.WORKLOADS["mid"], capacity_rows=1 << 15, zipf_universe=1 << 15, batch=256)
    bt = to_device(WL.as_numpy(WL.make_batch(w, 0)))
    other = to_device(WL.as_numpy(WL.make_batch(w, 1)))
    kw = dict(init_seed=7, n_replicas=2 if kstep else 1, kstep=kstep, bias_correction=variant == "bias_corrected")
    eager, graphed = CtrTable(w.capacity_rows, w.dim, **kw), CtrTable(w.capacity_rows, w.dim, **kw)
    if variant.startswith("ordered_spans"):
        assert graphed.set_push_order(8, 1 if variant.endswith("own_launch") else 0, 0) == CTR_OK
        assert eager.set_push_order(0, 0, 0) == CTR_OK
    mode = CTR_STEP_MERGE_PENDING if kstep else CTR_STEP_LOCAL
    G = w.n_segments
    pooled_e = torch.empty((G, w.dim), dtype=torch.float32, device="cuda:0")
    pooled_g = torch.empty_like(pooled_e)

    def step(t, b, pooled):
        st, h, _ = t.pull_pool(0, b["keys"], b["offsets"], pooled)
        assert st == CTR_OK
        assert t.push_adam(0, h, b["grad"], mode) == CTR_OK
        if kstep:
            assert t.kstep_merge() == CTR_OK

    for t, p in ((eager, pooled_e), (graphed, pooled_g)):     # one eager step first: workspaces exist, rows inserted
        step(t, bt, p)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            step(graphed, bt, pooled_g)
    torch.cuda.synchronize()
    # the capture itself ran nothing: the graphed table is one step behind until the first replay
    for replay in range(3):
        g.replay()
        torch.cuda.synchronize()
        step(eager, bt, pooled_e)
        torch.cuda.synchronize()
        assert graphed.last_status() == CTR_OK and eager.last_status() == CTR_OK
        assert torch.equal(pooled_g, pooled_e), replay
        a, b = graphed.table_export(0), eager.table_export(0)
        for f in ("keys", "x", "m", "v"):
            assert np.array_equal(a[f], b[f]), (replay, f)
        # unrelated eager work between replays, on both tables
        step(eager, other, pooled_e)
        step(graphed, other, pooled_g)
        torch.cuda.synchronize()
