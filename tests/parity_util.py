"""Helpers shared by the GPU parity tests: run the same batches through the HIP path and the
oracle and compare element by element.

Bars (from the build's problem statement): keys, unique sets, row ids and inverse maps are
compared bit-exactly; float32 parameters and moments within |gpu - ref| <= 1e-6 + 1e-5 |ref|.
A pooled output is a sum of parameters, so its bound is the same bound propagated through the
sum: |gpu - ref| <= sum over the segment's occurrences of (1e-6 + 1e-5 |x_ref|) (a sum of large
rows that cancels to a small value cannot be closer than its summands are).
"""
import numpy as np

ATOL, RTOL = 1e-6, 1e-5


def pooled_tolerance(x_ref, rows, inverse, offsets):
    """Per (segment, column) bound: the parameter tolerance summed over the segment's rows."""
    per_occ = ATOL + RTOL * np.abs(x_ref[rows[inverse]].astype(np.float64))
    c = np.concatenate([np.zeros((1, x_ref.shape[1])), np.cumsum(per_occ, axis=0)])
    off = offsets.astype(np.int64)
    return np.maximum(c[off[1:]] - c[off[:-1]], ATOL)


def assert_close(gpu, ref, what, tol=None):
    gpu = np.asarray(gpu, np.float64)
    ref = np.asarray(ref, np.float64)
    assert gpu.shape == ref.shape, (what, gpu.shape, ref.shape)
    err = np.abs(gpu - ref)
    if tol is None:
        tol = ATOL + RTOL * np.abs(ref)
    bad = err > tol
    if bad.any():
        i = np.unravel_index(np.argmax(err - tol), err.shape)
        raise AssertionError("%s: %d of %d outside tolerance; worst at %s gpu=%r ref=%r" % (
            what, int(bad.sum()), bad.size, i, gpu[i], ref[i]))


def compare_tables(gt, ot, replicas=None, what=""):
    """gt: CtrTable (HIP), ot: OracleTable."""
    assert gt.n_rows == ot.n_rows, (what, gt.n_rows, ot.n_rows)
    for j in (range(ot.W) if replicas is None else replicas):
        g, o = gt.table_export(j), ot.table_export(j)
        assert np.array_equal(g["keys"], o["keys"]), what + " key->row map"
        for f in ("x", "m", "v"):
            if g[f] is None:                     # AdaGrad rows keep no first moment
                assert f == "m" and not o[f].any()
                continue
            assert_close(g[f], o[f], "%s replica %d %s" % (what, j, f))
        if o["vhat"] is not None:
            assert_close(g["vhat"], o["vhat"], "%s shared denominator" % what)


def compare_batch(gt, gbatch, ot, n_keys, what=""):
    gu, gr, gi = gt.batch_export(gbatch, n_keys)
    ou, orows, oi = ot.batch_export(n_keys)
    assert np.array_equal(gu, ou), what + " unique keys"
    assert np.array_equal(gr, orows), what + " rows"
    assert np.array_equal(gi, oi), what + " inverse"


def run_step(gt, ot, batch_t, batch_np, replica=0, mode=0, check_batch=True, what=""):
    """One pull+push on both sides; returns the GPU pooled tensor (host)."""
    from paper_2201_05500_amd import binding as B
    st, gb, pooled = gt.pull_pool(replica, batch_t["keys"], batch_t["offsets"])
    assert st == B.CTR_OK, (what, st)
    ost, opooled = ot.pull_pool(replica, batch_np["keys"], batch_np["offsets"])
    assert ost == 0, (what, ost)
    assert gt.last_status() == B.CTR_OK, what
    if check_batch:
        compare_batch(gt, gb, ot, batch_np["keys"].size, what)
    gp = pooled.cpu().numpy()
    _, orows, oinv = ot.batch_export(batch_np["keys"].size)
    tol = pooled_tolerance(ot.table_export(replica)["x"], orows, oinv, batch_np["offsets"])
    assert_close(gp, opooled, what + " pooled", tol)
    assert gt.push_adam(replica, gb, batch_t["grad"], mode) == B.CTR_OK
    assert ot.push_adam(replica, batch_np["grad"], mode) == 0
    if check_batch:
        u, n_new = gt.batch_stats()
        assert n_new == ot.n_new_last, (what, n_new, ot.n_new_last)
        assert u == np.unique(batch_np["keys"]).size, what
    return gp


def to_device(batch_np, device="cuda:0"):
    import torch
    return {
        "keys": torch.from_numpy(batch_np["keys"].view(np.int64)).to(device),
        "offsets": torch.from_numpy(batch_np["offsets"].view(np.int32)).to(device),
        "grad": torch.from_numpy(batch_np["grad"]).to(device),
    }
