"""The entry point that allocates nothing (ctr_lookup_pool_noalloc) against ctr_lookup_pool, through the C ABI:
two calls in a row on the shared fixed scratch, the second with a smaller input; the size limit; no effect on
a live batch.  The file name sorts last on purpose: a failure here must not hide the other GPU tests."""
import pytest

from oracle import ctr_oracle as O
from paper_2201_05500_amd import workloads as WL
from tests.parity_util import run_step, to_device

pytestmark = pytest.mark.gpu


def _noalloc(B, gt, replica, keys, offsets, out):
    import torch
    n_keys, n_seg = keys.numel(), offsets.numel() - 1
    bf16 = out.dtype == torch.bfloat16
    ptr = out.data_ptr() if n_seg else None
    return B.ctr_lookup_pool_noalloc(gt._handle, replica, keys.data_ptr() if n_keys else None, n_keys,
                                     offsets.data_ptr(), n_seg, None if bf16 else ptr, ptr if bf16 else None,
                                     gt.stream)


@pytest.mark.parametrize("dim", [8, 64])
def test_noalloc_lookup_equals_lookup_on_two_calls_in_a_row(dim):
    import torch
    from paper_2201_05500_amd import binding as B
    w = WL.scaled(WL.WORKLOADS["large"], capacity_rows=1 << 15, zipf_universe=40000, batch=64, slots=24, dim=dim)
    gt = B.CtrTable(w.capacity_rows, w.dim, init_seed=8, init_std=0.05)
    ot = O.OracleTable(w.capacity_rows, w.dim, init_seed=8, init_std=0.05)
    for s in range(3):
        bn = WL.as_numpy(WL.make_batch(w, s))
        run_step(gt, ot, to_device(bn), bn, what="training step %d" % s)
    big = to_device(WL.as_numpy(WL.make_batch(w, 50)))            # part of its keys were never seen
    small = to_device(WL.as_numpy(WL.make_batch(WL.scaled(w, batch=9, slots=7), 51)))
    assert small["keys"].numel() < big["keys"].numel() // 4
    # the reference results first, with the caller's workspace
    ref = []
    for b in (big, small):
        st, p = gt.lookup_pool(0, b["keys"], b["offsets"])
        assert st == B.CTR_OK
        st, p16 = gt.lookup_pool(0, b["keys"], b["offsets"], bf16=True)
        assert st == B.CTR_OK
        ref.append((p.clone(), p16.clone()))
    torch.cuda.synchronize()
    # then the fixed-scratch entry point: large call, smaller call, large call again, nothing in between
    outs = []
    for b in (big, small, big):
        n_seg = b["offsets"].numel() - 1
        p = torch.full((n_seg, dim), float("nan"), dtype=torch.float32, device="cuda")
        p16 = torch.full((n_seg, dim), float("nan"), dtype=torch.bfloat16, device="cuda")
        assert _noalloc(B, gt, 0, b["keys"], b["offsets"], p) == B.CTR_OK
        assert _noalloc(B, gt, 0, b["keys"], b["offsets"], p16) == B.CTR_OK
        outs.append((p, p16))
    assert gt.last_status() == B.CTR_OK
    for (p, p16), (rp, rp16) in zip(outs, (ref[0], ref[1], ref[0])):
        assert torch.equal(p, rp) and torch.equal(p16, rp16)       # same kernels, same order: bit-identical


def test_noalloc_limit_errors_and_live_batch():
    import torch
    from paper_2201_05500_amd import binding as B
    w = WL.scaled(WL.WORKLOADS["tiny"], capacity_rows=4096, zipf_universe=3000, batch=16)
    gt = B.CtrTable(w.capacity_rows, w.dim, init_seed=2)
    bt = to_device(WL.as_numpy(WL.make_batch(w, 0)))
    st, h, _ = gt.pull_pool(0, bt["keys"], bt["offsets"])
    assert st == B.CTR_OK
    n_seg = bt["offsets"].numel() - 1
    out = torch.empty((n_seg, w.dim), dtype=torch.float32, device="cuda")
    # beyond the fixed scratch: rejected on the host, nothing enqueued (the key pointer is never read)
    too_many = B.CTR_NOALLOC_MAX_KEYS + 1
    assert B.ctr_lookup_pool_noalloc(gt._handle, 0, bt["keys"].data_ptr(), too_many, bt["offsets"].data_ptr(), n_seg,
                                     out.data_ptr(), None, gt.stream) == B.CTR_E_NOMEM
    assert B.ctr_lookup_pool_noalloc(gt._handle, 1, bt["keys"].data_ptr(), bt["keys"].numel(),
                                     bt["offsets"].data_ptr(), n_seg, out.data_ptr(), None,
                                     gt.stream) == B.CTR_E_INVAL      # no such replica
    assert B.ctr_lookup_pool_noalloc(gt._handle, 0, bt["keys"].data_ptr(), bt["keys"].numel(),
                                     bt["offsets"].data_ptr(), n_seg, None, None, gt.stream) == B.CTR_E_INVAL
    # the scratch is not the batch's workspace: the live batch survives a lookup and can still be pushed
    assert _noalloc(B, gt, 0, bt["keys"], bt["offsets"], out) == B.CTR_OK
    assert gt.push_adam(0, h, bt["grad"]) == B.CTR_OK
    assert gt.last_status() == B.CTR_OK
    # deferred errors as in ctr_lookup_pool
    keys = torch.tensor([5, -1, 7], dtype=torch.int64, device="cuda")
    offs = torch.tensor([0, 1, 3], dtype=torch.int32, device="cuda")
    out2 = torch.empty((2, w.dim), dtype=torch.float32, device="cuda")
    assert _noalloc(B, gt, 0, keys, offs, out2) == B.CTR_OK
    assert gt.last_status() == B.CTR_E_BADKEY and gt.last_status() == B.CTR_OK
