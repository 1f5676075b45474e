"""GPU parity of ctr_push_adam_bf16: pooled gradients handed over as bfloat16.  The oracle takes the same
values widened to fp32 (a bf16 value is an fp32 value with 16 zero low bits, so nothing is rounded on the way),
and the bar is the one of the fp32 push."""
import numpy as np
import pytest

from oracle import ctr_oracle as O
from paper_2201_05500_amd import workloads as WL
from tests.parity_util import compare_tables, run_step, to_device

pytestmark = pytest.mark.gpu


def _bf16_batch(w, s, replica=0):
    """(device batch with a bfloat16 gradient, host batch with the same values as fp32)."""
    import torch
    bn = WL.as_numpy(WL.make_batch(w, s, replica=replica))
    g16 = torch.from_numpy(bn["grad"]).to(torch.bfloat16)
    bn["grad"] = g16.to(torch.float32).numpy()
    assert not (bn["grad"].view(np.uint32) & 0xFFFF).any()
    bt = to_device(bn)
    bt["grad"] = g16.to("cuda:0")
    return bt, bn


def _pair(w, variant=O.VAR_ALG2, seed=21):
    from paper_2201_05500_amd.binding import CtrTable
    hp = dict(lr=w.lr, beta1=w.beta1, beta2=w.beta2, eps=w.eps, init_seed=seed, init_std=w.init_std)
    kstep = w.k_step > 0
    gt = CtrTable(w.capacity_rows, w.dim, n_replicas=w.n_replicas, kstep=kstep, load_factor=w.load_factor,
                  adagrad=variant == O.VAR_ADAGRAD, bias_correction=variant == O.VAR_KINGMA, **hp)
    ot = O.OracleTable(w.capacity_rows, w.dim, n_replicas=w.n_replicas, kstep=kstep, variant=variant, **hp)
    return gt, ot


@pytest.mark.parametrize("dim", [4, 12, 64, 100, 256])
def test_bf16_gradients_every_lane_group_width(dim):
    w = WL.scaled(WL.WORKLOADS["tiny"], dim=dim, batch=96, capacity_rows=6000, zipf_universe=3000)
    gt, ot = _pair(w)
    for s in range(3):
        bt, bn = _bf16_batch(w, s)
        run_step(gt, ot, bt, bn, what="dim %d step %d" % (dim, s))
        compare_tables(gt, ot, what="dim %d after step %d" % (dim, s))


def test_bf16_gradients_hot_key_over_many_spans():
    """Configuration 3's shape reduced: the hot key's occurrences run over many work spans, so partial sums
    of widened bf16 gradients go through the fix-up kernels too."""
    w = WL.scaled(WL.WORKLOADS["large"], capacity_rows=(1 << 16) + 9, zipf_universe=40000, batch=192)
    gt, ot = _pair(w)
    for s in range(3):
        bt, bn = _bf16_batch(w, s)
        run_step(gt, ot, bt, bn, what="large/bf16 step %d" % s)
        compare_tables(gt, ot, what="large/bf16 after step %d" % s)


@pytest.mark.parametrize("variant", [O.VAR_ADAGRAD, O.VAR_KINGMA])
def test_bf16_gradients_other_row_updates(variant):
    w = WL.scaled(WL.WORKLOADS["mid"], capacity_rows=1 << 14, zipf_universe=1 << 14, batch=128)
    gt, ot = _pair(w, variant)
    for s in range(3):
        bt, bn = _bf16_batch(w, s)
        run_step(gt, ot, bt, bn, what="variant %d step %d" % (variant, s))
        compare_tables(gt, ot, what="variant %d after step %d" % (variant, s))


def test_bf16_gradients_kstep_with_deferred_step():
    """Algorithm 2 on 3 replicas, k = 2: local steps on the shared denominator, the k-th step deferred into
    the merge, all with bf16 gradients."""
    from paper_2201_05500_amd import binding as B
    w = WL.scaled(WL.WORKLOADS["kstep"], capacity_rows=1 << 13, zipf_universe=6000, batch=32, n_replicas=3)
    gt, ot = _pair(w)
    step = 0
    for rnd in range(3):
        for i in range(2):
            mode = B.CTR_STEP_MERGE_PENDING if i == 1 else B.CTR_STEP_LOCAL
            for j in range(3):
                bt, bn = _bf16_batch(w, step, replica=j)
                run_step(gt, ot, bt, bn, replica=j, mode=mode, what="round %d step %d replica %d" % (rnd, i, j))
            step += 1
        assert gt.kstep_merge() == B.CTR_OK
        ot.kstep_merge()
        compare_tables(gt, ot, what="after merge %d" % rnd)


def test_bf16_and_fp32_pushes_of_the_same_values_agree_bit_for_bit():
    import torch
    from paper_2201_05500_amd.binding import CTR_OK, CtrTable
    w = WL.scaled(WL.WORKLOADS["large"], capacity_rows=1 << 15, zipf_universe=9000, batch=64, slots=40)
    ta, tb = (CtrTable(w.capacity_rows, w.dim, init_seed=3, init_std=0.02) for _ in range(2))
    for s in range(2):
        bt, bn = _bf16_batch(w, s)
        for t, g in ((ta, bt["grad"]), (tb, bt["grad"].to(torch.float32))):
            st, h, _ = t.pull_pool(0, bt["keys"], bt["offsets"])
            assert st == CTR_OK
            assert t.push_adam(0, h, g) == CTR_OK
            assert t.last_status() == CTR_OK
    ea, eb = ta.table_export(0), tb.table_export(0)
    for k in ("keys", "x", "m", "v"):
        assert np.array_equal(ea[k], eb[k]), k


def test_bf16_gradient_pointer_must_be_8_byte_aligned():
    import torch
    from paper_2201_05500_amd import binding as B
    w = WL.scaled(WL.WORKLOADS["tiny"], batch=8)
    gt, _ = _pair(w)
    bt, bn = _bf16_batch(w, 0)
    st, h, _ = gt.pull_pool(0, bt["keys"], bt["offsets"])
    assert st == B.CTR_OK
    flat = torch.empty(bt["grad"].numel() + 1, dtype=torch.bfloat16, device="cuda:0")
    off = flat[1:]
    assert off.data_ptr() % 8 != 0
    assert B.lib().ctr_push_adam_bf16(gt._handle, 0, h, off.data_ptr(), B.CTR_STEP_LOCAL, gt.stream) == B.CTR_E_INVAL
    assert gt.push_adam(0, h, bt["grad"]) == B.CTR_OK        # the batch is still live after CTR_E_INVAL
