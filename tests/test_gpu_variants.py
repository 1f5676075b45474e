"""GPU parity for the optimizer variants (AdaGrad, prose reading of the merge, Kingma-form Adam)."""
import numpy as np
import pytest

from oracle import ctr_oracle as O
from paper_2201_05500_amd import workloads as WL
from tests.parity_util import compare_tables, run_step, to_device

pytestmark = pytest.mark.gpu


def _pair(w, variant, seed=11, **kw):
    from paper_2201_05500_amd.binding import CtrTable
    hp = dict(lr=w.lr, beta1=w.beta1, beta2=w.beta2, eps=w.eps, init_seed=seed, init_std=w.init_std)
    hp.update(kw)
    kstep = variant == O.VAR_PROSE
    W = w.n_replicas if kstep else 1
    gt = CtrTable(w.capacity_rows, w.dim, n_replicas=W, kstep=kstep, adagrad=variant == O.VAR_ADAGRAD,
                  prose=variant == O.VAR_PROSE, bias_correction=variant == O.VAR_KINGMA, **hp)
    ot = O.OracleTable(w.capacity_rows, w.dim, n_replicas=W, kstep=kstep, variant=variant, **hp)
    return gt, ot


@pytest.mark.parametrize("variant", [O.VAR_ADAGRAD, O.VAR_KINGMA])
@pytest.mark.parametrize("name,kw", [
    ("tiny", {}),
    ("large", dict(capacity_rows=(1 << 16) + 3, zipf_universe=50000, batch=128)),
    ("mid", dict(capacity_rows=1 << 15, zipf_universe=1 << 15, batch=256)),
])
def test_single_table_variants(variant, name, kw):
    w = WL.scaled(WL.WORKLOADS[name], **kw)
    gt, ot = _pair(w, variant)
    for s in range(4):
        bn = WL.as_numpy(WL.make_batch(w, s))
        run_step(gt, ot, to_device(bn), bn, what="%s variant %d step %d" % (name, variant, s))
        compare_tables(gt, ot, what="%s variant %d after step %d" % (name, variant, s))


def test_adagrad_export_has_no_first_moment():
    from paper_2201_05500_amd import binding as B
    import ctypes as C
    w = WL.scaled(WL.WORKLOADS["tiny"], batch=8)
    gt, ot = _pair(w, O.VAR_ADAGRAD)
    bn = WL.as_numpy(WL.make_batch(w, 0))
    run_step(gt, ot, to_device(bn), bn)
    buf = np.empty((gt.n_rows, w.dim), np.float32)
    st = B.lib().ctr_table_export(gt._handle, 0, None, None, buf.ctypes.data_as(C.c_void_p), None, None, gt.stream)
    assert st == B.CTR_E_INVAL
    assert gt.kstep_merge() == B.CTR_E_INVAL


@pytest.mark.parametrize("W,k", [(3, 2), (8, 4), (1, 1)])
def test_prose_merge_variant(W, k):
    w = WL.scaled(WL.WORKLOADS["kstep"], capacity_rows=1 << 13, zipf_universe=6000, batch=32, n_replicas=W)
    gt, ot = _pair(w, O.VAR_PROSE)
    from paper_2201_05500_amd import binding as B
    step = 0
    for rnd in range(3):
        for i in range(k):
            for j in range(W):
                bn = WL.as_numpy(WL.make_batch(w, step, replica=j))
                run_step(gt, ot, to_device(bn), bn, replica=j, what="prose round %d step %d replica %d" % (rnd, i, j))
            step += 1
        assert gt.kstep_merge() == 0 and ot.kstep_merge() == 0
        compare_tables(gt, ot, what="prose after merge %d" % rnd)
    # the deferred step of Algorithm 2 does not exist in this reading
    bt = to_device(WL.as_numpy(WL.make_batch(w, 99)))
    st, gb, _ = gt.pull_pool(0, bt["keys"], bt["offsets"])
    assert gt.push_adam(0, gb, bt["grad"], B.CTR_STEP_MERGE_PENDING) == B.CTR_E_INVAL
    assert gt.push_adam(0, gb, bt["grad"]) == B.CTR_OK
