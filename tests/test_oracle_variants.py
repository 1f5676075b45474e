"""Pins for the oracle's optimizer variants: AdaGrad (the paper's optimizer for sparse parameters,
Section 5), the prose reading of the k-step merge (Section 4), and the cited Adam of Kingma & Ba."""
import numpy as np
import pytest

from oracle import ctr_oracle as O

F32 = np.float32
LD = np.longdouble


def _one(key, D, g):
    return np.array([key], np.uint64), np.array([0, 1], np.uint32), np.full((1, D), g, np.float32)


def _step(t, j, keys, off, grad, mode=O.STEP_LOCAL):
    st, pooled = t.pull_pool(j, keys, off)
    assert st == O.OK
    assert t.push_adam(j, grad, mode) == O.OK
    return pooled


# ---------------------------------------------------------------- AdaGrad


@pytest.mark.parametrize("g", [0.5, -3.0, 1e-3])
def test_adagrad_constant_gradient_closed_form(g):
    """G_t = eps + t g^2 and x_T = x_0 - lr sum_t g / sqrt(eps + t g^2)."""
    D, T, lr, eps = 4, 40, 1e-2, 1e-8
    t = O.OracleTable(4, D, lr=lr, eps=eps, init_seed=2, variant=O.VAR_ADAGRAD)
    keys, off, grad = _one(7, D, g)
    x0 = None
    xs = None
    for k in range(1, T + 1):
        p = _step(t, 0, keys, off, grad)
        if k == 1:
            x0 = p[0].astype(LD)
            xs = x0.copy()
        gg = LD(F32(g))
        xs = xs - LD(F32(lr)) * gg / np.sqrt(LD(F32(eps)) + k * gg * gg)
        if k in (1, 2, 9, T):
            s = t.table_export()
            np.testing.assert_allclose(s["v"][0].astype(LD), LD(F32(eps)) + k * gg * gg, rtol=3e-6)
            np.testing.assert_allclose(s["x"][0].astype(LD), xs, rtol=3e-6, atol=1e-7)
            assert np.all(s["m"] == 0)                   # no first moment is kept


def test_adagrad_first_step_and_new_row_and_laziness():
    D = 4
    t = O.OracleTable(8, D, lr=1e-2, eps=1e-8, init_seed=5, variant=O.VAR_ADAGRAD)
    keys = np.array([3, 4, 3], np.uint64)
    off = np.array([0, 1, 3], np.uint32)
    st, p = t.pull_pool(0, keys, off)
    s0 = t.table_export()
    assert np.all(s0["v"] == F32(1e-8))                 # accumulator starts at eps
    g = np.array([[2.0, -1.0, 0.5, 4.0], [1.0, 1.0, -1.0, 0.25]], F32)
    assert t.push_adam(0, g) == O.OK
    s1 = t.table_export()
    # key 3 (row 0) occurs in both segments: one step with the summed gradient; key 4 (row 1) once
    gs = [g[0] + g[1], g[1]]
    for r in range(2):
        np.testing.assert_allclose(s1["v"][r], 1e-8 + gs[r].astype(np.float64) ** 2, rtol=1e-6)
        np.testing.assert_allclose(s0["x"][r].astype(np.float64) - s1["x"][r],
                                   1e-2 * np.sign(gs[r]), rtol=1e-4)   # |g| >> sqrt(eps): step = lr sign(g)
    _step(t, 0, np.array([4], np.uint64), np.array([0, 1], np.uint32), g[:1])
    s2 = t.table_export()
    assert np.array_equal(s1["x"][0], s2["x"][0]) and np.array_equal(s1["v"][0], s2["v"][0])


def test_adagrad_is_single_table_only():
    with pytest.raises(ValueError):
        O.OracleTable(8, 4, n_replicas=2, kstep=True, variant=O.VAR_ADAGRAD)
    t = O.OracleTable(8, 4, variant=O.VAR_ADAGRAD)
    assert t.kstep_merge() == O.E_INVAL


# ---------------------------------------------------------------- Kingma & Ba form


@pytest.mark.parametrize("g", [0.5, -3.0])
def test_bias_corrected_adam_constant_gradient(g):
    """With a constant gradient from the first step, mhat = g and vhat = g^2 at every step, so each step
    moves x by lr g / (|g| + eps) exactly: x_T = x_0 - T lr g / (|g| + eps)."""
    D, T, lr, eps = 4, 30, 1e-3, 1e-8
    t = O.OracleTable(4, D, lr=lr, eps=eps, init_seed=2, variant=O.VAR_KINGMA)
    keys, off, grad = _one(7, D, g)
    x0 = None
    for k in range(1, T + 1):
        p = _step(t, 0, keys, off, grad)
        if k == 1:
            x0 = p[0].astype(np.float64)
            assert np.all(t.table_export()["v"] > 0)
        if k in (1, 5, T):
            s = t.table_export()
            np.testing.assert_allclose(s["x"][0], x0 - k * float(F32(lr)) * g / (abs(g) + float(F32(eps))),
                                       rtol=2e-6, atol=1e-7)
            np.testing.assert_allclose(s["m"][0], (1 - float(F32(0.9)) ** k) * g, rtol=2e-6)
            np.testing.assert_allclose(s["v"][0], (1 - float(F32(0.999)) ** k) * g * g, rtol=2e-5)


def test_bias_corrected_adam_uses_the_global_step_count_and_zero_moments():
    D = 2
    t = O.OracleTable(4, D, lr=1e-3, eps=1e-8, init_seed=2, variant=O.VAR_KINGMA)
    ka, off, ga = _one(1, D, 1.0)
    kb, _, gb = _one(2, D, -2.0)
    st, _ = t.pull_pool(0, ka, off)
    assert np.all(t.table_export()["v"] == 0) and np.all(t.table_export()["m"] == 0)
    assert t.push_adam(0, ga) == O.OK
    for _ in range(3):
        _step(t, 0, ka, off, ga)
    st, p = t.pull_pool(0, kb, off)                      # key 2 first seen at the 5th push
    x0 = p[0].astype(np.float64)
    assert t.push_adam(0, gb) == O.OK
    b1, b2 = float(F32(0.9)), float(F32(0.999))
    m = (1 - b1) * -2.0
    v = (1 - b2) * 4.0
    step = float(F32(1e-3)) * (m / (1 - b1 ** 5)) / (np.sqrt(v / (1 - b2 ** 5)) + float(F32(1e-8)))
    np.testing.assert_allclose(t.table_export()["x"][1], x0 - step, rtol=2e-6)


# ---------------------------------------------------------------- prose reading of the merge


def _random_batch(rng, D, n_keys=12):
    G = int(rng.integers(1, 5))
    counts = rng.integers(0, 4, G)
    off = np.concatenate([[0], np.cumsum(counts)]).astype(np.uint32)
    keys = rng.integers(1, n_keys, off[-1]).astype(np.uint64)
    return keys, off, rng.standard_normal((G, D)).astype(F32)


def test_prose_one_worker_is_plain_adam_bitwise_with_or_without_merges():
    rng = np.random.default_rng(3)
    D = 4
    a = O.OracleTable(16, D, init_seed=9)
    b = O.OracleTable(16, D, init_seed=9, kstep=True, variant=O.VAR_PROSE)
    for s in range(10):
        keys, off, g = _random_batch(rng, D)
        _step(a, 0, keys, off, g)
        _step(b, 0, keys, off, g)
        if s % 3 == 2:
            assert b.kstep_merge() == O.OK
    sa, sb = a.table_export(), b.table_export()
    for f in ("keys", "x", "m", "v"):
        assert np.array_equal(sa[f], sb[f]), f
    assert sb["vhat"] is None


def test_prose_local_steps_are_standard_adam_and_merge_averages_x_and_v():
    """Between merges each worker runs the single-table update on its own state; the merge sets every
    x to the mean of the x_j and every v_j to the mean of the v_j, and leaves m alone."""
    rng = np.random.default_rng(4)
    D, W = 2, 3
    t = O.OracleTable(16, D, n_replicas=W, kstep=True, init_seed=1, variant=O.VAR_PROSE)
    singles = [O.OracleTable(16, D, init_seed=1) for _ in range(W)]
    keys = np.arange(1, 6, dtype=np.uint64)
    off = np.arange(0, 6, dtype=np.uint32)
    for s in range(3):                                   # no merge yet: each worker == its own single table
        for j in range(W):
            g = rng.standard_normal((5, D)).astype(F32)
            _step(t, j, keys, off, g)
            _step(singles[j], 0, keys, off, g)
    pre = [t.table_export(j) for j in range(W)]
    for j in range(W):
        sj = singles[j].table_export()
        for f in ("x", "m", "v"):
            assert np.array_equal(pre[j][f], sj[f]), (j, f)
    assert t.push_adam(0, np.zeros((5, D), F32), O.STEP_MERGE_PENDING) == O.E_INVAL
    assert t.kstep_merge() == O.OK
    post = [t.table_export(j) for j in range(W)]
    xbar = np.mean([p["x"].astype(np.float64) for p in pre], axis=0)
    vbar = np.mean([p["v"].astype(np.float64) for p in pre], axis=0)
    for j in range(W):
        np.testing.assert_allclose(post[j]["x"], xbar, rtol=2e-7, atol=1e-12)
        np.testing.assert_allclose(post[j]["v"], vbar, rtol=2e-7)
        assert np.array_equal(post[j]["x"], post[0]["x"]) and np.array_equal(post[j]["v"], post[0]["v"])
        assert np.array_equal(post[j]["m"], pre[j]["m"])


def test_prose_merge_skips_untouched_rows():
    D, W = 2, 3
    t = O.OracleTable(8, D, n_replicas=W, kstep=True, init_seed=1, variant=O.VAR_PROSE)
    ka, off, g = _one(10, D, 1.0)
    kb, _, _ = _one(20, D, 1.0)
    _step(t, 0, ka, off, g)
    _step(t, 1, kb, off, g)
    t.kstep_merge()
    s0 = [t.table_export(j) for j in range(W)]
    _step(t, 2, ka, off, g)
    t.kstep_merge()
    s1 = [t.table_export(j) for j in range(W)]
    for j in range(W):
        for f in ("x", "v"):
            assert np.array_equal(s0[j][f][1], s1[j][f][1])     # key 20 untouched in merge round 2


def test_variant_argument_checks():
    with pytest.raises(ValueError):
        O.OracleTable(8, 4, variant=O.VAR_PROSE)                  # prose needs k-step mode
    with pytest.raises(ValueError):
        O.OracleTable(8, 4, kstep=True, variant=O.VAR_KINGMA)
    with pytest.raises(ValueError):
        O.OracleTable(8, 4, n_replicas=2)                         # replicas exist to be merged


# ---------------------------------------------------------------- working-set load / collection


def test_load_then_pull_pools_the_loaded_rows_and_collect_returns_them():
    """Algorithm 1: insert_into_hash_table of a parameter partition, then pulls see those parameters;
    pull_updates_peer_GPU hands back what the table holds."""
    rng = np.random.default_rng(8)
    D = 4
    for kw in (dict(), dict(n_replicas=3, kstep=True), dict(variant=O.VAR_ADAGRAD)):
        t = O.OracleTable(8, D, init_seed=1, **kw)
        keys = np.array([50, 10, 30], np.uint64)
        x = rng.standard_normal((3, D)).astype(F32)
        m = rng.standard_normal((3, D)).astype(F32)
        v = rng.random((3, D)).astype(F32) + 0.1
        assert t.table_load(keys, x, m, v) == O.OK
        assert t.n_rows == 3 and [t.lookup(int(k)) for k in keys] == [0, 1, 2]     # rows in the order given
        st, pooled = t.pull_pool(0, np.array([10, 30, 10, 77], np.uint64), np.array([0, 3, 4], np.uint32))
        np.testing.assert_allclose(pooled[0], (2 * x[1].astype(np.float64) + x[2]).astype(F32), rtol=1e-6)
        assert t.n_rows == 4                                        # 77 was new: ordinary insert-on-miss
        for j in range(t.W):
            st, cx, cm, cv, found = t.table_collect(j, np.array([30, 99, 50], np.uint64))
            assert st == O.OK and list(found) == [1, 0, 1]
            assert np.array_equal(cx[0], x[2]) and np.array_equal(cx[2], x[0]) and not cx[1].any()
            assert np.array_equal(cv[0], v[2])
            if t.variant != O.VAR_ADAGRAD:
                assert np.array_equal(cm[2], m[0])
        assert t.lookup(99) == -1                                   # collecting never inserts
        if t.kstep:
            assert np.array_equal(t.table_export(0)["vhat"][:3], v)    # shared denominator := v
        # loading an existing key overwrites its row and creates none
        assert t.table_load(np.array([10], np.uint64), x[:1] + 1, m[:1], v[:1]) == O.OK
        assert t.n_rows == 4 and np.array_equal(t.table_export(0)["x"][1], x[0] + 1)


def test_load_capacity_and_sentinel_leave_the_table_unchanged():
    D = 2
    t = O.OracleTable(3, D, init_seed=1)
    z = np.zeros((4, D), F32)
    assert t.table_load(np.array([1, 2], np.uint64), z[:2], z[:2], z[:2] + 1) == O.OK
    assert t.table_load(np.array([2, 3, 4], np.uint64), z[:3], z[:3], z[:3] + 1) == O.E_FULL
    assert t.table_load(np.array([2, 2 ** 64 - 1], np.uint64), z[:2], z[:2], z[:2] + 1) == O.E_BADKEY
    assert t.n_rows == 2 and t.lookup(3) == -1
    assert t.table_load(np.array([2, 3], np.uint64), z[:2], z[:2], z[:2] + 1) == O.OK and t.n_rows == 3


def test_clear_makes_the_table_equal_to_a_fresh_one():
    """Algorithm 1's outer loop: the hash table is emptied and the next working set loaded.  After a clear,
    everything behaves as in a table that was just created (rows renumbered from 0, old keys unknown)."""
    rng = np.random.default_rng(3)
    D = 4
    for kw in (dict(), dict(n_replicas=2, kstep=True)):
        a = O.OracleTable(16, D, init_seed=2, **kw)
        b = O.OracleTable(16, D, init_seed=2, **kw)
        keys = np.array([7, 8, 9, 7], np.uint64)
        off = np.array([0, 2, 4], np.uint32)
        g = rng.standard_normal((2, D)).astype(F32)
        mode = O.STEP_MERGE_PENDING if a.kstep else O.STEP_LOCAL
        assert a.pull_pool(0, keys, off)[0] == O.OK and a.push_adam(0, g, mode) == O.OK
        assert a.table_clear() == O.OK
        assert a.n_rows == 0 and a.lookup(7) == -1
        assert a.push_adam(0, g) != O.OK                            # the batch of before the clear is gone
        if a.kstep:
            assert a.kstep_merge() == O.OK                          # nothing pending, nothing touched
        keys2 = np.array([9, 5, 9], np.uint64)
        off2 = np.array([0, 1, 3], np.uint32)
        for t in (a, b):
            st, pooled = t.pull_pool(0, keys2, off2)
            assert st == O.OK and t.push_adam(0, g, mode) == O.OK
            if t.kstep:
                assert t.kstep_merge() == O.OK
        assert a.lookup(9) == 0 and a.lookup(5) == 1 and a.n_rows == 2
        ea, eb = a.table_export(0), b.table_export(0)
        for f in ("keys", "x", "m", "v"):
            assert np.array_equal(ea[f], eb[f]), f


def test_lookup_pool_reads_without_inserting():
    """Prediction path: pooling over the keys that are in the table, nothing for the others, no side effects."""
    from fractions import Fraction
    rng = np.random.default_rng(12)
    D = 4
    t = O.OracleTable(16, D, init_seed=5)
    train_keys = np.array([3, 4, 5, 3], np.uint64)
    off = np.array([0, 2, 4], np.uint32)
    st, pooled_train = t.pull_pool(0, train_keys, off)
    assert st == O.OK and t.push_adam(0, rng.standard_normal((2, D)).astype(F32)) == O.OK
    before = t.table_export(0)
    # all keys present: the same sums a pull would give now
    st, a = t.lookup_pool(0, train_keys, off)
    st2, b = t.pull_pool(0, train_keys, off)
    assert st == O.OK and st2 == O.OK and np.array_equal(a, b)
    # absent keys (77, 99) add nothing and are not inserted; exact rational sums of the present rows
    keys = np.array([77, 4, 99, 5, 5, 99], np.uint64)
    off2 = np.array([0, 1, 3, 3, 6], np.uint32)
    st, p = t.lookup_pool(0, keys, off2)
    assert st == O.OK and t.n_rows == 3 and t.lookup(77) == -1 and t.lookup(99) == -1
    x = before["x"]
    row = {3: 0, 4: 1, 5: 2}
    want = [[Fraction(0)] * D, [Fraction(float(x[row[4]][d])) for d in range(D)], [Fraction(0)] * D,
            [2 * Fraction(float(x[row[5]][d])) for d in range(D)]]
    for g in range(4):
        for d in range(D):
            assert p[g, d] == F32(float(want[g][d])), (g, d)
    after = t.table_export(0)
    for f in ("keys", "x", "m", "v"):
        assert np.array_equal(before[f], after[f])
    # error conventions as for a pull
    assert t.lookup_pool(0, np.array([1, 2 ** 64 - 1], np.uint64), np.array([0, 2], np.uint32))[0] == O.E_BADKEY
    assert t.lookup_pool(0, keys, np.array([0, 4, 3, 6], np.uint32))[0] == O.E_INVAL
    assert t.lookup_pool(1, keys, off2)[0] == O.E_INVAL
