"""Pins for the CPU oracle: what the paper and the mathematics fix, checked without the HIP path.

Each test names the passage it pins.  None of them re-runs the oracle's own
recurrence: they use closed forms of Algorithm 2 for a constant gradient, the
identities of the convergence proof (Section 4, proof sketch), special cases
(k = 1 with one worker is plain Adam, identical workers), and brute force with
exact rational sums on tiny inputs.
"""
from fractions import Fraction

import numpy as np
import pytest

from oracle import ctr_oracle as O

F32 = np.float32
LD = np.longdouble


def one_key_batch(key, D, g):
    keys = np.array([key], np.uint64)
    offsets = np.array([0, 1], np.uint32)
    grad = np.full((1, D), g, np.float32) if np.isscalar(g) else np.asarray(g, np.float32).reshape(1, D)
    return keys, offsets, grad


def step(t, replica, keys, offsets, grad, mode=O.STEP_LOCAL):
    st, pooled = t.pull_pool(replica, keys, offsets)
    assert st == O.OK
    assert t.push_adam(replica, grad, mode) == O.OK
    return pooled


# ---------------------------------------------------------------- Algorithm 2, lines for m, v, x


@pytest.mark.parametrize("g", [0.5, -2.0, 1e-3, 37.0])
@pytest.mark.parametrize("beta1", [0.9, 0.0])
def test_constant_gradient_closed_form(g, beta1):
    """Algorithm 2 with N = 1, k = 1 and a constant gradient has the closed forms
    m_t = (1 - b1^t) g,  v_t = b2^t eps + (1 - b2^t) g^2,  x_T = x_0 - a sum_t m_t / sqrt(v_t)."""
    lr, beta2, eps, D, T = 1e-3, 0.999, 1e-8, 4, 60
    t = O.OracleTable(8, D, lr=lr, beta1=beta1, beta2=beta2, eps=eps, init_seed=3, init_std=0.01)
    keys, offsets, grad = one_key_batch(12345, D, g)
    st, pooled0 = t.pull_pool(0, keys, offsets)
    assert st == O.OK
    x0 = pooled0[0].astype(LD)           # a one-key segment pools to the row itself
    assert t.push_adam(0, grad) == O.OK
    b1, b2, a, e, gg = LD(F32(beta1)), LD(F32(beta2)), LD(F32(lr)), LD(F32(eps)), LD(F32(g))
    xs = x0.copy()
    for k in range(1, T + 1):
        if k > 1:
            step(t, 0, keys, offsets, grad)
        m_k = (1 - b1 ** k) * gg
        v_k = b2 ** k * e + (1 - b2 ** k) * gg * gg
        xs = xs - a * m_k / np.sqrt(v_k)
        if k in (1, 2, 7, T):
            s = t.table_export()
            np.testing.assert_allclose(s["m"][0].astype(LD), m_k, rtol=2e-6, atol=0)
            np.testing.assert_allclose(s["v"][0].astype(LD), v_k, rtol=2e-6, atol=0)
            np.testing.assert_allclose(s["x"][0].astype(LD), xs, rtol=5e-6, atol=1e-7)


def test_beta1_zero_first_step_size():
    """With beta1 = 0 (the paper's production setting, Section 5) m_t = g_t exactly, and the first
    step is a g / sqrt(b2 eps + (1 - b2) g^2), about a / sqrt(1 - b2) = 31.62 a for |g| >> 1e-2.5."""
    D = 4
    t = O.OracleTable(4, D, lr=1e-3, beta1=0.0, beta2=0.999, eps=1e-8, init_seed=1)
    g = np.array([[1.0, -1.0, 3.25, -0.75]], np.float32)
    keys, offsets, _ = one_key_batch(99, D, 0.0)
    st, p0 = t.pull_pool(0, keys, offsets)
    assert t.push_adam(0, g) == O.OK
    s = t.table_export()
    assert np.array_equal(s["m"][0], g[0])
    dx = p0[0].astype(np.float64) - s["x"][0].astype(np.float64)
    np.testing.assert_allclose(dx, np.sign(g[0]) * 1e-3 / np.sqrt(1 - 0.999), rtol=2e-3)
    expect = 1e-3 * g[0].astype(np.float64) / np.sqrt(
        float(F32(0.999)) * float(F32(1e-8)) + (1 - float(F32(0.999))) * g[0].astype(np.float64) ** 2)
    np.testing.assert_allclose(dx, expect * (float(F32(1e-3)) / 1e-3), rtol=1e-5)


def test_v_positive_and_lower_bound():
    """v stays positive; from the v line of Algorithm 2, v after n touches is >= b2^n eps
    (zero gradient attains it)."""
    D = 2
    t = O.OracleTable(4, D, init_seed=1)
    keys, offsets, grad = one_key_batch(5, D, 0.0)
    for n in range(1, 30):
        step(t, 0, keys, offsets, grad)
        v = t.table_export()["v"][0].astype(np.float64)
        assert np.all(v > 0)
        np.testing.assert_allclose(v, float(F32(0.999)) ** n * float(F32(1e-8)), rtol=1e-5)


def test_new_row_state():
    """Algorithm 2, Initialize: m_0 = 0, v_0 = eps; x_0 is the deterministic init of the key."""
    D = 8
    t = O.OracleTable(16, D, eps=1e-8, init_seed=11, init_std=0.01, kstep=True, n_replicas=2)
    keys = np.array([7, 9, 7, 3], np.uint64)
    offsets = np.array([0, 4], np.uint32)
    st, _ = t.pull_pool(1, keys, offsets)
    assert st == O.OK and t.n_rows == 3
    for j in range(2):
        s = t.table_export(j)
        assert list(s["keys"]) == [7, 9, 3]          # first-occurrence order
        assert np.all(s["m"] == 0)
        assert np.all(s["v"] == F32(1e-8)) and np.all(s["vhat"] == F32(1e-8))
        for r, k in enumerate([7, 9, 3]):
            for d in range(D):
                assert s["x"][r, d] == F32(O.init_value(11, k, d, 0.01))


def test_init_value_distribution():
    """The init stand-in is centred, has the requested spread, is bounded, and depends on each of
    seed, key and column."""
    n = 40000
    vals = np.array([O.init_value(5, 1000003 * i + 17, i % 64, 0.01) for i in range(n)])
    assert abs(vals.mean()) < 3 * 0.01 / np.sqrt(n) * 1.5
    assert abs(vals.std() - 0.01) < 0.01 * 0.02
    assert np.abs(vals).max() <= 131070 * (0.01 / 37837.2) * (1 + 1e-6)
    a = O.init_value(5, 42, 0, 0.01)
    assert a == O.init_value(5, 42, 0, 0.01)
    assert len({a, O.init_value(6, 42, 0, 0.01), O.init_value(5, 43, 0, 0.01),
                O.init_value(5, 42, 1, 0.01)}) == 4
    assert O.init_value(5, 42, 0, 0.02) == pytest.approx(2 * a, rel=1e-6)


# ---------------------------------------------------------------- push: duplicates, laziness


def test_duplicate_keys_equal_summed_gradient():
    """A key occurring c times takes one step with the sum of its c gradients."""
    D = 4
    ga = np.array([[0.5, 1.25, -2.0, 8.0], [0.25, -0.25, 4.0, 1.0], [1.0, 1.0, 1.0, 1.0],
                   [-3.5, 0.125, 0.5, 2.0]], np.float32)
    ta = O.OracleTable(8, D, init_seed=2)
    tb = O.OracleTable(8, D, init_seed=2)
    # A: key 77 in segments 0, 1 (twice) and 3; key 5 in segment 2
    keys_a = np.array([77, 77, 77, 5, 77], np.uint64)
    off_a = np.array([0, 1, 3, 4, 5], np.uint32)
    # B: key 77 once with the summed gradient; key 5 once
    keys_b = np.array([77, 5], np.uint64)
    off_b = np.array([0, 1, 2], np.uint32)
    gb = np.stack([ga[0] + 2 * ga[1] + ga[3], ga[2]]).astype(np.float32)
    for _ in range(3):
        step(ta, 0, keys_a, off_a, ga)
        step(tb, 0, keys_b, off_b, gb)
    sa, sb = ta.table_export(), tb.table_export()
    for f in ("keys", "x", "m", "v"):
        assert np.array_equal(sa[f], sb[f]), f


def test_untouched_rows_do_not_change():
    """Sparse update: a push changes the rows of its batch only."""
    D = 4
    t = O.OracleTable(8, D, init_seed=2)
    step(t, 0, np.array([1, 2, 3], np.uint64), np.array([0, 3], np.uint32), np.ones((1, D), F32))
    before = t.table_export()
    step(t, 0, np.array([2], np.uint64), np.array([0, 1], np.uint32), np.ones((1, D), F32))
    after = t.table_export()
    for f in ("x", "m", "v"):
        assert np.array_equal(before[f][[0, 2]], after[f][[0, 2]])
        assert not np.array_equal(before[f][1], after[f][1])


def test_empty_segment_pools_to_zero_and_gets_no_gradient():
    D = 4
    t = O.OracleTable(8, D, init_seed=2)
    keys = np.array([4, 6], np.uint64)
    off = np.array([0, 1, 1, 2, 2], np.uint32)          # segments 1 and 3 are empty
    grad = np.arange(16, dtype=np.float32).reshape(4, D) + 1
    st, pooled = t.pull_pool(0, keys, off)
    assert np.all(pooled[1] == 0) and np.all(pooled[3] == 0)
    assert t.push_adam(0, grad) == O.OK
    s = t.table_export()
    # beta1 = 0.9: m = 0.1 * g of the segment that holds the key
    np.testing.assert_allclose(s["m"][0], (1 - float(F32(0.9))) * grad[0], rtol=1e-6)
    np.testing.assert_allclose(s["m"][1], (1 - float(F32(0.9))) * grad[2], rtol=1e-6)


# ---------------------------------------------------------------- k-step merge (Algorithm 2)


def _run_single_vs_k1(T=12, D=4):
    rng = np.random.default_rng(4)
    a = O.OracleTable(16, D, init_seed=9)
    b = O.OracleTable(16, D, init_seed=9, kstep=True, n_replicas=1)
    for s in range(T):
        n = rng.integers(1, 9)
        keys = rng.integers(1, 12, n).astype(np.uint64)
        off = np.array([0, n // 2, n], np.uint32)
        grad = rng.standard_normal((2, D)).astype(F32)
        step(a, 0, keys, off, grad)
        step(b, 0, keys, off, grad, O.STEP_MERGE_PENDING)
        assert b.kstep_merge() == O.OK
    return a.table_export(), b.table_export()


def test_k1_one_worker_is_plain_adam_bitwise():
    """Algorithm 2 with N = 1 and k = 1: every step is a merge step, v_t = v_{t,1}, and the update is
    the single-table step; the two code paths must agree bit for bit."""
    sa, sb = _run_single_vs_k1()
    for f in ("keys", "x", "m", "v"):
        assert np.array_equal(sa[f], sb[f]), f
    assert np.array_equal(sb["vhat"], sb["v"])


def _dense_toy(W=3, k=3, T=9, D=2, n_keys=4, seed=0, same_grads=False, beta1=0.9):
    """Every replica touches every row at every step.  Returns per-step records."""
    rng = np.random.default_rng(seed)
    t = O.OracleTable(n_keys, D, n_replicas=W, kstep=True, init_seed=5, beta1=beta1)
    keys = np.arange(1, n_keys + 1, dtype=np.uint64)
    off = np.arange(0, n_keys + 1, dtype=np.uint32)
    rec = []
    for s in range(1, T + 1):
        before = [t.table_export(j) for j in range(W)] if t.n_rows else None
        g = rng.standard_normal((W, n_keys, D)).astype(F32)
        if same_grads:
            g[:] = g[0]
        mode = O.STEP_MERGE_PENDING if s % k == 0 else O.STEP_LOCAL
        for j in range(W):
            step(t, j, keys, off, g[j], mode)
        after_push = [t.table_export(j) for j in range(W)]
        if s % k == 0:
            assert t.kstep_merge() == O.OK
        after = [t.table_export(j) for j in range(W)]
        rec.append(dict(step=s, merge=(s % k == 0), g=g, before=before, after_push=after_push, after=after))
    return t, rec


def _mean(states, f):
    return np.mean([s[f].astype(np.float64) for s in states], axis=0)


def test_averaged_iterate_identity():
    """Proof sketch, Section 4: the averaged model obeys xbar_{t+1} = xbar_t - a mbar_t / sqrt(v_t)
    at every step, local or merge, with v_t the shared denominator in force at step t."""
    lr = float(F32(1e-3))
    _, rec = _dense_toy()
    for r in rec[1:]:
        xbar_t = _mean(r["before"], "x")
        mbar_t = _mean(r["after_push"], "m")
        vhat_t = r["after"][0]["vhat"].astype(np.float64)
        xbar_next = _mean(r["after"], "x")
        np.testing.assert_allclose(xbar_next, xbar_t - lr * mbar_t / np.sqrt(vhat_t),
                                   rtol=3e-6, atol=1e-6)


def test_shared_denominator_frozen_between_merges_and_averaged_at_merge():
    """Algorithm 2: v_t = v_{t-1} on local steps; v_t = (1/N) sum_i v_{t,i} on merge steps, while the
    local v_{t,i} keep their own recursion."""
    _, rec = _dense_toy()
    for r in rec[1:]:
        old = r["before"][0]["vhat"]
        new = r["after"][0]["vhat"]
        if r["merge"]:
            np.testing.assert_allclose(new, _mean(r["after"], "v"), rtol=2e-7)
            vs = [s["v"] for s in r["after"]]
            assert not np.array_equal(vs[0], vs[1])      # local v not overwritten
        else:
            assert np.array_equal(old, new)


def test_consensus_zero_after_merge_and_error_between_merges():
    """Right after a merge all workers hold the same model; between merges
    xbar_t - x_{t,i} = a sum_l (m_{l,i} - mbar_l) / sqrt(v_l) over the local steps since the merge
    (the consensus-error expression of the proof sketch)."""
    lr = float(F32(1e-3))
    W = 3
    _, rec = _dense_toy(W=W, k=4, T=12)
    acc = None
    for r in rec:
        if r["merge"]:
            xs = [s["x"] for s in r["after"]]
            for j in range(1, W):
                assert np.array_equal(xs[0], xs[j])
            acc = np.zeros((W,) + xs[0].shape)
            continue
        if acc is None:
            continue                                     # before the first merge models start equal too
        vhat = r["after"][0]["vhat"].astype(np.float64)
        mbar = _mean(r["after_push"], "m")
        for j in range(W):
            acc[j] += (r["after_push"][j]["m"].astype(np.float64) - mbar) / np.sqrt(vhat)
        xbar = _mean(r["after"], "x")
        for j in range(W):
            np.testing.assert_allclose(xbar - r["after"][j]["x"].astype(np.float64), lr * acc[j],
                                       rtol=1e-4, atol=2e-6)


def test_mean_of_local_v_follows_single_recursion():
    """The v line of Algorithm 2 is linear, so (1/N) sum_i v_{t,i} follows
    vbar_t = b2 vbar_{t-1} + (1 - b2) mean_i g_{t,i}^2 from vbar_0 = eps."""
    b2, eps = float(F32(0.999)), float(F32(1e-8))
    _, rec = _dense_toy(W=4, k=3, T=9)
    vbar = None
    for r in rec:
        g2 = np.mean(r["g"].astype(np.float64) ** 2, axis=0)
        vbar = b2 * (eps if vbar is None else vbar) + (1 - b2) * g2
        np.testing.assert_allclose(_mean(r["after"], "v"), vbar, rtol=5e-6)


def test_identical_workers_stay_identical_and_match_one_worker():
    """Symmetry of Algorithm 2: the same gradients on every worker give identical workers, equal
    to a one-worker run with the same k (N = 4 keeps the average exact in binary)."""
    _, rec4 = _dense_toy(W=4, k=3, T=9, same_grads=True, seed=3)
    _, rec1 = _dense_toy(W=1, k=3, T=9, same_grads=True, seed=3)
    # the generators draw (W, n, D) arrays, so compare on the state reached with the same g[0]
    for r4 in rec4:
        for j in range(1, 4):
            for f in ("x", "m", "v"):
                assert np.array_equal(r4["after"][0][f], r4["after"][j][f])
    # rerun one worker fed exactly worker 0's gradients
    t = O.OracleTable(4, 2, n_replicas=1, kstep=True, init_seed=5)
    keys = np.arange(1, 5, dtype=np.uint64)
    off = np.arange(0, 5, dtype=np.uint32)
    for r4 in rec4:
        mode = O.STEP_MERGE_PENDING if r4["merge"] else O.STEP_LOCAL
        step(t, 0, keys, off, r4["g"][0], mode)
        if r4["merge"]:
            t.kstep_merge()
        s = t.table_export()
        for f in ("x", "m", "v", "vhat"):
            assert np.array_equal(s[f], r4["after"][0][f]), (r4["step"], f)


def test_merge_step_uses_new_denominator():
    """Algorithm 2, merge branch: the k-th update divides by the freshly averaged v, which already
    holds that step's g^2; a local step divides by the value frozen at the previous merge."""
    lr = float(F32(1e-3))
    D = 1
    t = O.OracleTable(2, D, n_replicas=2, kstep=True, init_seed=1, beta1=0.0)
    keys, off, _ = one_key_batch(8, D, 0.0)
    g = [np.array([[2.0]], F32), np.array([[-1.0]], F32)]
    for j in range(2):
        step(t, j, keys, off, g[j], O.STEP_MERGE_PENDING)
    pre = [t.table_export(j) for j in range(2)]
    assert np.array_equal(pre[0]["x"], pre[1]["x"])      # pending steps have not moved x
    t.kstep_merge()
    post = t.table_export(0)
    vhat = np.mean([p["v"].astype(np.float64) for p in pre], axis=0)
    np.testing.assert_allclose(post["vhat"], vhat, rtol=2e-7)
    expect = np.mean([p["x"].astype(np.float64) - lr * p["m"].astype(np.float64) / np.sqrt(vhat)
                      for p in pre], axis=0)
    np.testing.assert_allclose(post["x"], expect, rtol=1e-6)
    # m is neither averaged nor reset
    assert np.array_equal(t.table_export(0)["m"], pre[0]["m"])
    assert np.array_equal(t.table_export(1)["m"], pre[1]["m"])


def test_merge_skips_untouched_rows_and_absent_worker_counts_as_init():
    """Sparse reading of the merge: rows nobody touched since the last merge keep their bits; a
    worker that never saw a key enters the average with the row's initial state and no step."""
    D = 2
    W = 3
    t = O.OracleTable(4, D, n_replicas=W, kstep=True, init_seed=1)
    ka, off, _ = one_key_batch(10, D, 0.0)
    kb, _, _ = one_key_batch(20, D, 0.0)
    g = np.array([[1.0, -2.0]], F32)
    step(t, 0, ka, off, g, O.STEP_MERGE_PENDING)
    step(t, 1, kb, off, g, O.STEP_MERGE_PENDING)
    t.kstep_merge()
    s0 = [t.table_export(j) for j in range(W)]
    # merge round 2 touches key 10 only, by worker 2, with a local step then a merge
    step(t, 2, ka, off, g, O.STEP_LOCAL)
    pre = [t.table_export(j) for j in range(W)]
    t.kstep_merge()
    s1 = [t.table_export(j) for j in range(W)]
    for j in range(W):
        assert np.array_equal(s0[j]["x"][1], s1[j]["x"][1])          # key 20 untouched in merge round 2
    xbar = np.mean([p["x"][0].astype(np.float64) for p in pre], axis=0)   # no pending step terms
    np.testing.assert_allclose(s1[0]["x"][0], xbar, rtol=1e-6)
    # merge round 1, key 10: workers 1 and 2 held init(key) and contributed no step
    init = np.array([O.init_value(1, 10, d, 0.01) for d in range(D)])
    v0 = (float(F32(0.999)) * 1e-8 + (1 - float(F32(0.999))) * g[0].astype(np.float64) ** 2)
    vhat = (v0 + 2 * float(F32(1e-8))) / 3
    m0 = (1 - float(F32(0.9))) * g[0].astype(np.float64)
    expect = init - float(F32(1e-3)) * m0 / np.sqrt(vhat) / 3
    np.testing.assert_allclose(s0[0]["x"][0], expect, rtol=2e-6)


# ---------------------------------------------------------------- dedup, lookup, pooling


def test_dedup_and_lookup_invariants():
    rng = np.random.default_rng(1)
    t = O.OracleTable(5000, 4, init_seed=3)
    seen = {}
    for s in range(4):
        n = 3000
        keys = (rng.zipf(1.3, n) % 4000).astype(np.uint64) * np.uint64(0x9E3779B97F4A7C15)
        off = np.sort(rng.integers(0, n + 1, 200)).astype(np.uint32)
        off[0], off[-1] = 0, n
        st, _ = t.pull_pool(0, keys, off)
        assert st == O.OK
        uniq, rows, inv = t.batch_export(n)
        assert np.all(uniq[1:] > uniq[:-1])
        assert np.array_equal(uniq[inv], keys)
        assert np.array_equal(uniq, np.unique(keys))
        assert len(set(rows.tolist())) == rows.size
        for k, r in zip(uniq.tolist(), rows.tolist()):
            assert seen.setdefault(k, r) == r            # same row for the table's lifetime
            assert t.lookup(k) == r
        assert t.n_rows == len(seen)
        # first-occurrence order of the new keys
        n_before = t.n_rows - t.n_new_last
        first = {}
        for p, k in enumerate(keys.tolist()):
            first.setdefault(k, p)
        new = sorted((k for k in first if seen[k] >= n_before), key=lambda k: first[k])
        assert [seen[k] for k in new] == list(range(n_before, t.n_rows))
        # a second pull of the same batch inserts nothing
        st, _ = t.pull_pool(0, keys, off)
        assert st == O.OK and t.n_new_last == 0 and t.n_rows == len(seen)


def test_pooling_brute_force_exact():
    """Tiny inputs, nested loops over a dict, exact rational sums."""
    rng = np.random.default_rng(2)
    for trial in range(20):
        B, S, D = rng.integers(1, 5), rng.integers(1, 4), int(rng.choice([1, 2, 4]))
        G = B * S
        counts = rng.integers(0, 4, G)
        off = np.concatenate([[0], np.cumsum(counts)]).astype(np.uint32)
        keys = rng.integers(1, 7, off[-1]).astype(np.uint64)
        t = O.OracleTable(8, D, init_seed=trial, init_std=1.0)
        st, pooled = t.pull_pool(0, keys, off)
        assert st == O.OK
        s = t.table_export()
        row = {int(k): i for i, k in enumerate(s["keys"])}
        total = [Fraction(0)] * D
        for g in range(G):
            for d in range(D):
                acc = Fraction(0)
                for p in range(off[g], off[g + 1]):
                    acc += Fraction(float(s["x"][row[int(keys[p])], d]))
                assert pooled[g, d] == F32(float(acc)), (trial, g, d)
                total[d] += acc
            if counts[g] == 1:
                assert np.array_equal(pooled[g], s["x"][row[int(keys[off[g]])]])
            if counts[g] == 0:
                assert np.all(pooled[g] == 0)
        # sum over segments == sum over distinct keys of count * row
        cnt = {}
        for k in keys.tolist():
            cnt[k] = cnt.get(k, 0) + 1
        for d in range(D):
            rhs = sum(Fraction(c) * Fraction(float(s["x"][row[k], d])) for k, c in cnt.items())
            assert rhs == total[d]


def _brute_cycle(R, D, W, kstep, hp, seed, init_std, script):
    """Independent restatement with dicts and exact sums; script = list of
    ("step", replica, keys, off, grad, mode) and ("merge",)."""
    lr, b1, b2, eps = (float(F32(h)) for h in hp)
    row, X, M, V, VH = {}, [], [], [], []
    pend, touched = [set() for _ in range(W)], set()
    for op in script:
        if op[0] == "merge":
            for r in sorted(touched):
                vh = np.array([F32(float(sum(Fraction(float(V[r][j][d])) for j in range(W)) / W))
                               for d in range(D)], F32)
                VH[r] = vh
                xb = []
                for d in range(D):
                    acc = 0.0
                    for j in range(W):
                        y = float(X[r][j][d])
                        if r in pend[j]:
                            y -= lr * float(M[r][j][d]) / np.sqrt(float(vh[d]))
                        acc += y
                    xb.append(F32(acc / W))
                for j in range(W):
                    X[r][j] = np.array(xb, F32)
            touched.clear()
            for p in pend:
                p.clear()
            continue
        _, j, keys, off, grad, mode = op
        for k in keys.tolist():
            if k not in row:
                row[k] = len(row)
                x0 = np.array([O.init_value(seed, k, d, init_std) for d in range(D)], F32)
                X.append([x0.copy() for _ in range(W)])
                M.append([np.zeros(D, F32) for _ in range(W)])
                V.append([np.full(D, eps, F32) for _ in range(W)])
                VH.append(np.full(D, eps, F32))
        gs = {}
        for g in range(len(off) - 1):
            for p in range(off[g], off[g + 1]):
                acc = gs.setdefault(int(keys[p]), [Fraction(0)] * D)
                for d in range(D):
                    acc[d] += Fraction(float(grad[g, d]))
        for k, acc in gs.items():
            r = row[k]
            for d in range(D):
                g = float(acc[d])
                M[r][j][d] = F32(b1 * float(M[r][j][d]) + (1 - b1) * g)
                V[r][j][d] = F32(b2 * float(V[r][j][d]) + (1 - b2) * (g * g))
                if not kstep:
                    X[r][j][d] = F32(float(X[r][j][d]) - lr * float(M[r][j][d]) / np.sqrt(float(V[r][j][d])))
                elif mode == O.STEP_LOCAL:
                    X[r][j][d] = F32(float(X[r][j][d]) - lr * float(M[r][j][d]) / np.sqrt(float(VH[r][d])))
            if kstep:
                touched.add(r)
                if mode == O.STEP_MERGE_PENDING:
                    pend[j].add(r)
    return row, X, M, V, VH


@pytest.mark.parametrize("W,kstep", [(1, False), (1, True), (3, True)])
def test_full_cycle_brute_force(W, kstep):
    rng = np.random.default_rng(10 + W)
    R, D, k = 16, 2, 2
    hp = (1e-3, 0.9, 0.999, 1e-8)
    t = O.OracleTable(R, D, n_replicas=W, kstep=kstep, init_seed=77, init_std=0.01)
    script = []
    for s in range(1, 7):
        mode = O.STEP_MERGE_PENDING if (kstep and s % k == 0) else O.STEP_LOCAL
        for j in range(W):
            G = int(rng.integers(1, 5))
            counts = rng.integers(0, 4, G)
            off = np.concatenate([[0], np.cumsum(counts)]).astype(np.uint32)
            keys = rng.integers(1, 12, off[-1]).astype(np.uint64)
            grad = rng.standard_normal((G, D)).astype(F32)
            script.append(("step", j, keys, off, grad, mode))
            step(t, j, keys, off, grad, mode)
        if kstep and s % k == 0:
            script.append(("merge",))
            assert t.kstep_merge() == O.OK
    row, X, M, V, VH = _brute_cycle(R, D, W, kstep, hp, 77, 0.01, script)
    for j in range(W):
        s = t.table_export(j)
        assert {int(k): i for i, k in enumerate(s["keys"])} == row
        for r in range(len(row)):
            np.testing.assert_allclose(s["x"][r], X[r][j], rtol=3e-7, atol=0)
            np.testing.assert_allclose(s["m"][r], M[r][j], rtol=3e-7, atol=1e-12)
            np.testing.assert_allclose(s["v"][r], V[r][j], rtol=3e-7, atol=0)
            if kstep:
                np.testing.assert_allclose(s["vhat"][r], VH[r], rtol=3e-7, atol=0)


# ---------------------------------------------------------------- error conventions


def test_capacity_edge_and_sentinel():
    D = 2
    t = O.OracleTable(4, D, init_seed=1)
    off = np.array([0, 4], np.uint32)
    st, _ = t.pull_pool(0, np.array([1, 2, 3, 4], np.uint64), off)
    assert st == O.OK and t.n_rows == 4                  # exactly R distinct keys fit
    assert t.push_adam(0, np.ones((1, D), F32)) == O.OK
    before = t.table_export()
    st, _ = t.pull_pool(0, np.array([1, 2, 9, 4], np.uint64), off)
    assert st == O.E_FULL and t.n_rows == 4 and t.lookup(9) == -1
    st, _ = t.pull_pool(0, np.array([1, 2, 2 ** 64 - 1, 4], np.uint64), off)
    assert st == O.E_BADKEY
    st, _ = t.pull_pool(0, np.array([1, 2, 3, 4], np.uint64), np.array([0, 3], np.uint32))
    assert st == O.E_INVAL
    st, _ = t.pull_pool(0, np.array([1, 2, 3, 4], np.uint64), np.array([0, 3, 2, 4], np.uint32))
    assert st == O.E_INVAL
    after = t.table_export()
    for f in ("keys", "x", "m", "v"):
        assert np.array_equal(before[f], after[f])
    assert t.push_adam(0, np.ones((1, D), F32)) == O.E_STATE      # failed pulls leave no batch
    st, _ = t.pull_pool(1, np.array([1], np.uint64), np.array([0, 1], np.uint32))
    assert st == O.E_INVAL                                         # replica out of range


def test_push_needs_matching_pull():
    D = 2
    t = O.OracleTable(4, D, n_replicas=2, kstep=True)
    keys, off, g = one_key_batch(3, D, 1.0)
    assert t.push_adam(0, g) == O.E_STATE
    st, _ = t.pull_pool(0, keys, off)
    assert t.push_adam(1, g) == O.E_STATE
    assert t.push_adam(0, g, 7) == O.E_INVAL
    assert t.push_adam(0, g) == O.OK
    assert t.push_adam(0, g) == O.E_STATE                # a batch is consumed by its push
    t1 = O.OracleTable(4, D)
    st, _ = t1.pull_pool(0, keys, off)
    assert t1.push_adam(0, g, O.STEP_MERGE_PENDING) == O.E_INVAL   # single-table mode has no merge
    assert t1.kstep_merge() == O.E_INVAL
