"""GPU parity at the full size of the benchmarked configuration (2^24-row table, dim 64, batch
32768 x 300 slots, ~39 M key occurrences), in the launch configuration bench.py times.

The oracle runs the same two steps on the host (about half a minute each); the final table is
compared element by element; the pooled outputs of the first step on EVERY segment (the tolerance of a
segment needs its rows: built chunk by chunk), those of the second step on a sample of segments.
"""
import time

import numpy as np
import pytest

from oracle import ctr_oracle as O
from paper_2201_05500_amd import workloads as WL
from tests.parity_util import ATOL, RTOL

pytestmark = pytest.mark.gpu


def _say(capsys, *a):
    """Progress line that reaches the terminal even under output capture (these tests run for minutes)."""
    with capsys.disabled():
        print("[full size %s]" % time.strftime("%H:%M:%S"), *a, flush=True)


def _close_chunked(g, o, what, chunk=1 << 18):
    assert g.shape == o.shape, what
    for i in range(0, g.shape[0], chunk):
        a = g[i:i + chunk].astype(np.float64)
        b = o[i:i + chunk].astype(np.float64)
        bad = np.abs(a - b) > ATOL + RTOL * np.abs(b)
        if bad.any():
            j = np.argwhere(bad)[0]
            raise AssertionError("%s: %d outside tolerance in rows %d..; first at row %d col %d gpu=%r ref=%r" % (
                what, int(bad.sum()), i, i + j[0], j[1], a[tuple(j)], b[tuple(j)]))


def _all_pooled_close(pooled, opooled, ox, orow, oi, off, n_seg, say, chunk=1 << 18):
    """Every pooled segment against the oracle's, each with the parameter tolerance summed over its own rows."""
    D = ox.shape[1]
    for g0 in range(0, n_seg, chunk):
        g1 = min(g0 + chunk, n_seg)
        p0, p1 = int(off[g0]), int(off[g1])
        per_occ = ATOL + RTOL * np.abs(ox[orow[oi[p0:p1]]].astype(np.float64))
        c = np.concatenate([np.zeros((1, D)), np.cumsum(per_occ, axis=0)])
        rel = off[g0:g1 + 1] - p0
        tol = np.maximum(c[rel[1:]] - c[rel[:-1]], ATOL)
        gp = pooled[g0:g1].cpu().numpy().astype(np.float64)
        bad = np.abs(gp - opooled[g0:g1]) > tol
        if bad.any():
            j = np.argwhere(bad)[0]
            raise AssertionError("pooled: %d outside tolerance in segments %d..%d; first at segment %d col %d" % (
                int(bad.sum()), g0, g1, g0 + j[0], j[1]))
        if (g0 // chunk) % 8 == 0:
            say("pooled segments %d..%d of %d compared" % (g0, g1, n_seg))


@pytest.mark.timeout(1200)
def test_large_config_two_steps_full_table(capsys):
    import torch
    from paper_2201_05500_amd.binding import CTR_OK, CtrTable
    w = WL.WORKLOADS["large"]
    gt = CtrTable(w.capacity_rows, w.dim, lr=w.lr, beta1=w.beta1, beta2=w.beta2, eps=w.eps, init_seed=1,
                  init_std=w.init_std, load_factor=w.load_factor)
    ot = O.OracleTable(w.capacity_rows, w.dim, lr=w.lr, beta1=w.beta1, beta2=w.beta2, eps=w.eps,
                       init_seed=1, init_std=w.init_std)
    rng = np.random.default_rng(0)
    for step in range(2):
        bt = WL.make_batch(w, step, device="cuda:0")
        bn = WL.as_numpy(bt)
        L = bn["keys"].size
        _say(capsys, "step", step, "L", L)
        st, gb, pooled = gt.pull_pool(0, bt["keys"], bt["offsets"])
        assert st == CTR_OK and gt.last_status() == CTR_OK
        ost, opooled = ot.pull_pool(0, bn["keys"], bn["offsets"])
        assert ost == 0
        _say(capsys, "oracle pull done")
        # dedup result, bit-exact
        gu, gr, gi = gt.batch_export(gb, L)
        ou, orow, oi = ot.batch_export(L)
        assert np.array_equal(gu, ou) and np.array_equal(gr, orow) and np.array_equal(gi, oi)
        # pooled: bound = parameter tolerance summed over the segment's rows.  Step 0: EVERY segment (the
        # bound is built chunk by chunk); step 1: a sample of segments
        ox = ot.table_export(0)["x"]
        off = bn["offsets"].astype(np.int64)
        if step == 0:
            _all_pooled_close(pooled, opooled, ox, orow, oi, off, w.n_segments, lambda m: _say(capsys, m))
        else:
            segs = rng.integers(0, w.n_segments, 20000)
            gp = pooled[torch.from_numpy(segs).to("cuda:0")].cpu().numpy().astype(np.float64)
            for n, g in enumerate(segs):
                rows = orow[oi[off[g]:off[g + 1]]]
                tol = np.maximum((ATOL + RTOL * np.abs(ox[rows].astype(np.float64))).sum(axis=0), ATOL)
                assert np.all(np.abs(gp[n] - opooled[g]) <= tol), ("pooled", step, g)
        del ox, gu, gr, gi, ou, oi
        assert gt.push_adam(0, gb, bt["grad"]) == CTR_OK
        assert ot.push_adam(0, bn["grad"]) == 0
        u, n_new = gt.batch_stats()
        assert u == orow.size and n_new == ot.n_new_last
        _say(capsys, "oracle push done")
        del bt, bn, pooled, opooled
    assert gt.last_status() == CTR_OK and gt.n_rows == ot.n_rows
    g, o = gt.table_export(0), ot.table_export(0)
    assert np.array_equal(g["keys"], o["keys"])
    for f in ("x", "m", "v"):
        _close_chunked(g[f], o[f], "large config, " + f)


@pytest.mark.timeout(1200)
@pytest.mark.parametrize("grad_bf16", [False, True])
def test_full_step_config_one_step(capsys, grad_bf16):
    """The whole training step at the size bench.py --workload full times: batch 16384 x 300 slots into the
    2^24-row table, tower 19200-1024-512-256-1.  The tower is compared with its oracle on the very pooled
    input the GPU produced; the table with the table oracle fed the very gradient the GPU tower produced.
    grad_bf16: the tower hands the gradient of the pooled input to the push as bf16 (bench.py --grad-bf16)."""
    import torch
    from oracle import mlp_oracle as M
    from paper_2201_05500_amd.binding import CTR_OK, CtrTable
    from paper_2201_05500_amd.binding_mlp import CtrMlp
    from tests.test_gpu_mlp import close_enough, close_rows
    w = WL.WORKLOADS["full"]
    in_dim = w.slots * w.dim
    gt = CtrTable(w.capacity_rows, w.dim, lr=w.lr, beta1=w.beta1, beta2=w.beta2, eps=w.eps, init_seed=1,
                  init_std=w.init_std, load_factor=w.load_factor)
    ot = O.OracleTable(w.capacity_rows, w.dim, lr=w.lr, beta1=w.beta1, beta2=w.beta2, eps=w.eps,
                       init_seed=1, init_std=w.init_std)
    gm = CtrMlp(in_dim, WL.FULL_STEP_HIDDEN, lr=w.lr, beta1=w.beta1, beta2=w.beta2, eps=w.eps, init_seed=3)
    om = M.MlpOracle(in_dim, WL.FULL_STEP_HIDDEN, lr=w.lr, beta1=w.beta1, beta2=w.beta2, eps=w.eps, init_seed=3)
    bt = WL.make_batch(w, 0, device="cuda:0", with_grad=False)
    labels = WL.make_labels(w, 0, device="cuda:0")
    bn = WL.as_numpy(bt)
    L = bn["keys"].size
    _say(capsys, "full step, L", L, "(bf16 gradient hand-over)" if grad_bf16 else "")

    st, gb, pooled16, pooled = gt.pull_pool_bf16(0, bt["keys"], bt["offsets"], want_f32=True)
    assert st == CTR_OK and gt.last_status() == CTR_OK
    assert torch.equal(pooled16, pooled.to(torch.bfloat16))
    g16 = torch.empty((w.batch, in_dim), dtype=torch.bfloat16, device="cuda:0") if grad_bf16 else None
    st, loss, gp = gm.step(0, pooled16.view(w.batch, in_dim), labels, grad_pooled=g16)
    assert st == CTR_OK and gp.dtype == (torch.bfloat16 if grad_bf16 else torch.float32)
    assert gt.push_adam(0, gb, gp.view(w.n_segments, w.dim)) == CTR_OK
    assert gt.last_status() == CTR_OK
    _say(capsys, "GPU step done, loss", float(loss.cpu()[0]))

    ost, opooled = ot.pull_pool(0, bn["keys"], bn["offsets"])
    assert ost == 0
    _say(capsys, "oracle pull done")
    _, orow, oi = ot.batch_export(L)
    ox = ot.table_export(0)["x"]
    rng = np.random.default_rng(5)
    segs = rng.integers(0, w.n_segments, 20000)
    gsel = pooled[torch.from_numpy(segs).to("cuda:0")].cpu().numpy().astype(np.float64)
    off = bn["offsets"].astype(np.int64)
    for n, g in enumerate(segs):
        rows = orow[oi[off[g]:off[g + 1]]]
        tol = np.maximum((ATOL + RTOL * np.abs(ox[rows].astype(np.float64))).sum(axis=0), ATOL)
        assert np.all(np.abs(gsel[n] - opooled[g]) <= tol), ("pooled", g)
    del ox, opooled, gsel, oi

    pooled_h = pooled.cpu().numpy().reshape(w.batch, in_dim)
    del pooled, pooled16
    oloss, ogp = om.step(0, pooled_h, labels.cpu().numpy(), grad_bf16=grad_bf16)
    _say(capsys, "oracle tower done, loss", float(oloss))
    assert abs(float(loss.cpu()[0]) - float(oloss)) <= 1e-4 * max(1.0, float(oloss))
    gp_h = gp.to(torch.float32).cpu().numpy()                           # widening a bf16 value is exact
    from tests.test_gpu_mlp import OBSERVED
    n_round, n_mask = close_rows(gp_h, ogp, "gradient of the pooled input", in_dim)
    _say(capsys, "gradient rows with rounding cascades:", n_round, "with a flipped mask:", n_mask, "of", w.batch,
         "| worst row error %.3g, norm-wise error of the other rows %.3g" % OBSERVED["gradient of the pooled input"][2:4])
    e = gm.export()
    close_enough(e["params"], om.params[0], "tower parameters", rtol=1e-3, norm_tol=1e-3)
    close_enough(e["m"], om.m[0], "tower first moment")
    del ogp, pooled_h

    assert ot.push_adam(0, gp_h.reshape(w.n_segments, w.dim)) == 0       # the GPU tower's gradient
    _say(capsys, "oracle push done")
    u, n_new = gt.batch_stats()
    assert u == orow.size and n_new == ot.n_new_last and gt.n_rows == ot.n_rows
    g, o = gt.table_export(0), ot.table_export(0)
    assert np.array_equal(g["keys"], o["keys"])
    for f in ("x", "m", "v"):
        _close_chunked(g[f], o[f], "full step, table " + f)


@pytest.mark.timeout(900)
def test_mid_config_full_size(capsys):
    """Configuration 2 as benchmarked (2^22 x 16 table, 8192 x 100 slots, ~2.5 M occurrences per batch):
    all 20 steps of the configuration, every output compared after every step."""
    from tests.test_gpu_parity import run_workload
    w = WL.WORKLOADS["mid"]
    assert w.steps == 20
    _say(capsys, "mid config, %d steps" % w.steps)
    gt, ot = run_workload(w, w.steps, say=lambda m: _say(capsys, m))
    assert gt.n_rows == ot.n_rows


@pytest.mark.timeout(1200)
def test_kstep_config_full_size(capsys):
    """Configuration 4 as benchmarked (W = 8 replicas, k = 4, 2^22 x 16 table, 4096 x 100 slots per replica
    step): three of the configuration's ten merge rounds (each: 3 local steps, the merge step, the merge), every
    replica step and the tables before and after every merge compared.  (The oracle needs about 40 s per round:
    all ten would take most of the time the whole GPU suite has.)"""
    from tests.test_gpu_parity import _kstep_rounds
    _say(capsys, "k-step config, three merge rounds of 8 replicas")
    gt, ot = _kstep_rounds(WL.WORKLOADS["kstep"], 3, 4, say=lambda m: _say(capsys, m))
    assert gt.n_rows == ot.n_rows


@pytest.mark.timeout(900)
def test_maximum_batch_size_closed_form(capsys):
    """The largest batch one call accepts (just under 2^31 key occurrences; 2^25 - 1 segments of 64 keys) against
    closed forms: keys cycle through 1..K, so every count, every pooled sum and the one Adam step are known
    without running the oracle's loop over 2 G occurrences.  Exercises 32-bit index arithmetic near its limit,
    a pull in which every occurrence is pending, rows whose occurrences span 16 K work spans."""
    import torch
    from paper_2201_05500_amd.binding import CTR_OK, CtrTable
    free, _ = torch.cuda.mem_get_info()
    if free < 140 << 30:
        pytest.skip("needs 140 GiB of free device memory")
    K, D, S = 1000, 4, 64
    G = (1 << 25) - 1
    n = G * S                                                   # 2^31 - 64
    lr, b1, b2, eps, std, seed = 1e-3, 0.9, 0.999, 1e-8, 0.01, 9
    gt = CtrTable(1 << 16, D, lr=lr, beta1=b1, beta2=b2, eps=eps, init_seed=seed, init_std=std)
    dev = "cuda:0"
    keys = torch.arange(n, dtype=torch.int64, device=dev)
    keys.remainder_(K).add_(1)
    offs = (torch.arange(G + 1, dtype=torch.int64, device=dev) * S).to(torch.int32)
    _say(capsys, "max batch: n =", n, "G =", G)
    st, gb, pooled = gt.pull_pool(0, keys, offs)
    assert st == CTR_OK and gt.last_status() == CTR_OK
    assert gt.n_rows == K
    _say(capsys, "pull done")
    init = np.array([[O.init_value(seed, k, d, std) for d in range(D)] for k in range(1, K + 1)], np.float32)
    # segment g holds keys ((64 g + j) mod K) + 1, j < 64: sums over a cyclic window of the init table
    c = np.concatenate([np.zeros((1, D)), np.cumsum(np.concatenate([init, init]).astype(np.float64), axis=0)])
    rng = np.random.default_rng(1)
    segs = np.concatenate([[0, 1, G - 1], rng.integers(0, G, 50000)])
    start = (segs * S) % K
    want = c[start + S] - c[start]
    got = pooled[torch.from_numpy(segs).to(dev)].cpu().numpy().astype(np.float64)
    tol = S * (ATOL + RTOL * np.abs(init).max())
    assert np.all(np.abs(got - want) <= tol), "pooled"
    del pooled
    grad = torch.ones((G, D), dtype=torch.float32, device=dev)
    assert gt.push_adam(0, gb, grad) == CTR_OK
    assert gt.last_status() == CTR_OK
    u, n_new = gt.batch_stats()
    assert u == K and n_new == K
    _say(capsys, "push done")
    e = gt.table_export(0)
    assert np.array_equal(e["keys"], np.arange(1, K + 1, dtype=np.uint64))      # rows in order of first occurrence
    cnt = ((n + K - 1 - np.arange(K)) // K).astype(np.float64)                   # occurrences of key k + 1
    assert cnt.sum() == n
    g = cnt[:, None] * np.ones((1, D))
    m = (1 - np.float64(np.float32(b1))) * g
    v = np.float64(np.float32(b2)) * np.float64(np.float32(eps)) + (1 - np.float64(np.float32(b2))) * g * g
    m32, v32 = m.astype(np.float32), v.astype(np.float32)
    x = init.astype(np.float64) - np.float64(np.float32(lr)) * m32.astype(np.float64) / np.sqrt(v32.astype(np.float64))
    for name, got_a, want_a in (("m", e["m"], m), ("v", e["v"], v), ("x", e["x"], x)):
        assert np.all(np.abs(got_a.astype(np.float64) - want_a) <= ATOL + RTOL * np.abs(want_a)), name


@pytest.mark.timeout(900)
def test_maximum_capacity_closed_form(capsys):
    """The largest table the build accepts (2^29 rows at the default load factor: 2^30 index slots; dim 4) filled to the last row by ONE
    batch of 2^29 distinct keys, then one Adam step on every row, checked on sampled keys against closed forms;
    one more new key must then be refused without side effects.  Exercises 64-bit offsets into the row storage."""
    import torch
    from paper_2201_05500_amd.binding import CTR_E_FULL, CTR_OK, CtrTable
    free, _ = torch.cuda.mem_get_info()
    if free < 100 << 30:
        pytest.skip("needs 100 GiB of free device memory")
    R, D, S = 1 << 29, 4, 64
    G = R // S
    lr, b1, b2, eps, std, seed = 1e-3, 0.9, 0.999, 1e-8, 0.01, 4
    dev = "cuda:0"
    gt = CtrTable(R, D, lr=lr, beta1=b1, beta2=b2, eps=eps, init_seed=seed, init_std=std)
    keys = torch.arange(1, R + 1, dtype=torch.int64, device=dev)
    offs = (torch.arange(G + 1, dtype=torch.int64, device=dev) * S).to(torch.int32)
    _say(capsys, "max capacity: R =", R)
    st, gb, pooled = gt.pull_pool(0, keys, offs)
    assert st == CTR_OK and gt.last_status() == CTR_OK
    assert gt.n_rows == R
    _say(capsys, "pull done, table full")
    rng = np.random.default_rng(2)
    segs = np.concatenate([[0, G - 1], rng.integers(0, G, 300)])
    got = pooled[torch.from_numpy(segs).to(dev)].cpu().numpy().astype(np.float64)
    for i, g in enumerate(segs):
        want = np.sum([[np.float64(O.init_value(seed, int(g) * S + j + 1, d, std)) for d in range(D)] for j in range(S)],
                      axis=0)
        assert np.all(np.abs(got[i] - want) <= S * (ATOL + RTOL * 0.1)), ("pooled", g)
    del pooled
    grad = torch.ones((G, D), dtype=torch.float32, device=dev)
    assert gt.push_adam(0, gb, grad) == CTR_OK and gt.last_status() == CTR_OK
    u, n_new = gt.batch_stats()
    assert u == R and n_new == R
    _say(capsys, "push done")
    sample = np.concatenate([[1, 2, R - 1, R], rng.integers(1, R + 1, 2000)]).astype(np.int64)
    st, x, m, v, found = gt.table_collect(0, torch.from_numpy(sample).to(dev))
    assert st == CTR_OK and bool(found.all())
    init = np.array([[O.init_value(seed, int(k), d, std) for d in range(D)] for k in sample], np.float32)
    m_w = 1 - np.float64(np.float32(b1))
    v_w = np.float64(np.float32(b2)) * np.float64(np.float32(eps)) + (1 - np.float64(np.float32(b2)))
    x_w = init.astype(np.float64) - np.float64(np.float32(lr)) * np.float64(np.float32(m_w)) / np.sqrt(np.float64(np.float32(v_w)))
    for name, got_a, want_a in (("m", m, np.full_like(x_w, m_w)), ("v", v, np.full_like(x_w, v_w)), ("x", x, x_w)):
        ga = got_a.cpu().numpy().astype(np.float64)
        assert np.all(np.abs(ga - want_a) <= ATOL + RTOL * np.abs(want_a)), name
    # one key too many: refused, nothing changes
    extra = torch.tensor([R + 5], dtype=torch.int64, device=dev)
    st, _, _ = gt.pull_pool(0, extra, torch.tensor([0, 1], dtype=torch.int32, device=dev))
    assert st == CTR_OK and gt.last_status() == CTR_E_FULL and gt.n_rows == R
    st, _, _, _, found = gt.table_collect(0, extra)
    assert st == CTR_OK and int(found[0]) == 0
    st, x2, _, _, found = gt.table_collect(0, torch.from_numpy(sample[:8]).to(dev))
    assert bool(found.all()) and torch.equal(x2, x[:8])


@pytest.mark.timeout(900)
def test_batch_of_five_million_occurrences(capsys):
    """A batch size between the benchmarked ones (4096 x 300 slots, ~4.9 M occurrences into a 2^22-row table):
    the host picks work spans of 64 occurrences and 8 probes per thread here, a combination no other test runs."""
    from tests.test_gpu_parity import run_workload
    w = WL.scaled(WL.WORKLOADS["large"], capacity_rows=1 << 22, zipf_universe=1 << 22, batch=4096)
    gt, ot = run_workload(w, 2, say=lambda m: _say(capsys, m))
    assert gt.n_rows == ot.n_rows
