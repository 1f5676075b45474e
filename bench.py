#!/usr/bin/env python3
"""Benchmark of the sparse embedding cycle on one MI355X.

A step is one pass of the whole hot path over one synthetic mini-batch: ctr_pull_pool (probe with
insert-on-miss, row gather + per-slot sum, grouping of occurrences by row) followed by
ctr_push_adam (gradient segment-reduce fused with sparse Adam).  All inputs of all steps are
generated on the device before the timed region starts.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload large|mid|tiny|kstep|full]

With --workload full a step is the whole training step of Algorithm 1: pull, the dense tower
(forward, loss, backward, dense Adam) on the pooled embeddings, push of the tower's gradient.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X published HBM3E bandwidth
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X published dense bf16 matrix-core rate

KERNEL_OF_STAGE = {"push": "k_push_span", "pool": "k_pool", "merge": "k_merge"}


def measured_traffic(workload):
    """HBM traffic per launch from the rocprofv3 FETCH_SIZE / WRITE_SIZE runs whose figures are committed as
    profiles/<workload>_step_traffic.json (written by paper_2201_05500_amd/profile_summary.py from the counter
    output, each counter scaled by what it reads for a copy of known size in the same run).  Returns
    (per-kernel bytes, whole-step bytes, provenance) or ({}, None, None) when there is no such file.  The
    provenance says at which commit and source hash the counters were taken and whether the sources the
    library was built from still hash the same."""
    path = os.path.join(ROOT, "profiles", "%s_step_traffic.json" % workload)
    if not os.path.exists(path):
        return {}, None, None
    from paper_2201_05500_amd.build import source_hash
    with open(path) as f:
        rec = json.load(f)
    fs, wsf = rec["scale"]["fetch"], rec["scale"]["write"]
    per = {k: v["fetch_KiB"] * 1024 * fs + v["write_KiB"] * 1024 * wsf for k, v in rec["kernels"].items()}
    step = rec["step"]["fetch_KiB"] * 1024 * fs + rec["step"]["write_KiB"] * 1024 * wsf
    prov = {"file": "profiles/%s_step_traffic.json" % workload, "commit": rec.get("commit"),
            "source_hash": rec.get("source_hash"), "matches_current_sources": rec.get("source_hash") == source_hash()}
    return per, step, prov


def algorithmic_bytes_step(L, G, U, n_new, D, kstep, n_state=3, grad_bytes=4):
    """Bytes one step must move (no sort scratch, no re-reads of hot rows)."""
    b = 8 * L                   # keys read
    b += 2 * 4 * (G + 1)        # offsets read by pull and by push-side bookkeeping
    b += 2 * 8 * U              # distinct set written and read
    b += 3 * 4 * L              # occurrence -> distinct map written, read by pool, read by push
    b += 16 * U + 16 * n_new    # index probe (key + row id) per distinct key, plus inserts
    b += 4 * D * U              # compulsory row reads for pooling
    b += 4 * D * G              # pooled write
    b += grad_bytes * D * G     # pooled-gradient read
    b += 2 * n_state * 4 * D * U  # optimizer: read + write x, m, v (x, G for AdaGrad)
    if kstep:
        b += 4 * D * U          # shared denominator read
    return b


def algorithmic_bytes_push_kernel(L, G, U, D, kstep, n_state=3, grad_bytes=4):
    """The push kernel's share: occurrence map read, pooled-gradient read, row state read + write."""
    return 4 * L + grad_bytes * D * G + 2 * n_state * 4 * D * U + (4 * D * U if kstep else 0)


def algorithmic_bytes_pool_kernel(L, G, U, D, out_bytes=4):
    """The pool kernel's share: offsets and occurrence map read, compulsory row reads, pooled write."""
    return 4 * (G + 1) + 4 * L + 4 * D * U + out_bytes * D * G


def algorithmic_bytes_merge_kernel(rows_merged, pending_pairs, n_rows, D, W, shared_den):
    """One k-step merge: the state word of every row in use; per merged row the second moment and the model of
    every replica read, the model of every replica written, the shared denominator written (Algorithm 2 as
    printed) or every replica's second moment written (prose reading); the first moment of the (row, replica)
    pairs whose last step is applied inside the merge."""
    per_row = (2 * W + W + (1 if shared_den else W)) * 4 * D
    return 4 * n_rows + rows_merged * per_row + pending_pairs * 4 * D


def copy_ceiling(torch, dev, nbytes=1 << 30, reps=5):
    """GB/s (read + write) of the library's streaming copy kernel on nbytes, best of the plain and the
    non-temporal form: the practical rate of this GPU's memory system, measured in this run."""
    from paper_2201_05500_amd.binding import CTR_OK, ctr_stream_copy
    src = torch.ones(nbytes // 4, dtype=torch.float32, device=dev)
    dst = torch.empty_like(src)
    stream = int(torch.cuda.current_stream(dev).cuda_stream)
    best, which = 0.0, None
    for nt in (0, 1):
        for r in range(reps + 1):                                  # the first one warms up
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            if ctr_stream_copy(dst.data_ptr(), src.data_ptr(), nbytes, nt, stream) != CTR_OK:
                raise RuntimeError("ctr_stream_copy failed")
            e1.record()
            torch.cuda.synchronize()
            rate = 2 * nbytes / (e0.elapsed_time(e1) * 1e-3) / 1e9
            if r and rate > best:
                best, which = rate, "non-temporal" if nt else "plain"
    if not bool((dst[:: 1 << 16] == 1).all()):
        raise RuntimeError("ctr_stream_copy copied wrongly")
    del src, dst
    return best, which


def tower_flops(batch, in_dim, hidden):
    """Multiply-adds x 2 of one tower step: every layer's forward product, weight-gradient product
    and input-gradient product (the first layer's input gradient is the push's input)."""
    dims = [in_dim] + list(hidden) + [1]
    return 3 * 2 * batch * sum(dims[i] * dims[i + 1] for i in range(len(dims) - 1))


def cpu_baseline_full(w, WL, seconds_hint=20.0):
    """Table oracle (one thread) and tower oracle (numpy, the BLAS's threads) chained on a bounded sample."""
    import numpy as np
    from oracle import ctr_oracle as O
    from oracle import mlp_oracle as M
    ws = WL.scaled(w, batch=max(8, w.batch // 16))
    in_dim = ws.slots * ws.dim
    ot = O.OracleTable(ws.capacity_rows, ws.dim, n_replicas=1, lr=ws.lr, beta1=ws.beta1, beta2=ws.beta2,
                       eps=ws.eps, init_seed=1, init_std=ws.init_std)
    om = M.MlpOracle(in_dim, WL.FULL_STEP_HIDDEN, lr=ws.lr, beta1=ws.beta1, beta2=ws.beta2, eps=ws.eps, init_seed=3)
    try:
        from threadpoolctl import threadpool_info
        threads = max([int(i.get("num_threads", 1)) for i in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    n_steps, keys_done, t_spent = 0, 0, 0.0
    while t_spent < seconds_hint / 2 and n_steps < 4:
        bn = WL.as_numpy(WL.make_batch(ws, n_steps % w.steps, with_grad=False))
        labels = WL.make_labels(ws, n_steps % w.steps).numpy()
        t0 = time.perf_counter()
        st, pooled = ot.pull_pool(0, bn["keys"], bn["offsets"])
        assert st == 0
        _, gp = om.step(0, np.asarray(pooled, np.float32).reshape(ws.batch, in_dim), labels)
        assert ot.push_adam(0, gp.reshape(ws.n_segments, ws.dim)) == 0
        t_spent += time.perf_counter() - t0
        keys_done += bn["keys"].size
        n_steps += 1
    ot.close()
    return {
        "value": keys_done / t_spent, "unit": "keys/s", "cores": threads, "kind": "oracle",
        "sample": "%d full step(s) (table oracle on one thread, tower oracle in numpy float64 on %d BLAS threads) of "
                  "the first %d of %d samples per batch (%d key occurrences), table starting empty, %.1f s" % (
                      n_steps, threads, ws.batch, w.batch, keys_done, t_spent),
    }


def cpu_baseline(w, WL, seconds_hint=20.0):
    """The oracle as it stands, one thread, on a bounded sample of the same workload."""
    from oracle import ctr_oracle as O
    if w.name == "full":
        return cpu_baseline_full(w, WL, seconds_hint)
    frac = {"large": 8, "mid": 1, "tiny": 1, "kstep": 1}.get(w.name, 1)
    ws = WL.scaled(w, batch=max(1, w.batch // frac))
    ot = O.OracleTable(ws.capacity_rows, ws.dim, n_replicas=1, lr=ws.lr, beta1=ws.beta1, beta2=ws.beta2,
                       eps=ws.eps, init_seed=1, init_std=ws.init_std)
    # two untimed steps first, so that the timed ones are not dominated by the inserts of an empty table
    n_warm, n_steps, keys_done, t_spent, t_warm = 2, 0, 0, 0.0, 0.0
    for step in range(n_warm + 3):
        if step >= n_warm and t_spent >= seconds_hint / 2:
            break
        bn = WL.as_numpy(WL.make_batch(ws, step % w.steps))   # the configuration's own distinct batches, then repeated
        t0 = time.perf_counter()
        st, _ = ot.pull_pool(0, bn["keys"], bn["offsets"])
        assert st == 0
        assert ot.push_adam(0, bn["grad"]) == 0
        dt = time.perf_counter() - t0
        if step < n_warm:
            t_warm += dt
            continue
        t_spent += dt
        keys_done += bn["keys"].size
        n_steps += 1
    rows = ot.n_rows
    ot.close()
    return {
        "value": keys_done / t_spent, "unit": "keys/s", "cores": 1, "kind": "oracle",
        "sample": "%d timed step(s) after %d untimed ones (%.1f s) of the first %d of %d samples per batch (%d key "
                  "occurrences timed, %d rows in the table at the end), %.1f s" % (
                      n_steps, n_warm, t_warm, ws.batch, w.batch, keys_done, rows, t_spent),
    }


def seam_bench(args, torch, WL, CtrTable, CTR_OK, dev):
    """Working-set seam at the size of the benchmarked table: ctr_table_load of every row of the table in
    chunks (the keys are new, so this is insert + state write), ctr_table_collect of the same keys,
    ctr_table_clear.  One JSON line; `steps` is the number of load / collect / clear cycles timed."""
    w = WL.WORKLOADS[args.workload]
    D, R = w.dim, w.capacity_rows
    chunk = min(R, 1 << 22)
    n_chunks = R // chunk
    table = CtrTable(R, D, lr=w.lr, beta1=w.beta1, beta2=w.beta2, eps=w.eps, init_seed=1, init_std=w.init_std,
                     load_factor=w.load_factor, device=dev)
    table.reserve(chunk, 0)
    gen = torch.Generator(device=dev)
    gen.manual_seed(5)
    x = torch.randn((chunk, D), device=dev, generator=gen) * 0.01
    m = torch.randn((chunk, D), device=dev, generator=gen) * 0.01
    v = torch.rand((chunk, D), device=dev, generator=gen) + 1e-8
    # distinct keys: an odd multiplier is a bijection of the integers modulo 2^key_bits
    idx = torch.arange(n_chunks * chunk, dtype=torch.int64, device=dev)
    keys = ((idx * -7046029254386353131) & ((1 << w.key_bits) - 1)).view(n_chunks, chunk)  # 0x9E37...7C15 as int64
    ev = lambda: torch.cuda.Event(enable_timing=True)
    t_load = t_collect = t_clear = 0.0
    cycles = max(1, args.steps)
    for c in range(args.warmup + cycles):
        e = [ev() for _ in range(4)]
        e[0].record()
        for i in range(n_chunks):
            if table.table_load(keys[i], x, m, v) != CTR_OK:
                raise RuntimeError("ctr_table_load failed")
        e[1].record()
        for i in range(n_chunks):
            st, gx, gm, gv, found = table.table_collect(0, keys[i])
            if st != CTR_OK:
                raise RuntimeError("ctr_table_collect failed")
        e[2].record()
        if c == 0:                         # once, untimed: the state read back is the state loaded
            torch.cuda.synchronize()
            if table.last_status() != CTR_OK or table.n_rows != n_chunks * chunk:
                raise RuntimeError("load did not create every row")
            if not (bool(found.all()) and torch.equal(gx, x) and torch.equal(gm, m) and torch.equal(gv, v)):
                raise RuntimeError("collect does not return what load wrote")
        del gx, gm, gv, found
        if table.table_clear() != CTR_OK:
            raise RuntimeError("ctr_table_clear failed")
        e[3].record()
        torch.cuda.synchronize()
        if c >= args.warmup:
            t_load += e[0].elapsed_time(e[1])
            t_collect += e[1].elapsed_time(e[2])
            t_clear += e[2].elapsed_time(e[3])
    rows = n_chunks * chunk
    row_bytes = 8 + 16 + 2 * 3 * 4 * D     # key read, index slot, state read from the caller + written to the table
    n_slots = 1 << max(6, (int(R / w.load_factor) - 1).bit_length())
    ms_load, ms_collect, ms_clear = t_load / cycles, t_collect / cycles, t_clear / cycles
    out = {
        "metric": "working-set seam: rows loaded into / collected from the table per second (1 GPU)",
        "value": rows / (ms_load * 1e-3), "unit": "rows/s (load)", "n_gpus": 1, "steps": cycles, "warmup": args.warmup,
        "ms_per_step": ms_load + ms_collect + ms_clear, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "seam of %s: %d rows of dim %d (x, m, v) in %d chunks of %d keys, %d-bit keys, every key new"
                   % (w.name, rows, D, n_chunks, chunk, w.key_bits)},
        "load": {"ms": ms_load, "rows_per_s": rows / (ms_load * 1e-3),
                 "algorithmic_GBps": rows * row_bytes / (ms_load * 1e-3) / 1e9,
                 "frac_of_hbm_peak": rows * row_bytes / (ms_load * 1e-3) / 1e9 / HBM_PEAK_GBPS},
        "collect": {"ms": ms_collect, "rows_per_s": rows / (ms_collect * 1e-3),
                    "algorithmic_GBps": rows * (row_bytes + 4) / (ms_collect * 1e-3) / 1e9,
                    "frac_of_hbm_peak": rows * (row_bytes + 4) / (ms_collect * 1e-3) / 1e9 / HBM_PEAK_GBPS},
        "clear": {"ms": ms_clear, "algorithmic_GBps": (16 * n_slots + 4 * R) / (ms_clear * 1e-3) / 1e9,
                  "frac_of_hbm_peak": (16 * n_slots + 4 * R) / (ms_clear * 1e-3) / 1e9 / HBM_PEAK_GBPS},
    }
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=40,
                    help="timed steps (default 40: with the 10 warm-up steps the 50 steps of the large configuration, "
                         "each on its own batch; the 10 merge rounds of the k-step configuration)")
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="large")
    ap.add_argument("--variant", default="alg2", choices=["alg2", "adagrad", "prose", "kingma"],
                    help="row update: Algorithm 2's Adam (default), AdaGrad, the prose reading of the merge, "
                         "bias-corrected Adam")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--predict", action="store_true",
                    help="full workload: the timed steps are predictions (lookup without insert + tower forward) "
                         "on a table filled by the warm-up's training steps")
    ap.add_argument("--grad-bf16", action="store_true",
                    help="the pooled gradients reach the push as bfloat16 (ctr_push_adam_bf16): not the "
                         "configuration the metric is quoted on, which has fp32 gradients")
    ap.add_argument("--push-order", default="default",
                    help="order in which the push runs its work spans (ctr_debug_set_push_order): default (the "
                         "library's: win32 for gradient arrays of 256 MiB and more), list, winN (spans inside one "
                         "row first, grouped by N windows of the gradient array), splitN (those in a launch of "
                         "their own), mixN (the other spans dealt between the windows)")
    ap.add_argument("--ab-push-order", default="",
                    help="comma-separated orders (as for --push-order) compared AFTER the timed region in this same "
                         "process: 8 rounds, one step per order and round, medians reported as push_order_ab")
    ap.add_argument("--seam", action="store_true",
                    help="time the working-set seam instead of training steps: ctr_table_load of every row of the "
                         "workload's table, ctr_table_collect of the same keys, ctr_table_clear (one cycle per step)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (one shard of the parameter server); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2201_05500_amd import workloads as WL
    from paper_2201_05500_amd.binding import (CTR_OK, CTR_STEP_LOCAL, CTR_STEP_MERGE_PENDING, CtrTable)

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    dev = "cuda:0"
    if args.seam:
        seam_bench(args, torch, WL, CtrTable, CTR_OK, dev)
        return
    w = WL.WORKLOADS[args.workload]
    kstep = w.k_step > 0
    full = w.name == "full"
    if args.predict and not full:
        print("bench.py: --predict goes with --workload full", file=sys.stderr)
        sys.exit(2)
    if full and args.variant != "alg2":
        print("bench.py: the full step is timed with Algorithm 2's update only", file=sys.stderr)
        sys.exit(2)
    if (args.variant == "prose") != kstep and args.variant != "alg2":
        print("bench.py: --variant prose needs the kstep workload, adagrad/kingma a single-table one", file=sys.stderr)
        sys.exit(2)
    n_state = 2 if args.variant == "adagrad" else 3
    shared_den = kstep and args.variant == "alg2"
    K, Wm = args.steps, args.warmup
    total_steps = K + Wm

    table = CtrTable(w.capacity_rows, w.dim, n_replicas=w.n_replicas, lr=w.lr, beta1=w.beta1,
                     beta2=w.beta2, eps=w.eps, init_seed=1, init_std=w.init_std, kstep=kstep,
                     load_factor=w.load_factor, device=dev, adagrad=args.variant == "adagrad",
                     prose=args.variant == "prose", bias_correction=args.variant == "kingma")

    def set_push_order(name):
        if name == "default":
            return
        kinds = {"list": None, "win": 0, "split": 1, "mix": 2}
        kind = next((k for k in kinds if name.startswith(k)), None)
        if kind is None:
            raise SystemExit("bench.py: unknown push order %r" % name)
        windows = 0 if kind == "list" else int(name[len(kind):])
        if table.set_push_order(windows, kinds[kind] or 0, 0) != CTR_OK:
            raise SystemExit("bench.py: push order %r refused" % name)
    set_push_order(args.push_order)

    # every input of every step resident in HBM before timing; for the k-step workload a "step"
    # is one local step of every replica (plus the merge on every k-th)
    reps = w.n_replicas if kstep else 1
    staged = []                                  # the configuration's own number of distinct batches, then repeated
    max_keys = 1
    for s in range(min(total_steps, w.steps)):
        for j in range(reps):
            b = WL.make_batch(w, s, replica=j, device=dev, with_grad=not full)
            if full:
                b["labels"] = WL.make_labels(w, s, device=dev)
            elif args.grad_bf16:
                b["grad"] = b["grad"].to(torch.bfloat16)
            staged.append(b)
            max_keys = max(max_keys, b["keys"].numel())
    # batches[s * reps + j]: the inputs of step s, replica j (a bounded set of device buffers however many steps)
    batches = [staged[(s % w.steps) * reps + j] for s in range(total_steps) for j in range(reps)]
    G = w.n_segments
    table.reserve(max_keys, G)
    pooled = torch.empty((G, w.dim), dtype=torch.float32, device=dev)
    tower = None
    if full:
        from paper_2201_05500_amd.binding_mlp import CtrMlp
        in_dim = w.slots * w.dim
        tower = CtrMlp(in_dim, WL.FULL_STEP_HIDDEN, lr=w.lr, beta1=w.beta1, beta2=w.beta2, eps=w.eps, init_seed=3,
                       device=dev)
        tower.reserve(w.batch)
        grad_pooled = torch.empty((G, w.dim), dtype=torch.bfloat16 if args.grad_bf16 else torch.float32, device=dev)
        pooled_bf16 = torch.empty((G, w.dim), dtype=torch.bfloat16, device=dev)
        loss = torch.empty(1, dtype=torch.float32, device=dev)
        tower_events = []
    torch.cuda.synchronize()
    def predict_step(s):
        b = batches[s]
        st, _ = table.lookup_pool(0, b["keys"], b["offsets"], out=pooled_bf16)
        if st != CTR_OK:
            raise RuntimeError("ctr_lookup_pool: %d" % st)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        st, _ = tower.forward(0, pooled_bf16.view(w.batch, in_dim))
        e1.record()
        tower_events.append((e0, e1))
        if st != CTR_OK:
            raise RuntimeError("ctr_mlp_forward: %d" % st)

    def run_step(s):
        mode = CTR_STEP_LOCAL
        merge_now = kstep and (s + 1) % w.k_step == 0
        if merge_now and args.variant == "alg2":
            mode = CTR_STEP_MERGE_PENDING
        for j in range(reps):
            b = batches[s * reps + j]
            if full:   # the tower's products take bf16: the pull writes that copy itself
                st, h, _, _ = table.pull_pool_bf16(j, b["keys"], b["offsets"], pooled_bf16)
            else:
                st, h, _ = table.pull_pool(j, b["keys"], b["offsets"], pooled)
            if st != CTR_OK:
                raise RuntimeError("ctr_pull_pool: %d" % st)
            grad = None if full else b["grad"]
            if full:
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                st, _, _ = tower.step(0, pooled_bf16.view(w.batch, in_dim), b["labels"],
                                      grad_pooled.view(w.batch, in_dim), loss=loss)
                e1.record()
                tower_events.append((e0, e1))
                if st != CTR_OK:
                    raise RuntimeError("ctr_mlp_step: %d" % st)
                grad = grad_pooled
            st = table.push_adam(j, h, grad, mode)
            if st != CTR_OK:
                raise RuntimeError("ctr_push_adam: %d" % st)
        if merge_now:
            st = table.kstep_merge()
            if st != CTR_OK:
                raise RuntimeError("ctr_kstep_merge: %d" % st)

    ceiling_GBps, ceiling_kind = copy_ceiling(torch, dev)   # same run, before the timed region

    table.profile_enable(True)
    for s in range(Wm):
        run_step(s)
    torch.cuda.synchronize()
    if table.last_status() != CTR_OK:
        raise RuntimeError("device status after warmup")
    table.profile_read()                       # drop the warmup records
    if full:
        tower_events.clear()
    rows_before = table.n_rows
    merged_before = table.merge_stats() if kstep else (0, 0)

    step_marks = [torch.cuda.Event(enable_timing=True) for _ in range(K + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(Wm, total_steps):
        step_marks[s - Wm].record()
        if args.predict:
            predict_step(s)
        else:
            run_step(s)
    step_marks[K].record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    step_ms = sorted(step_marks[i].elapsed_time(step_marks[i + 1]) for i in range(K))
    steady = sorted(step_marks[i].elapsed_time(step_marks[i + 1]) for i in range(K // 5, K))   # the last 80 %
    median = lambda v: 0.5 * (v[(len(v) - 1) // 2] + v[len(v) // 2])

    stages = table.profile_read()              # HIP events recorded on the launch stream, timed steps only
    status = table.last_status()
    if status != CTR_OK:
        raise RuntimeError("device status %d after the timed steps" % status)
    rows_after = table.n_rows
    elapsed = t1 - t0

    push_order_ab = None
    if args.ab_push_order and not args.predict and not kstep:     # same process, same table, same batches: only the order differs
        names = [n for n in args.ab_push_order.split(",") if n]
        acc = {n: {"push": [], "step": []} for n in names}
        s_ab = Wm
        for _ in range(8):
            for n in names:
                set_push_order(n)
                table.profile_read()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                run_step(Wm + (s_ab - Wm) % K)
                e1.record()
                torch.cuda.synchronize()
                st_ab = table.profile_read()
                acc[n]["push"].append(st_ab["push"][0] / max(st_ab["push"][1], 1) +      # the span walk ...
                                      st_ab["order"][0] / max(st_ab["order"][1], 1))     # ... and what orders it
                acc[n]["step"].append(e0.elapsed_time(e1))
                s_ab += 1
        push_order_ab = {n: {"push_ms_median": median(sorted(v["push"])), "step_ms_median": median(sorted(v["step"]))}
                         for n, v in acc.items()}
        if table.last_status() != CTR_OK:
            raise RuntimeError("device status after the order comparison")
    keys_total = sum(batches[i]["keys"].numel() for i in range(Wm * reps, total_steps * reps))
    L_mean = keys_total / (K * reps)

    # distinct keys per batch, measured on the timed batches (not timed)
    uniq = [int(torch.unique(batches[i]["keys"]).numel()) for i in range(Wm * reps, total_steps * reps)]
    U_mean = sum(uniq) / len(uniq)
    n_new_mean = (rows_after - rows_before) / (K * reps)

    D = w.dim
    gb = 2 if args.grad_bf16 else 4
    step_bytes = algorithmic_bytes_step(L_mean, G, U_mean, n_new_mean, D, shared_den, n_state, gb)
    ms_step = elapsed * 1e3 / K
    stage_ms = {n: (ms / c if c else 0.0) for n, (ms, c) in stages.items()}
    kernel_bytes = {
        "push": algorithmic_bytes_push_kernel(L_mean, G, U_mean, D, shared_den, n_state, gb),
        "pool": algorithmic_bytes_pool_kernel(L_mean, G, U_mean, D, 2 if full else 4),
    }
    n_merges = stages["merge"][1]
    if kstep and n_merges:
        merged_after = table.merge_stats()
        rows_merged = (merged_after[0] - merged_before[0]) / n_merges
        pending_pairs = (merged_after[1] - merged_before[1]) / n_merges
        kernel_bytes["merge"] = algorithmic_bytes_merge_kernel(rows_merged, pending_pairs, rows_after, D,
                                                               w.n_replicas, shared_den)
    # the dominant kernel: the one whose single launch takes longest (stage times are per launch)
    dominant = max(kernel_bytes, key=lambda n: stage_ms[n])
    achieved = kernel_bytes[dominant] / (stage_ms[dominant] * 1e-3) / 1e9 if stage_ms[dominant] else 0.0
    standard = args.variant == "alg2" and not args.grad_bf16 and not full
    traffic_kernel, traffic_step, traffic_prov = measured_traffic(w.name) if standard else ({}, None, None)

    out = {
        "metric": "pulled+updated keys/sec per step and achieved HBM GB/s vs peak (1 GPU)",
        "value": keys_total / elapsed,
        "unit": "keys/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": Wm,
        "ms_per_step": ms_step,
        "ms_per_step_median": median(step_ms),
        "push_order": args.push_order,
        "push_order_ab": push_order_ab,
        "ms_per_step_median_last_80pct": median(steady),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {
            "workload": "%s: R=%d rows, dim %d, batch %d x %d slots, Zipf s=%g over %d ranks, %d-bit keys%s" % (
                w.name, w.capacity_rows, w.dim, w.batch, w.slots, w.zipf_s, w.zipf_universe, w.key_bits,
                (", W=%d replicas, k=%d" % (w.n_replicas, w.k_step)) if kstep else "") + (
                "" if args.variant == "alg2" else ", row update: " + args.variant) + (
                ", pooled gradients bf16" if args.grad_bf16 else ""),
            "keys_per_batch": L_mean,
            "distinct_keys_per_batch": U_mean,
            "new_rows_per_batch": n_new_mean,
            "rows_in_table": rows_after,
        },
        "rows_per_s": U_mean * K * reps / elapsed,
        "step_algorithmic_GBps": step_bytes * reps / (ms_step * 1e-3) / 1e9,
        "step_frac_of_hbm_peak": step_bytes * reps / (ms_step * 1e-3) / 1e9 / HBM_PEAK_GBPS,
        "copy_ceiling_GBps": ceiling_GBps,
        "copy_ceiling_kernel": "ctr_stream_copy (%s), 1 GiB, best of 5, timed in this run" % ceiling_kind,
        "step_frac_of_copy_ceiling": step_bytes * reps / (ms_step * 1e-3) / 1e9 / ceiling_GBps,
        "step_counter_traffic_GBps": traffic_step / (ms_step * 1e-3) / 1e9 if traffic_step else None,
        "stage_ms": stage_ms,
        "stage_launches_per_step": {n: c / K for n, (ms, c) in stages.items()},
        "roofline": {
            "bound": "hbm",
            "kernel": KERNEL_OF_STAGE[dominant],
            "achieved": achieved,
            "peak": HBM_PEAK_GBPS,
            "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBPS,
            "frac_of_copy_ceiling": achieved / ceiling_GBps,
            "algorithmic_bytes_per_launch": kernel_bytes[dominant],
            "traffic": traffic_kernel.get(KERNEL_OF_STAGE[dominant]),
            "traffic_source": traffic_prov,
        },
    }
    # every kernel with a byte model, not only the dominant one
    out["kernel_rooflines"] = {
        KERNEL_OF_STAGE[n]: {"ms_per_launch": stage_ms[n], "algorithmic_bytes_per_launch": kernel_bytes[n],
                             "achieved_GBps": kernel_bytes[n] / (stage_ms[n] * 1e-3) / 1e9,
                             "frac": kernel_bytes[n] / (stage_ms[n] * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                             "frac_of_copy_ceiling": kernel_bytes[n] / (stage_ms[n] * 1e-3) / 1e9 / ceiling_GBps,
                             "traffic": traffic_kernel.get(KERNEL_OF_STAGE[n])}
        for n in kernel_bytes if stage_ms[n]}
    if full:
        tower_ms = sum(a.elapsed_time(b) for a, b in tower_events) / len(tower_events)
        fl = tower_flops(w.batch, in_dim, WL.FULL_STEP_HIDDEN)
        if args.predict:
            fl //= 3                       # forward products only
        out["metric"] = ("prediction (lookup without insert, tower forward): " if args.predict else
                         "full training step (pull, dense tower, push): ") + out["metric"]
        out["dtype"] = "f32 table, bf16 x bf16 -> f32 tower products"
        out["samples_per_s"] = w.batch * K / elapsed
        out["final_loss"] = None if args.predict else float(loss.cpu()[0])
        out["stage_ms"]["tower"] = tower_ms
        out["config"]["tower"] = "%d-%s-1, click rate %g, matrix products by the library's own MFMA kernel" % (
            in_dim, "-".join(str(h) for h in WL.FULL_STEP_HIDDEN), WL.FULL_STEP_CLICK_RATE)
        out["roofline_tower"] = {
            "bound": "mfma", "kernel": ("ctr_mlp_forward" if args.predict else "ctr_mlp_step") +
            " (all products and element-wise kernels of one tower call)",
            "achieved": fl / (tower_ms * 1e-3) / 1e12, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
            "frac": fl / (tower_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, "traffic": None,
        }
    if args.predict:                       # the byte model above is the training step's
        out["step_algorithmic_GBps"] = out["step_frac_of_hbm_peak"] = None
    if not args.no_cpu_baseline and not args.predict:
        out["cpu_baseline"] = cpu_baseline(w, WL)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
