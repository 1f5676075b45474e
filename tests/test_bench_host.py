"""Host-side parts of the measurement: the byte models bench.py prices the step and its kernels with, the
one-GPU refusal, and the script that turns rocprofv3 CSV output into the committed summaries (no GPU needed)."""
import csv
import json
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def test_byte_models_written_out_for_one_case():
    """Algorithmic bytes of a step and of its two large kernels, term by term, for small round numbers."""
    import bench
    L, G, U, n_new, D = 1000, 300, 200, 10, 64
    step = (8 * L                      # keys
            + 8 * (G + 1)              # offsets, pull and push side
            + 16 * U                   # distinct set written and read
            + 12 * L                   # occurrence -> row map: written, read by the pool, read by the push
            + 16 * U + 16 * n_new      # one 16-byte index slot per distinct key, plus the inserts
            + 4 * D * U                # rows gathered for pooling, once each
            + 4 * D * G                # pooled output
            + 4 * D * G                # pooled gradient
            + 24 * D * U)              # x, m, v read and written
    assert bench.algorithmic_bytes_step(L, G, U, n_new, D, False) == step
    assert bench.algorithmic_bytes_step(L, G, U, n_new, D, True) == step + 4 * D * U        # shared denominator
    assert bench.algorithmic_bytes_step(L, G, U, n_new, D, False, n_state=2) == step - 8 * D * U   # AdaGrad rows [x | G]
    assert bench.algorithmic_bytes_step(L, G, U, n_new, D, False, grad_bytes=2) == step - 2 * D * G
    assert bench.algorithmic_bytes_push_kernel(L, G, U, D, False) == 4 * L + 4 * D * G + 24 * D * U
    assert bench.algorithmic_bytes_pool_kernel(L, G, U, D) == 4 * (G + 1) + 4 * L + 4 * D * U + 4 * D * G
    # merge: 8 replicas, every merged row: v and x of every replica read, x written, shared v written once
    W = 8
    assert bench.algorithmic_bytes_merge_kernel(50, 7, 90, 16, W, True) == 4 * 90 + 50 * (3 * W + 1) * 64 + 7 * 64
    assert bench.algorithmic_bytes_merge_kernel(50, 0, 90, 16, W, False) == 4 * 90 + 50 * (4 * W) * 64


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_committed_traffic_records_are_read_with_their_provenance():
    import bench
    per, step, prov = bench.measured_traffic("large")
    assert prov["file"] == "profiles/large_step_traffic.json" and prov["commit"] and prov["source_hash"]
    assert isinstance(prov["matches_current_sources"], bool)
    assert per["k_push_span"] > 1e10 and step > per["k_push_span"] + per["k_pool"]
    assert bench.measured_traffic("no such workload") == ({}, None, None)


def _write_csv(path, header, rows):
    os.makedirs(os.path.dirname(path), exist_ok=True)
    with open(path, "w", newline="") as f:
        w = csv.writer(f)
        w.writerow(header)
        w.writerows(rows)


def test_profile_summary_scales_counters_by_the_copy_kernel(tmp_path):
    """Synthetic rocprofv3 output: the copy kernel reads 1 GiB and the fetch counter books half of it, so a kernel
    whose last dispatch shows 1000 KiB fetched and 500 KiB written moved (2 * 1000 + 500) KiB."""
    t, f, w, out = (str(tmp_path / n) for n in ("trace", "fetch", "write", "out"))
    os.makedirs(out)
    push = "void ctr::k_push_span<16>(ctr::DevHeader const*, unsigned int)"
    copy = "void ctr::k_stream_copy<false>(float const*, float*, unsigned long)"
    _write_csv(t + "/vm/1_kernel_stats.csv", ["Name", "Calls", "TotalDurationNs", "AverageNs", "Percentage", "MinNs", "MaxNs", "StdDev"],
               [[push, 4, 4000000, 1000000.0, "80.0", 900000, 1100000, 1.0], [copy, 2, 1000000, 500000.0, "20.0", 1, 2, 1.0]])
    head = ["Dispatch_Id", "Kernel_Name", "Counter_Name", "Counter_Value"]
    _write_csv(f + "/vm/2_counter_collection.csv", head,
               [[1, copy, "FETCH_SIZE", 524288], [2, push, "FETCH_SIZE", 900], [3, push, "FETCH_SIZE", 1000]])
    _write_csv(w + "/vm/3_counter_collection.csv", head,
               [[1, copy, "WRITE_SIZE", 1048576], [2, push, "WRITE_SIZE", 400], [3, push, "WRITE_SIZE", 500]])
    subprocess.check_call([sys.executable, "-m", "paper_2201_05500_amd.profile_summary", "unit_step", t, f, w,
                           "--steps", "2", "--out-dir", out, "--command", "python3 bench.py"], cwd=ROOT,
                          stdout=subprocess.DEVNULL)
    rec = json.load(open(os.path.join(out, "unit_step_traffic.json")))
    assert rec["scale"] == {"fetch": 2.0, "write": 1.0}
    k = rec["kernels"]["k_push_span"]
    assert (k["fetch_KiB"], k["write_KiB"], k["launches_per_step"]) == (1000.0, 500.0, 1.0)
    assert rec["step"] == {"fetch_KiB": 1000.0, "write_KiB": 500.0}
    assert rec["source_hash"] and rec["workload"] == "unit_step"
    text = open(os.path.join(out, "unit_step_kernels.txt")).read()
    assert "k_push_span<16>" in text and "fetch x2.000, write x1.000" in text and "python3 bench.py" in text


def test_cpu_baseline_runs_the_oracle_on_the_configurations_own_batches():
    """The tiny configuration has one distinct batch, repeated: the baseline must repeat it too (five different
    batches would overflow its 2^16-row table)."""
    import bench
    from paper_2201_05500_amd import workloads as WL
    cb = bench.cpu_baseline(WL.WORKLOADS["tiny"], WL)
    assert cb["kind"] == "oracle" and cb["unit"] == "keys/s" and cb["cores"] == 1 and cb["value"] > 0
    assert "timed step(s)" in cb["sample"]
