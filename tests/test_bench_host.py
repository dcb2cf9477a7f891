"""Host logic of bench.py that decides what the JSON line may claim (no GPU): the batch-against-loop self-check, the
gate that ties counter figures under profiles/ to the kernel sources they were measured on, and the refusal of more
than one GPU."""
import importlib.util
import os
import subprocess
import sys

import numpy as np
import pytest
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def bench():
    spec = importlib.util.spec_from_file_location("bench_under_test", os.path.join(ROOT, "bench.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def _batch(accept, best, p, delta, H, pmax, near):
    t = torch.as_tensor
    return {"accept_len": t(np.asarray(accept, np.int32)), "best_cand": t(np.asarray(best, np.int32)),
            "tok_p": t(np.asarray(p, np.float32)), "tok_delta": t(np.asarray(delta, np.float32)),
            "row_entropy": t(np.asarray(H, np.float32)), "row_pmax": t(np.asarray(pmax, np.float32)),
            "near_count": t(np.asarray(near, np.int32))}


def test_self_check_accepts_equal_results_and_reports_the_counts(bench):
    B, C, k = 3, 1, 4
    p = np.full((B, C, k), 0.5); d = np.full((B, C, k), 0.2)
    b = _batch([2, 0, 4], [0, 0, 0], p, d, np.full((B, 5), 0.5), np.full((B, 5), 0.9), [1, 0, 2])
    rep = bench.check_batch_against_loop(np, "case", b, np.array([2, 0, 4]), np.array([0, 0, 0]), 0.1, 0.1, C, k)
    assert rep == {"sequences": 3, "batch_vs_loop_differences": 0, "differences_outside_1e-6_of_threshold": 0,
                   "every_threshold_is_row_max": False, "near_threshold_decisions": 3}


def test_self_check_allows_a_difference_only_at_a_threshold(bench):
    B, C, k = 2, 1, 4
    p = np.full((B, C, k), 0.5); d = np.full((B, C, k), 0.2)
    p[1, 0, 2] = 0.2000003; d[1, 0, 2] = 0.2           # the deciding token of sequence 1 sits on its threshold
    H, pmax = np.full((B, 5), 0.5), np.full((B, 5), 0.9)   # alpha*H + beta = 0.15 < pmax: thresholds are not clamped
    b = _batch([4, 3], [0, 0], p, d, H, pmax, [0, 1])
    rep = bench.check_batch_against_loop(np, "case", b, np.array([4, 2]), np.array([0, 0]), 0.1, 0.1, C, k)
    assert rep["batch_vs_loop_differences"] == 1 and rep["differences_outside_1e-6_of_threshold"] == 0
    p[1, 0, 2] = 0.3                                    # the same difference away from any threshold is an error
    b = _batch([4, 3], [0, 0], p, d, H, pmax, [0, 0])
    with pytest.raises(AssertionError, match="away from any threshold"):
        bench.check_batch_against_loop(np, "case", b, np.array([4, 2]), np.array([0, 0]), 0.1, 0.1, C, k)


def test_self_check_allows_no_difference_where_every_threshold_is_the_row_maximum(bench):
    B, C, k = 2, 1, 4
    p = np.full((B, C, k), 0.5); d = np.full((B, C, k), 0.5)   # p = delta = Delta everywhere: "near", but exact
    H, pmax = np.full((B, 5), 9.0), np.full((B, 5), 0.5)       # alpha*H + beta = 1.0 > pmax: clamped everywhere
    b = _batch([4, 3], [0, 0], p, d, H, pmax, [4, 3])
    with pytest.raises(AssertionError, match="every threshold is the row maximum"):
        bench.check_batch_against_loop(np, "case", b, np.array([4, 2]), np.array([0, 0]), 0.1, 0.1, C, k)


def test_counter_files_parse_and_carry_the_hash_of_the_kernel_sources(bench, tmp_path):
    f = tmp_path / "t.txt"
    f.write_text("# comment = ignored\nkernel_source_sha = abc\nw.verify_sweep.rows = 4608\n\nw.verify_sweep.hbm_bytes_per_launch = 12\n")
    got = bench.read_traffic(str(f))
    assert got == {"kernel_source_sha": "abc", "w.verify_sweep.rows": "4608", "w.verify_sweep.hbm_bytes_per_launch": "12"}
    assert bench.read_traffic(str(tmp_path / "missing.txt")) == {}
    sha = bench.kernel_source_sha()
    assert len(sha) == 16 and int(sha, 16) >= 0 and sha == bench.kernel_source_sha()
    # the files under profiles/ are quoted by bench.py only while this holds; both must name one and the same build
    shas = {bench.read_traffic(os.path.join(ROOT, "profiles", n)).get("kernel_source_sha")
            for n in ("row_sweep_traffic.txt", "gumbel_extras_counters.txt")}
    assert len(shas) == 1 and None not in shas


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "ONE GPU" in (r.stderr + r.stdout)
