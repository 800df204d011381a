"""Host logic of bench.py that needs no GPU: flop accounting, the row count of the backward products, the stored
counter figures (valid only for the GEMM sources they were taken on) and the refusal of more than one GPU."""
import os
import subprocess
import sys

import bench

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_flops_per_step_add_up_to_the_algorithmic_count():
    M, d, ff, V = 43008, 4096, 11008, 256
    f = bench.gemm_flops_per_step(M, d, ff, V)
    assert set(f) == set(bench.GEMM_STAGES)
    assert sum(f.values()) == 3.0 * (6.0 * d * ff + 2.0 * d * V) * M          # 817.9 MFLOP per kept token
    assert f["gemm_gate_up"] == 2.0 * M * d * 2 * ff and f["gemm_dWg_dWu"] == 2 * 2.0 * M * d * ff
    half = bench.gemm_flops_per_step(M, d, ff, V, M // 2)
    fwd = ("gemm_gate_up", "gemm_down", "gemm_logits_loss")
    assert all(half[k] == f[k] for k in fwd) and all(half[k] == f[k] / 2 for k in f if k not in fwd)


def test_backward_rows_follow_the_one_in_sixteen_rule():
    assert bench.backward_rows(1000, [0.5, 0.25], dense=False) == 625.0      # 500 and 750 rows
    assert bench.backward_rows(1000, [0.05, 0.5], dense=False) == 750.0      # below one in sixteen nothing is dropped
    assert bench.backward_rows(1000, [0.5], dense=True) == 1000.0
    assert bench.backward_rows(1000, [], dense=False) == 1000.0


def test_stored_traffic_is_bound_to_the_gemm_sources(tmp_path, monkeypatch):
    import paper_2605_16154_amd.profile_summary as ps
    assert bench.stored_traffic("no_such_file.txt") is None
    committed = bench.stored_traffic("gemm_gate_up_cfg2_traffic.txt")
    text = open(os.path.join(ROOT, "profiles", "gemm_gate_up_cfg2_traffic.txt")).read()
    stored_hash = [l.split("=", 1)[1] for l in text.splitlines() if l.startswith("source_hash=")][0]
    if stored_hash == ps.kernel_source_hash():
        assert committed is not None and 1e9 < committed < 1e11              # bytes beyond L2 per gate/up launch
    else:
        assert committed is None                                             # sources changed since the counters were taken


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "single-GPU" in (r.stdout + r.stderr)
