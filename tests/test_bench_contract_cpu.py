"""CPU checks of the benchmark's contract: the refusal of more than one GPU, the algorithmic work it
prices the kernels against (hand-computed for the C2 workload) and the staleness rule of the
stored HBM-traffic counters."""
import os
import subprocess
import sys

import numpy as np
import pytest

import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "one GPU" in r.stderr
    assert r.stdout.strip() == ""          # no JSON line


def test_algorithmic_work_of_c2_by_hand():
    w = bench.algorithmic_work(synth.get_config("c2"))
    T, H, E, k, I, Is, b = 4096, 2048, 64, 6, 1408, 2816, 2
    N = T * k
    assert N == 24576
    assert w["gate_up_flops"] == 4 * N * H * I == 283467841536
    assert w["down_flops"] == 2 * N * H * I
    assert w["shared_gate_up_flops"] == 4 * T * H * Is == 94489280512
    assert w["dispatch_bytes"] == (T + N) * H * b + 16 * N == 117833728
    assert w["combine_bytes"] == (N + 2 * T) * H * b + 8 * N == 134414336
    assert w["route_bytes"] == T * H * b + H * E * b + 12 * N


def test_stored_traffic_is_dropped_when_the_kernel_sources_change(tmp_path, monkeypatch):
    now = bench.stored_traffic("c2")
    if now is None:
        pytest.skip("no current counter summary for c2")
    assert now > 0.87e9                     # never below the algorithmic bytes
    monkeypatch.setattr(bench, "kernel_source_hash", lambda: "0" * 64)
    assert bench.stored_traffic("c2") is None
    assert bench.stored_traffic("no_such_workload") is None


def test_router_skew_changes_only_the_router_and_makes_the_load_uneven():
    import torch
    base = synth.scaled(synth.get_config("c2"), T=2048)
    skew = synth.scaled(base, router_skew=0.5)
    assert torch.equal(synth.draw_x(base), synth.draw_x(skew))
    assert torch.equal(synth.draw_expert(base, 3)["up"], synth.draw_expert(skew, 3)["up"])
    assert torch.equal(synth.draw_router(base), synth.draw_router(synth.scaled(base, router_skew=0.0)))

    def spread(cfg):
        top = (synth.draw_x(cfg).float() @ synth.draw_router(cfg).float()).topk(cfg.k, dim=1).indices
        cnt = np.bincount(top.numpy().ravel(), minlength=cfg.E)
        return cnt.max() / cnt.mean()
    assert spread(base) < 1.3 and spread(skew) > 2.0
