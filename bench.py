#!/usr/bin/env python3
"""Benchmark of the failure-remapped MoE layer on one MI355X.

A step is one pass of the whole hot path (route -> dispatch -> expert FFN -> combine) over one
batch of synthetic tokens, with the workload's failed ranks removed from the expert map, replayed
from one captured graph.  Prints one JSON line:

  value        tokens/s of the layer (T / mean step time), inputs resident in HBM
  roofline     the dominant kernel (grouped gate/up GEMM of the routed experts) against the bf16
               dense MFMA peak, from HIP-event timing of that kernel inside this run
  cpu_baseline the CPU oracle timed on this host on a bounded sample of the same workload (the same switch,
               --no-cpu-baseline, also drops the oracle check of the remap block: nothing else here uses the oracle)
  stages       per-kernel mean microseconds (one HIP-event pair per launch) and the stage rates (GB/s,
               TFLOP/s) from events recorded between the stages of the same eager step
  remap        latency from revive_update_map to the end of the first step under the new map,
               replaying the same graph executable
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_PEAK_TFLOPS = {"bf16": 2500.0, "fp32": 157.3}


def algorithmic_work(cfg):
    """Algorithmic bytes / flops per step of each stage (read every input once, write every output once)."""
    b = 2 if cfg.dtype == "bf16" else 4
    T, H, E, k, I, Is = cfg.T, cfg.H, cfg.E, cfg.k, cfg.I, cfg.I_shared
    N = T * k
    return {
        "route_bytes": T * H * b + H * E * b + T * k * 12,
        "dispatch_bytes": (T + N) * H * b + N * 16,
        "combine_bytes": (N + (2 if Is else 1) * T) * H * b + N * 8,
        "gate_up_flops": 4 * N * H * I,
        "down_flops": 2 * N * H * I,
        "shared_gate_up_flops": 4 * T * H * Is,
        "shared_down_flops": 2 * T * H * Is,
    }


DOMINANT_KERNEL_SOURCES = ("gemm_bf16.hpp", "ffn.hip", "ctx.hpp")


def kernel_source_hash():
    """SHA-256 over the sources of the dominant kernel, the key that ties stored counters to a kernel version."""
    import hashlib
    h = hashlib.sha256()
    for name in DOMINANT_KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_2602_21140_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def stored_traffic(workload):
    """HBM bytes per launch of the dominant kernel from the committed counter summary of this workload, or None
    when there is none or the kernel's sources have changed since the counters were collected."""
    path = os.path.join(ROOT, "profiles", f"{workload}_ffn_gate_up_hbm_traffic.txt")
    try:
        text = open(path).read()
    except OSError:
        return None
    fields = dict(line.split("=", 1) for line in text.splitlines() if "=" in line and not line.startswith(" "))
    fields = {k.strip(): v.strip() for k, v in fields.items()}
    if fields.get("kernel_sources_sha256") != kernel_source_hash():
        return None
    try:
        return float(fields["traffic_bytes_per_launch"])
    except (KeyError, ValueError):
        return None


def cpu_baseline(cfg, g, sample_tokens):
    """Time the oracle (as it stands) on the first `sample_tokens` tokens of the workload."""
    import numpy as np
    import torch
    import synth
    from oracle import revive_oracle as orc

    def f64(t):
        # widened on the device and copied: no CPU thread pool of torch's is left spinning beside the oracle's BLAS
        return t.detach().to(torch.float64).cpu().numpy()

    class DrawnOnDemand(dict):
        """Expert e's fp64 matrices, drawn from the seeded generator when the oracle asks for them (same seed and
        device: the bits the layer packed) and dropped afterwards: the large workloads' experts do not fit the host
        all at once.  The time spent drawing is kept apart; it is not the oracle's."""
        draw_s = 0.0

        def __missing__(self, e):
            t = time.perf_counter()
            w = {n: np.ascontiguousarray(f64(m)) for n, m in synth.draw_expert(cfg, int(e), g.device).items()}
            self.draw_s += time.perf_counter() - t
            return w

    x = f64(g.x[:sample_tokens])
    w_r = f64(g.w_router)
    experts = DrawnOnDemand()
    if 3 * cfg.H * cfg.I * 8 * cfg.E <= (8 << 30):   # everything fits the host: draw it all before the clock starts
        for e in range(cfg.E):
            experts[e] = experts.__missing__(e)
        experts.draw_s = 0.0
    sh = synth.draw_shared(cfg, g.device)
    shared = None if sh is None else {n: np.ascontiguousarray(f64(t)) for n, t in sh.items()}
    emap = orc.build_map(g.p2l, g.failed, cfg.slots_per_rank, cfg.E, cfg.max_replicas)
    t0 = time.perf_counter()
    orc.layer_staged(x, w_r, experts, shared, g.p2l, emap, cfg.k, cfg.score_fn, cfg.n_group, cfg.topk_group)
    dt = time.perf_counter() - t0 - experts.draw_s
    try:
        from threadpoolctl import threadpool_info
        threads = max([i.get("num_threads", 1) for i in threadpool_info()] or [1])
    except Exception:
        threads = len(os.sched_getaffinity(0))
    return {"value": sample_tokens / dt, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"first {sample_tokens} of {cfg.T} tokens, whole layer (route, dispatch, fp64 expert FFN over all "
                      f"{cfg.E} experts' weights, combine), {dt:.2f} s"}


def snapshot_step(cfg, g, n_tokens, n_out_tokens, seed):
    """Host copies of what the step that has just run produced for a seeded sample of tokens (a few
    device gathers; no arithmetic), to be judged later by check_against_oracle."""
    import numpy as np
    import torch
    rng = np.random.default_rng(seed)
    toks = np.sort(rng.choice(cfg.T, size=min(n_tokens, cfg.T), replace=False))
    idx = torch.from_numpy(toks).to(g.device)
    b = g.buf
    sub = idx[:n_out_tokens]
    return {"toks": toks, "failed": g.failed.copy(),
            "logits": b["logits"][idx].to(torch.float64).cpu().numpy(),
            "topk_logical": b["topk_logical"][idx].cpu().numpy(), "topk_phys": b["topk_phys"][idx].cpu().numpy(),
            "x": g.x[sub].to(torch.float64).cpu().numpy(), "out": b["out"][sub].to(torch.float64).cpu().numpy()}


def check_against_oracle(cfg, g, snap):
    """Was the snapshotted step the layer under the map then in force?  Compares, for the sampled tokens,
    the chosen experts and slots with the oracle's selection and remap under that map (on the step's own
    logits), and for the first few of them the complete output row with the oracle's fp64 layer."""
    import numpy as np
    import torch
    import synth
    from oracle import revive_oracle as orc

    def f64(t):
        return t.detach().to(torch.float64).cpu().numpy()

    toks = snap["toks"]
    m = orc.build_map(g.p2l, snap["failed"], cfg.slots_per_rank, cfg.E, cfg.max_replicas)
    s = orc.scores(snap["logits"], cfg.score_fn)
    ref_l = orc.select_topk(orc.masked_selection_scores(s, m.l2p_count), cfg.k, cfg.n_group, cfg.topk_group)
    ref_p = np.stack([[m.l2p_table[e, t % m.l2p_count[e]] for e in row] for t, row in zip(toks, ref_l)])
    ok = bool(np.array_equal(snap["topk_logical"], ref_l) and np.array_equal(snap["topk_phys"], ref_p))
    err = None
    n_out = snap["out"].shape[0]
    if ok and n_out > 0:
        w = orc.gate_weights(s[:n_out], ref_l[:n_out])
        xs = snap["x"]
        ref = np.zeros((n_out, cfg.H))
        for a in range(n_out):
            for j in range(cfg.k):
                we = {n: f64(t) for n, t in synth.draw_expert(cfg, int(ref_l[a, j]), g.device).items()}
                ref[a] += w[a, j] * orc.swiglu_ffn(xs[a:a + 1], we["gate"], we["up"], we["down"])[0]
        sh = synth.draw_shared(cfg, g.device)
        if sh is not None:
            ref += orc.swiglu_ffn(xs, f64(sh["gate"]), f64(sh["up"]), f64(sh["down"]))
        err = float(np.abs(snap["out"] - ref).max() / np.abs(ref).max())
        ok = ok and err < (1e-2 if cfg.dtype == "bf16" else 1e-4)
    return ok, err


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="c5",
                    help="c5 (default: the largest of the workloads, which one GPU holds), c4, c3, c2, c1")
    ap.add_argument("--cpu-sample-tokens", type=int, default=4096)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--overlap-shared", action="store_true",
                    help="run the shared expert on a side stream next to route/dispatch (off by default so that "
                         "every kernel of the step runs alone and its timing is its own)")
    ap.add_argument("--microbatches", type=int, default=0,
                    help="also time the same batch run as this many microbatches on separate streams inside one graph "
                         "(a secondary figure under 'microbatch'; the headline value is always the single batch)")
    ap.add_argument("--skew", type=float, default=0.0,
                    help="secondary run under uneven expert load: router column e is scaled by exp(skew * z_e), "
                         "z_e ~ N(0,1) (0.3 gives slots between a few rows and 2.5 times the mean); the headline "
                         "workload is the unskewed one")
    ap.add_argument("--vendor-gemm", action="store_true",
                    help="context only: also time the vendor library's dense bf16 GEMM (torch.matmul) on the gate/up "
                         "projection's shape taken as one dense product, with the same kind of random operands "
                         "(reported under 'context'; no part of the path uses it)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain device copy of 1 GiB (read 1 GiB, write 1 GiB) so that hardware "
                         "counters collected over this command can be scaled by a kernel of known traffic")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this library runs on one GPU only (expert-parallel ranks are simulated as rank segments "
              "inside one HBM); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import synth
    from synth.resident import ResidentLayer

    cfg = synth.get_config(args.workload)
    if args.skew != 0.0:
        cfg = synth.scaled(cfg, router_skew=args.skew)
    torch.cuda.set_device(0)
    g = ResidentLayer(cfg, device="cuda:0")
    L = g.layer
    work = algorithmic_work(cfg)
    stream = torch.cuda.Stream()
    K, W = args.steps, args.warmup

    with torch.cuda.stream(stream):
        ov = args.overlap_shared
        g.forward(stream=stream, overlap_shared=ov)   # eager pass (also configures the kernels)
        stream.synchronize()
        g.capture(stream, overlap_shared=ov)
        exec_id = L.graph_exec_id(g.graph)
        for _ in range(W):
            g.replay(stream)
        stream.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(K):
            g.replay(stream)
        e1.record(stream)
        stream.synchronize()
        ms_per_step = e0.elapsed_time(e1) / K

        # per-kernel HIP-event timing of the same step, launched eagerly on the same stream
        L.set_kernel_timing(True)
        L.reset_kernel_times()
        for _ in range(K):
            g.forward(stream=stream, overlap_shared=False)
        stream.synchronize()
        times = L.kernel_times()
        L.set_kernel_timing(False)

        # whole stages of the same eager step (one event between stages, no per-kernel events)
        marks = []
        for _ in range(K):
            g.forward(stream=stream, overlap_shared=False, stage_marks=marks)
        stream.synchronize()
        stage_us = {}
        for si, name in enumerate(("route", "dispatch", "expert_ffn", "combine")):
            stage_us[name] = 1e3 * sum(marks[5 * s + si].elapsed_time(marks[5 * s + si + 1]) for s in range(K)) / K

        # recovery: flip the mask, replay the same executable, time to the end of the first new step
        other = [r for r in range(cfg.n_ranks) if r not in cfg.failed_ranks]
        new_failed = list(cfg.failed_ranks[:-1]) + [other[len(other) // 2]] if cfg.failed_ranks else [other[0]]
        try_failed = new_failed if args.workload != "c5" else []
        remap, snaps = [], []
        for trial in range(5):
            target = try_failed if trial % 2 == 0 else list(cfg.failed_ranks)
            for _ in range(2):          # steady steps under the map still in force, so that the flip meets a busy GPU
                g.replay(stream)
            stream.synchronize()
            t0 = time.perf_counter()
            g.set_failed(target, stream=stream)
            t1 = time.perf_counter()
            g.replay(stream)
            stream.synchronize()
            t2 = time.perf_counter()
            phys = g.buf["topk_phys"]
            dead = torch.from_numpy(np.repeat(g.failed, cfg.slots_per_rank)).to(phys.device)
            ok = not bool(dead[phys.long()].any().item())
            remap.append(((t1 - t0) * 1e3, (t2 - t0) * 1e3, ok))
            # what that first step produced for sampled tokens, judged against the oracle once the timing is over
            # (every trial the routing, the first two trials also complete output rows)
            if not args.no_cpu_baseline:
                snaps.append(snapshot_step(cfg, g, 256, 2 if trial < 2 else 0, seed=100 + trial))
        g.set_failed(cfg.failed_ranks, stream=stream)
        g.replay(stream)   # leave the buffers as the workload's own failure set produces them
        stream.synchronize()
        same_exec = L.graph_exec_id(g.graph) == exec_id
    remap_checks = [check_against_oracle(cfg, g, sn) for sn in snaps]

    micro = None
    if args.microbatches > 1:
        from synth.resident import MicrobatchPipeline
        pipe = MicrobatchPipeline(g, args.microbatches)
        with torch.cuda.stream(stream):
            pipe.forward(stream)
            stream.synchronize()
            pipe.capture(stream)
            for _ in range(W):
                pipe.replay(stream)
            stream.synchronize()
            m0, m1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            m0.record(stream)
            for _ in range(K):
                pipe.replay(stream)
            m1.record(stream)
            stream.synchronize()
        micro = {"n": args.microbatches, "ms_per_step": m0.elapsed_time(m1) / K}
        micro["tokens_per_s"] = cfg.T / (micro["ms_per_step"] * 1e-3)
        pipe.close()

    context = None
    if args.vendor_gemm and cfg.dtype == "bf16":
        M, Kd, Nd = cfg.N, cfg.H, 2 * cfg.I
        a = torch.randn(M, Kd, device="cuda:0", dtype=torch.bfloat16)
        b = torch.randn(Nd, Kd, device="cuda:0", dtype=torch.bfloat16) * Kd ** -0.5
        for _ in range(5):
            c = a @ b.t()
        torch.cuda.synchronize()
        v0, v1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        v0.record()
        for _ in range(20):
            c = a @ b.t()
        v1.record()
        torch.cuda.synchronize()
        vms = v0.elapsed_time(v1) / 20
        context = {"vendor_dense_gemm_TFLOPs": 2.0 * M * Kd * Nd / (vms * 1e-3) / 1e12,
                   "shape": f"{M} x {Kd} x {Nd} bf16 (all routed rows against one expert's gate/up matrix), random operands",
                   "note": "what the vendor library's dense GEMM reaches on this GPU and data; not part of the path"}
        del a, b, c

    if args.calibration_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0").fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # rows per live slot of the step just timed (bench reporting only)
    off = g.buf["slot_offsets"].cpu().numpy().astype(np.int64)
    live_slots = np.repeat(~g.failed.astype(bool), cfg.slots_per_rank)
    rows = np.diff(off)[live_slots]
    load = {"rows_per_live_slot_min": int(rows.min()), "median": int(np.median(rows)), "max": int(rows.max())}

    avg_us = {n: (1e3 * ms / c if c else None) for n, (ms, c) in times.items()}
    dom = "ffn_gate_up"
    # with a shared expert the library serves routed and shared gate/up projections in one launch
    merged = cfg.I_shared > 0 and avg_us["ffn_shared_gate_up"] is None
    dom_flops = work["gate_up_flops"] + (work["shared_gate_up_flops"] if merged else 0)
    dom_tflops = dom_flops / (avg_us[dom] * 1e-6) / 1e12
    peak = MFMA_PEAK_TFLOPS[cfg.dtype]

    def gbs(nbytes, stage):
        return nbytes / (stage_us[stage] * 1e-6) / 1e9

    ffn_us = stage_us["expert_ffn"]
    ffn_flops = sum(work[n] for n in ("gate_up_flops", "down_flops", "shared_gate_up_flops", "shared_down_flops"))
    stages = {
        "kernel_us": {n: (round(v, 2) if v else None) for n, v in avg_us.items()},
        "stage_us": {n: round(v, 2) for n, v in stage_us.items()},
        "route_GBs": gbs(work["route_bytes"], "route"),
        "dispatch_GBs": gbs(work["dispatch_bytes"], "dispatch"),
        "dispatch_frac_of_hbm": None,
        "combine_GBs": gbs(work["combine_bytes"], "combine"),
        "ffn_TFLOPs": ffn_flops / (ffn_us * 1e-6) / 1e12,
        "ffn_frac_of_mfma_peak": ffn_flops / (ffn_us * 1e-6) / 1e12 / peak,
        "sum_kernel_us": round(sum(v for v in avg_us.values() if v), 1),
    }
    stages["dispatch_frac_of_hbm"] = stages["dispatch_GBs"] / HBM_PEAK_GBS
    stages["combine_frac_of_hbm"] = stages["combine_GBs"] / HBM_PEAK_GBS
    host_ms = sorted(r[0] for r in remap)[len(remap) // 2]
    first_ms = sorted(r[1] for r in remap)[len(remap) // 2]

    result = {
        "metric": "MoE-layer tokens/s with failed ranks", "value": cfg.T / (ms_per_step * 1e-3), "unit": "tokens/s",
        "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"{cfg.name}: T={cfg.T} H={cfg.H} E={cfg.E} top-{cfg.k} I={cfg.I} shared I={cfg.I_shared} "
                               f"{cfg.score_fn}" + (f" {cfg.n_group} groups/top-{cfg.topk_group}" if cfg.n_group > 1 else "")
                               + f", {cfg.n_ranks} simulated ranks x {cfg.slots_per_rank} slots, failed ranks "
                               f"{list(cfg.failed_ranks)}" + (f", router columns scaled by exp({cfg.router_skew} z)" if cfg.router_skew else ""),
                   "map": g.stats, "load": load, "execution": "one captured graph replayed per step" + (", shared expert on a side stream" if ov else "")},
        "roofline": {"bound": "mfma", "kernel": "gemm_bf16_dma_kernel<256,256,2,4,SwiGLU> (ffn_gate_up)" if cfg.dtype == "bf16" else "gemm_f32_kernel<SwiGLU> (ffn_gate_up)",
                     "achieved": dom_tflops, "peak": peak, "unit": "TFLOP/s", "frac": dom_tflops / peak,
                     "avg_launch_us": avg_us[dom], "flops_per_launch": dom_flops,
                     "launch_covers": "routed experts + shared expert gate/up projections" if merged else "routed experts gate/up projection",
                     "traffic": stored_traffic(cfg.name) if cfg.router_skew == 0.0 else None},
        "stages": stages,
        "remap": {"update_map_host_ms": host_ms, "update_to_first_step_done_ms": first_ms,
                  "minus_steady_step_ms": first_ms - ms_per_step, "routes_avoid_failed_ranks": all(r[2] for r in remap),
                  "first_step_matches_oracle_under_new_map": (None if args.no_cpu_baseline else all(c[0] for c in remap_checks)),
                  "first_step_out_rel_err": [c[1] for c in remap_checks if c[1] is not None],
                  "same_graph_exec": same_exec},
    }
    if micro is not None:
        result["microbatch"] = micro
    if context is not None:
        result["context"] = context
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg, g, min(args.cpu_sample_tokens, cfg.T))
    g.close()
    print(json.dumps(result))


if __name__ == "__main__":
    main()
