#!/usr/bin/env python3
"""Throughput of the DeepSqueeze step (ds_step) on one MI355X.

One "step" is one ds_step call: the whole fused compress-and-gossip pass (Algorithm 1, lines 5-9)
over all n workers of a benchmark configuration, gradients already resident in HBM.

A default run times the four bandwidth-bound configurations of the benchmark (1-4) one after the
other, plus the cache-resident configuration 0 as a report-only line, and prints ONE JSON line on
stdout.  Its headline (value, ms_per_step, config.workload, roofline) is configuration 4, the
largest one (32 workers x 25.6 M parameters, top-1 %); the `configs` array carries the same figures
for every configuration.  `roofline.achieved` is algorithmic bytes per step / device time per step
(HIP events on the launch stream around the K timed steps, all kernels of the step included)
against the 8 TB/s nameplate.  `cpu_baseline` is the CPU oracle timed on a bounded sample of the
headline workload, on all host cores and on one.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config i] [--no-cpu] [--hip-graph]

--config i restricts the run to one configuration (5, 6, 7: the extra workloads), which then is
the headline: the profiles under profiles/ are taken that way.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
HEADLINE = 4
DEFAULT_SET = [1, 2, 3, 4, 0]


def algorithmic_bytes_per_param(w) -> float:
    """Bytes the method must move per worker-parameter: read x, g, delta; write x, delta; write the message.
    CHOCO-SGD moves the same arrays (its public copies in place of delta); DCD-PSGD has no second state array:
    read x, g; write x; write the message."""
    from paper_1907_07346_amd import workloads as wl
    if w.kind == wl.KIND_QUANT_MAXABS:
        msg = w.bits / 8 + 4 / w.block
    elif w.kind == wl.KIND_SIGN_MEANABS:
        msg = 1 / 8 + 4 / w.block
    elif w.kind == wl.KIND_TOPK:
        msg = 8 * w.k / w.N
    elif w.kind == wl.KIND_QUANT_L2NORM:
        msg = w.bits / 8
    elif w.kind == wl.KIND_RAND_SPARSE:
        msg = 4 * w.k / w.N
    elif w.kind == wl.KIND_GSPAR:
        msg = 8 * w.k / w.N
    else:
        msg = 4.0
    return (12.0 if w.algo == wl.ALGO_DCD_PSGD else 20.0) + msg


def cpu_model() -> str:
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.lower().startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def _oracle_leg(ws, all_cores: bool, budget_s: float):
    import oracle
    from paper_1907_07346_amd import workloads as wl
    W = oracle.ring_matrix(ws.n) if ws.topo == wl.TOPO_RING else oracle.torus_matrix(*ws.torus)
    st = oracle.OracleState(n=ws.n, N=ws.N, W=W, kind=ws.kind, gamma=ws.gamma, eta=ws.eta, bits=ws.bits,
                            block=ws.block, k=ws.k, seed=ws.seed)
    c = wl.centres(ws) if ws.grad == "quadratic" else None
    gs = [wl.gradient(ws, t, st.x, c) for t in range(2)]
    oracle.step(st, gs[0], want_cv=False, want_msg=True, all_cores=all_cores)     # warm-up (page faults, code)
    steps, t0 = 0, time.perf_counter()
    while True:
        oracle.step(st, gs[steps % 2], want_cv=False, want_msg=True, all_cores=all_cores)
        steps += 1
        el = time.perf_counter() - t0
        if el > budget_s or steps >= 200:
            break
    return ws.n * ws.N * steps / el, steps, el, oracle.threads(all_cores)


def cpu_baseline(w, budget_s=9.0):
    """The CPU oracle, as it stands, on the first Ns columns of the same workload (all n workers): the build with
    its loops over workers spread over all host cores (OpenMP), and the plain single-thread build."""
    blk = w.block if w.block else 1024
    Ns = min(w.N, max(blk, (16_000_000 // w.n) // blk * blk))
    ws = w.scaled(Ns)
    v_all, s_all, el_all, thr = _oracle_leg(ws, True, budget_s)
    v_one, s_one, el_one, _ = _oracle_leg(ws, False, budget_s)
    nproc = os.cpu_count()
    try:
        nproc = len(os.sched_getaffinity(0))
    except (AttributeError, OSError):
        pass
    return {"value": v_all, "unit": "worker-param updates/s", "cores": thr, "kind": "oracle",
            "sample": f"{w.name}: first {Ns} of {w.N} columns, all {w.n} workers; {s_all} steps in {el_all:.1f} s on {thr} "
                      f"OpenMP threads (parallel for over workers), {s_one} steps in {el_one:.1f} s on one thread; g++ -O2",
            "value_one_thread": v_one, "nproc": nproc, "cpu_model": cpu_model()}


def yardsticks(torch, b):
    """What a trivial kernel reaches on this GPU: a plain copy, the access mix of ds_step (3 streaming loads,
    2 stores, in place) without its arithmetic, and the same for the DCD-PSGD step (2 loads, 1 store)."""
    nbytes = 1 << 30
    src = torch.empty(nbytes // 4, dtype=torch.float32, device="cuda").normal_()
    dst = torch.empty_like(src)
    for _ in range(3):
        b.ds_bench_copy(dst, src)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    reps = 20
    for _ in range(reps):
        b.ds_bench_copy(dst, src)
    e1.record()
    torch.cuda.synchronize()
    copy_gbs = 2 * nbytes * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9
    third = torch.zeros_like(src)
    dst.zero_()
    for _ in range(3):
        b.ds_bench_stream(dst, third, src)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(reps):
        b.ds_bench_stream(dst, third, src)
    e1.record()
    torch.cuda.synchronize()
    mix_gbs = 5 * nbytes * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9
    for _ in range(3):
        b.ds_bench_stream(dst, None, src)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(reps):
        b.ds_bench_stream(dst, None, src)
    e1.record()
    torch.cuda.synchronize()
    mix21_gbs = 3 * nbytes * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9
    del src, dst, third
    torch.cuda.empty_cache()
    return copy_gbs, mix_gbs, mix21_gbs


def run_config(torch, b, wl, w, K, Wm, hip_graph, copy_gbs, mix_gbs, mix21_gbs, traffic_table):
    """Times K steps of one configuration after Wm warm-up steps; returns its report entry."""
    ds = b.DeepSqueeze.from_workload(w)
    _, _, ld = ds.ds_state_ptrs()
    # A fresh i.i.d. gradient for every step, as the configuration says, all resident in HBM before the clock
    # starts; if K + W of them do not fit, the buffers are cycled (noted in the output).
    per_buf = w.n * ld * 4
    free_b, _ = torch.cuda.mem_get_info()
    nbuf = int(max(2, min(K + Wm, (free_b - (8 << 30)) // per_buf)))
    gs = []
    for t in range(nbuf):                                   # pitch = state pitch
        g = torch.zeros((w.n, ld), dtype=torch.float32, device="cuda")
        g[:, :w.N] = wl.device_gradient(w, t)
        gs.append(g)
    torch.cuda.synchronize()
    for t in range(Wm):
        ds.ds_step(gs[t % nbuf])
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    graph = None
    if hip_graph:
        # the step counter lives on the device and the steps' kernels advance it, so the captured steps run as
        # iterations W .. W+K-1 when the graph is replayed
        graph = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                for t in range(K):
                    ds.ds_step(gs[(Wm + t) % nbuf], side)
        torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev0.record()                                            # same stream ds_step launches on
    if graph is not None:
        graph.replay()
    else:
        for t in range(K):
            ds.ds_step(gs[(Wm + t) % nbuf])
    ev1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    dev_ms = ev0.elapsed_time(ev1)
    beta = algorithmic_bytes_per_param(w)
    achieved = beta * w.worker_params / (dev_ms * 1e-3 / K) / 1e9
    entry = {
        "workload": w.name, "n": w.n, "N": w.N, "plan": ds.ds_plan_name(), "gradient_buffers": nbuf,
        "launch": "hip-graph" if graph is not None else "eager",
        "update_rule": {0: "deepsqueeze", 1: "dcd-psgd", 2: "choco-sgd"}[w.algo],
        "compressor": {1: f"quant{w.bits}b/B{w.block}", 2: f"sign/B{w.block}", 3: f"top-{w.k}", 0: "identity",
                       4: f"l2norm{w.bits}b", 5: f"rand-{w.k}", 6: f"gspar-{w.k}"}[w.kind],
        "ms_per_step": wall * 1e3 / K, "value": w.worker_params * K / wall,
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic_table.get(w.name),
                     "bytes_per_param": beta, "bytes_per_step": beta * w.worker_params,
                     "device_ms_per_step": dev_ms / K, "plain_copy_GBps": copy_gbs,
                     "frac_of_plain_copy": achieved / copy_gbs, "stream_3r2w_GBps": mix_gbs,
                     "frac_of_3r2w_stream": achieved / mix_gbs},
    }
    if w.algo == 1:        # DCD-PSGD has no second state array: its bare stream is 2 loads / 1 store
        entry["roofline"]["stream_2r1w_GBps"] = mix21_gbs
        entry["roofline"]["frac_of_2r1w_stream"] = achieved / mix21_gbs
    ds.ds_destroy()
    del gs
    torch.cuda.empty_cache()
    return entry


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=None,
                    help="time only this configuration (index into the benchmark's list; 5, 6, 7: the extra workloads)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--hip-graph", action="store_true",
                    help="capture the K timed steps into one HIP graph and time its replay (for launch-bound sizes)")
    ap.add_argument("--copy-only", action="store_true", help="run only the yardstick kernels (counter calibration)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (n simulated workers on one device); "
              "--gpus must be 1, no multi-GPU figure exists.", file=sys.stderr)
        sys.exit(2)

    import torch

    from paper_1907_07346_amd.build import ensure_built
    ensure_built()
    from paper_1907_07346_amd import binding as b
    from paper_1907_07346_amd import workloads as wl

    torch.cuda.set_device(0)
    K, Wm = args.steps, args.warmup
    copy_gbs, mix_gbs, mix21_gbs = yardsticks(torch, b)
    if args.copy_only:
        print(json.dumps({"copy_GBps": copy_gbs, "bytes_per_launch": 2 * (1 << 30), "stream_3r2w_GBps": mix_gbs, "stream_2r1w_GBps": mix21_gbs}))
        return

    traffic_table = {}
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        with open(tpath) as f:
            traffic_table = json.load(f)
    all_w = wl.configs() + wl.extra_configs()
    todo = DEFAULT_SET if args.config is None else [args.config]
    head_idx = HEADLINE if args.config is None else args.config
    entries = {}
    for idx in todo:
        # the cache-resident configuration 0 is launch-bound: more steps cost nothing and steady the figure
        entries[idx] = run_config(torch, b, wl, all_w[idx], K, Wm, args.hip_graph, copy_gbs, mix_gbs, mix21_gbs, traffic_table)
        print(f"bench: {entries[idx]['workload']}: {entries[idx]['ms_per_step']:.4f} ms/step, "
              f"{entries[idx]['roofline']['frac']:.3f} of peak", file=sys.stderr, flush=True)
    head = entries[head_idx]
    out = {
        "metric": "worker-param updates/sec and achieved HBM GB/s (% peak) per ds_step",
        "value": head["value"], "unit": "worker-param updates/s", "n_gpus": 1, "steps": K, "warmup": Wm,
        "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {k: head[k] for k in ("workload", "n", "N", "plan", "gradient_buffers", "launch", "compressor")},
        "roofline": head["roofline"],
        "configs": [entries[i] for i in todo],
        "build_id": b.lib().ds_build_id().decode(),
    }
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(all_w[head_idx])
    print(json.dumps(out))


if __name__ == "__main__":
    main()
