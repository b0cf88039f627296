#!/usr/bin/env python3
"""Benchmark of the local-attention hot path on one MI355X.

A "step" is one pass of the whole path over one batch of synthetic input:
forward  = state_init + G x local_fwd + finalize            (paper Alg. 1)
backward = bwd_prepare + G x (local_bwd_dq + local_bwd_dkv)  (paper Alg. 2)
with all G key/value chunks already resident in HBM.  Prints ONE JSON line.

Throughput counts 4*pairs*d*H FLOP forward and 2.5x that backward (pairs = unmasked
query-key pairs per head), whatever the kernels actually execute.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2516.6      # MI355X dense bf16 MFMA peak: 256 CU x 4096 FLOP/clk x 2.4 GHz


def cpu_baseline(w, inputs, budget_s=15.0, max_heads=8):
    """Times the fp64 oracle (as it stands) on a bounded sample: complete heads (forward +
    backward, every output element), as many as fit in about `budget_s` seconds."""
    import numpy as np
    import torch
    from oracle import burst_oracle as orc
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    f64 = lambda t: t.detach().double().cpu().numpy()
    qp = w.q_off + np.arange(w.Nq)
    dt, heads = 0.0, 0
    for h in range(min(w.H, max_heads)):
        Q, dO = f64(inputs["Q"][0, h]), f64(inputs["dO"][0, h])
        K = np.concatenate([f64(k[0, h]) for k in inputs["K"]])
        V = np.concatenate([f64(v[0, h]) for v in inputs["V"]])
        kp = np.arange(K.shape[0])
        t0 = time.perf_counter()
        orc.full_forward(Q, K, V, w.scale, w.causal, qp, kp)
        orc.full_backward(Q, K, V, dO, w.scale, w.causal, qp, kp)
        dt += time.perf_counter() - t0
        heads += 1
        if dt * (heads + 1) / heads > budget_s:
            break
    flops = heads * 3.5 * 4.0 * w.visible_pairs_per_head() * w.d   # counted fwd + bwd FLOP of the sample
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": int(threads), "kind": "oracle",
            "sample": f"{heads} of {w.H} heads, complete fp64 forward+backward ({dt:.1f} s)"}


def overlap_measurement(w, inp, source, reps):
    """Forward walk of the workload three ways: chunks resident (compute only), the chunk copies
    alone, and the double-buffered walk that overlaps them.  Times in ms, median of `reps`."""
    import statistics
    import torch
    from paper_2403_09347_amd.harness import DoubleBufferedWalk, RingWalk
    Q, Ks, Vs = inp["Q"], inp["K"], inp["V"]
    k_offs = [w.k_off(j) for j in range(w.G)]
    if source == "pinned_host":
        src_K = [k.cpu().pin_memory() for k in Ks]
        src_V = [v.cpu().pin_memory() for v in Vs]
    else:
        src_K, src_V = Ks, Vs
    plain = RingWalk(Q, w.scale, w.causal, w.q_off)
    db = DoubleBufferedWalk(Q, w.scale, w.causal, w.q_off, max_chunk_rows=w.Nc)

    def timed(fn):
        ts = []
        for _ in range(reps + 1):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            fn()
            torch.cuda.synchronize()
            ts.append((time.perf_counter() - t0) * 1e3)
        return statistics.median(ts[1:])
    t_compute = timed(lambda: plain.forward(Ks, Vs, k_offs))
    t_copy = timed(lambda: db.copies_only(src_K, src_V))
    t_pipe = timed(lambda: db.forward(src_K, src_V, k_offs))
    chunk_bytes = 2 * Ks[0].numel() * Ks[0].element_size()
    return {"source": source, "compute_only_ms": t_compute, "copies_only_ms": t_copy, "double_buffered_ms": t_pipe,
            "overlap_efficiency": max(t_compute, t_copy) / t_pipe,
            "copy_GBps": w.G * chunk_bytes / (t_copy * 1e-3) / 1e9, "chunk_MiB": chunk_bytes / 2**20}


def ablation_measurement(w, inp, reps):
    """Forward and backward walks of the workload with the tiled chunk steps and with the steps that
    store the matrices of a block pair in HBM (the paper's "w/o LAO" ablation, Tables 2-3).  Times
    in ms, median of `reps`; memory is the workspace one chunk step needs on top of the inputs and
    the state."""
    import statistics
    import torch
    from paper_2403_09347_amd.harness import MaterializedWalk, RingWalk
    Q, Ks, Vs = inp["Q"], inp["K"], inp["V"]
    k_offs = [w.k_off(j) for j in range(w.G)]
    tiled = RingWalk(Q, w.scale, w.causal, w.q_off)
    stored = MaterializedWalk(Q, w.scale, w.causal, w.q_off, max_chunk_rows=w.Nc)

    def timed(fn):
        ts = []
        for _ in range(reps + 1):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            fn()
            torch.cuda.synchronize()
            ts.append((time.perf_counter() - t0) * 1e3)
        return statistics.median(ts[1:])
    t_tiled = timed(lambda: tiled.forward(Ks, Vs, k_offs))
    t_stored = timed(lambda: stored.forward(Ks, Vs, k_offs))
    fwd_ws = stored.workspace.numel() / 2**20
    dQ = torch.zeros(Q.shape, device=Q.device, dtype=torch.float32)
    dKs = [torch.empty(K.shape, device=Q.device, dtype=torch.float32) for K in Ks]
    dVs = [torch.empty(K.shape, device=Q.device, dtype=torch.float32) for K in Ks]
    t_tiled_b = timed(lambda: tiled.backward(Ks, Vs, k_offs, inp["dO"], dQ, dKs, dVs))
    stored.O, stored.lse = tiled.O, tiled.lse
    t_stored_b = timed(lambda: stored.backward(Ks, Vs, k_offs, inp["dO"], dQ, dKs, dVs))
    return {"tiled_forward_ms": t_tiled, "stored_forward_ms": t_stored, "slowdown": t_stored / t_tiled,
            "tiled_backward_ms": t_tiled_b, "stored_backward_ms": t_stored_b, "backward_slowdown": t_stored_b / t_tiled_b,
            "stored_workspace_MiB": fwd_ws, "stored_backward_workspace_MiB": stored.workspace.numel() / 2**20,
            "tiled_workspace_MiB": 0.0,
            "inputs_and_state_MiB": (Q.numel() * Q.element_size() * (1 + 2 * len(Ks)) + tiled.O_acc.numel() * 4
                                     + 2 * tiled.m.numel() * 4) / 2**20}


def hbm_step_measurement(w, walk, dO, reps=20):
    """The HBM-bound steps of the path (Alg. 1 initialisation, merge and last two steps; Alg. 2's D)
    one by one: `reps` launches between two events on the launch stream, algorithmic bytes per
    launch over the average duration, against the 8 TB/s peak.  The launches of one step run back
    to back on the same buffers, so the last-level cache may serve part of the traffic."""
    import torch
    from paper_2403_09347_amd import binding as B
    es = 2 if w.dtype == "bf16" else 4
    rows = w.B * w.H * w.Nq
    state = rows * (4 * w.d + 8)
    other = (torch.empty_like(walk.O_acc), torch.empty_like(walk.m), torch.empty_like(walk.l))
    p = walk.params(0, 0)
    B.burst_state_init(*other, p)
    steps = {
        "state_init": (lambda: B.burst_state_init(*other, p), state),
        "merge_state": (lambda: B.burst_merge_state(*other, walk.O_acc, walk.m, walk.l, p), 3 * state),
        "finalize": (lambda: walk.finalize(), state + rows * (es * w.d + 4)),
        "bwd_prepare": (lambda: walk.prepare(dO), rows * (2 * es * w.d + 4)),
    }
    out = {}
    for name, (fn, nbytes) in steps.items():
        fn()
        a, b = B.Event(), B.Event()
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        ms = a.elapsed_ms_until(b) / reps
        gbs = nbytes / (ms * 1e-3) / 1e9
        out[name] = {"avg_launch_ms": round(ms, 5), "bytes": nbytes, "GB/s": round(gbs, 1), "frac_of_8TB/s": round(gbs / 8000.0, 4)}
    return out


def graph_measurement(w, inp, reps):
    """The same step recorded once as a HIP graph and replayed (one launch per step) against the
    eager step (one launch per kernel): wall-clock ms per step over `reps` steps each."""
    import torch
    from paper_2403_09347_amd.harness import GraphedStep, RingWalk
    k_offs = [w.k_off(j) for j in range(w.G)]
    walk = RingWalk(inp["Q"], w.scale, w.causal, w.q_off)
    step = GraphedStep(walk, inp["K"], inp["V"], k_offs, inp["dO"])

    def timed(fn):
        fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / reps
    eager, graph = timed(step._run), timed(step.replay)
    return {"eager_ms_per_step": eager, "graph_ms_per_step": graph, "speedup": eager / graph}


def measured_traffic(kernel, workload):
    """HBM bytes per launch from the committed rocprofv3 FETCH_SIZE / WRITE_SIZE summary (None if absent)."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{workload}.txt")
    try:
        for line in open(path):
            f = line.split()
            if len(f) == 4 and f[0] == "traffic_bytes_per_launch" and f[1] == kernel and f[2] == workload:
                return int(f[3])
    except OSError:
        pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="llama7b_32k_G8")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--overlap", choices=["hbm", "pinned_host"], default=None,
                    help="also time the double-buffered chunk walk (paper Sec. 2.5): chunks are copied from a source "
                         "pool of that kind into two receive buffers on a second stream while the previous chunk "
                         "computes; adds an 'overlap' object to the JSON line")
    ap.add_argument("--ablation", action="store_true",
                    help="also time the forward and backward walks with the chunk steps that store S_ij, P_ij, dP_ij, dS_ij in HBM "
                         "(the paper's 'w/o LAO' ablation); adds an 'ablation' object to the JSON line")
    ap.add_argument("--graph", action="store_true",
                    help="also record the step as one HIP graph and time its replays against the eager step; "
                         "adds a 'graph' object to the JSON line")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also launch a plain elementwise copy kernel of known size (256 MiB read, 256 MiB "
                         "written) so that HBM counters of a profiler run can be scaled")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU's share of the ring; run with --gpus 1 "
              "(no collectives or multi-GPU path exist here)", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2403_09347_amd import binding as B
    from paper_2403_09347_amd import workloads
    from paper_2403_09347_amd.harness import RingWalk

    B.load()                                   # fails loudly if the HIP library is missing
    dev = "cuda:0"
    torch.cuda.set_device(0)
    w = workloads.by_name(args.workload)
    inp = workloads.make_inputs(w, dev)
    Q, Ks, Vs, dO = inp["Q"], inp["K"], inp["V"], inp["dO"]
    k_offs = [w.k_off(j) for j in range(w.G)]
    walk = RingWalk(Q, w.scale, w.causal, w.q_off)
    dQ = torch.zeros((w.B, w.H, w.Nq, w.d), device=dev, dtype=torch.float32)
    dKs = [torch.empty((w.B, w.H, w.Nc, w.d), device=dev, dtype=torch.float32) for _ in range(w.G)]
    dVs = [torch.empty_like(x) for x in dKs]

    ev = {k: [] for k in ("fwd", "dq", "dkv")}

    def step(timed):
        # Consecutive MFMA-kernel launches share one event (end of one = start of the next), so a
        # timed step records 26 events instead of 48; the stream is never idle between them.
        def mark():
            e = B.Event()
            e.record()
            return e
        walk.init()
        prev = mark() if timed else None
        for j in range(w.G):
            walk.step(Ks[j], Vs[j], k_offs[j])
            if timed:
                cur = mark()
                ev["fwd"].append((prev, cur))
                prev = cur
        walk.finalize()
        walk.prepare(dO)
        dQ.zero_()
        prev = mark() if timed else None
        for j in range(w.G):
            p = walk.params(w.Nc, k_offs[j])
            B.burst_local_bwd_dq(Q, Ks[j], Vs[j], dO, walk.lse, walk.D, dQ, p, True)
            if timed:
                cur = mark()
                ev["dq"].append((prev, cur))
                prev = cur
            B.burst_local_bwd_dkv(Q, Ks[j], Vs[j], dO, walk.lse, walk.D, dKs[j], dVs[j], p, False)
            if timed:
                cur = mark()
                ev["dkv"].append((prev, cur))
                prev = cur

    if args.calibration_copy:
        src = torch.ones(64 * 1024 * 1024, device=dev, dtype=torch.float32)
        for _ in range(3):
            dst = src * 1.0                    # one elementwise kernel: reads 256 MiB, writes 256 MiB
        del src, dst
    for _ in range(args.warmup):
        step(False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(True)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    avg = {k: sum(a.elapsed_ms_until(b) for a, b in v) / len(v) for k, v in ev.items()}
    pairs_launch = float(w.visible_pairs_per_head()) / w.G * w.H * w.B      # per chunk call (non-causal: equal)
    # contraction FLOP each kernel performs per launch: fwd 2 GEMMs, dq 3, dkv 4 (2*pairs*d each)
    gemms = {"fwd": 2, "dq": 3, "dkv": 4}
    kern = {k: {"avg_ms": avg[k], "tflops": gemms[k] * 2.0 * pairs_launch * w.d / (avg[k] * 1e-3) / 1e12}
            for k in avg}
    dom = max(avg, key=lambda k: avg[k])
    names = {"fwd": "burst_fwd_mfma_kernel", "dq": "burst_bwd_dq_kernel", "dkv": "burst_bwd_dkv_kernel"}
    if w.d == 64:
        names = {"fwd": "d64::burst_fwd_d64_kernel", "dq": "d64::burst_bwd_dq_d64_kernel", "dkv": "d64::burst_bwd_dkv_d64_kernel"}
    elif B.burst_kernel_family_for(walk.params(w.Nc, 0)) == 2:     # the 128-row kernels serve this shape
        names.update(fwd="d128p::burst_fwd_d64_kernel", dq="d128p::burst_bwd_dq_d64_kernel")
    roofline = {"bound": "mfma", "kernel": names[dom], "achieved": kern[dom]["tflops"], "peak": PEAK_BF16_TFLOPS,
                "unit": "TFLOP/s", "frac": kern[dom]["tflops"] / PEAK_BF16_TFLOPS,
                "traffic": measured_traffic(names[dom], w.name),
                "avg_launch_ms": avg[dom],
                "all_kernels": {names[k]: {"avg_launch_ms": round(kern[k]["avg_ms"], 4),
                                           "tflops": round(kern[k]["tflops"], 1),
                                           "frac": round(kern[k]["tflops"] / PEAK_BF16_TFLOPS, 4)} for k in kern}}

    total_flops = w.fwd_flops() + w.bwd_flops()
    value = total_flops / (ms_per_step * 1e-3) / 1e12
    fwd_ms = avg["fwd"] * w.G
    bwd_ms = (avg["dq"] + avg["dkv"]) * w.G
    out = {
        "metric": "local-attn fwd+bwd TFLOP/s & % bf16 MFMA peak, 7B-shape 32K/G=8 share",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if w.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"{w.name}: B={w.B} H={w.H} d={w.d} Nq={w.Nq} G={w.G} Nc={w.Nc} "
                               f"{w.dtype} {'causal' if w.causal else 'non-causal'}, fp32 accumulate"},
        "pct_of_bf16_peak": 100.0 * value / PEAK_BF16_TFLOPS,
        "fwd_tflops": w.fwd_flops() / (fwd_ms * 1e-3) / 1e12,
        "bwd_tflops": w.bwd_flops() / (bwd_ms * 1e-3) / 1e12,
        "fwd_kernels_ms": fwd_ms, "bwd_kernels_ms": bwd_ms,
        "roofline": roofline,
    }
    out["hbm_steps"] = hbm_step_measurement(w, walk, dO)
    if args.overlap:
        out["overlap"] = overlap_measurement(w, inp, args.overlap, max(3, args.steps // 2))
    if args.graph:
        out["graph"] = graph_measurement(w, inp, max(20, args.steps))
    if args.ablation:
        out["ablation"] = ablation_measurement(w, inp, max(3, args.steps // 2))
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, inp)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
