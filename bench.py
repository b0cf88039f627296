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
    # the backward walk with the query slice pinned streams the same chunks through the same buffers
    dQ = torch.zeros((w.B, w.H, w.Nq, w.d), device=Q.device, dtype=torch.float32)
    dKs = [torch.empty(K.shape, device=Q.device, dtype=torch.float32) for K in Ks]
    dVs = [torch.empty(K.shape, device=Q.device, dtype=torch.float32) for K in Ks]
    t_compute_b = timed(lambda: plain.backward(Ks, Vs, k_offs, inp["dO"], dQ, dKs, dVs))
    t_pipe_b = timed(lambda: db.backward(src_K, src_V, k_offs, inp["dO"], dQ, dKs, dVs))
    chunk_bytes = 2 * Ks[0].numel() * Ks[0].element_size()
    return {"source": source, "compute_only_ms": t_compute, "copies_only_ms": t_copy, "double_buffered_ms": t_pipe,
            "backward_compute_only_ms": t_compute_b, "backward_double_buffered_ms": t_pipe_b,
            "backward_compute_over_total": t_compute_b / t_pipe_b,
            "overlap_efficiency": max(t_compute, t_copy) / t_pipe,
            "compute_over_total": t_compute / t_pipe,
            # with the copies shorter than the attention, what the walk loses is what the attention
            # kernels lose to the concurrent copy traffic (and to waiting on the copy events)
            "kernel_slowdown_under_copy_traffic": t_pipe / t_compute if t_copy < t_compute else None,
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


def merge_state_measurement(w, walk, reps=12):
    """burst_merge_state is not part of a step (the chunk kernels merge in their epilogue); it is
    timed on its own, rotating over enough state copies that every launch reads and writes memory
    the 256 MB last-level cache no longer holds."""
    import torch
    from paper_2403_09347_amd import binding as B
    rows = w.B * w.H * w.Nq
    state = rows * (4 * w.d + 8)
    p = walk.params(0, 0)
    copies = max(2, min(8, -(-3 * 256 * 2**20 // (2 * state))))
    sets = []
    for _ in range(copies):
        a = (torch.empty_like(walk.O_acc), torch.empty_like(walk.m), torch.empty_like(walk.l))
        b = (torch.empty_like(walk.O_acc), torch.empty_like(walk.m), torch.empty_like(walk.l))
        for dst, src in zip(a + b, (walk.O_acc, walk.m, walk.l) * 2):      # a real state after a forward walk
            dst.copy_(src)
        sets.append((a, b))
    B.burst_merge_state(*sets[0][0], *sets[0][1], p)
    e0, e1 = B.Event(), B.Event()
    e0.record()
    for i in range(reps):
        a, b = sets[i % copies]
        B.burst_merge_state(*a, *b, p)
    e1.record()
    ms = e0.elapsed_ms_until(e1) / reps
    nbytes = 3 * state
    gbs = nbytes / (ms * 1e-3) / 1e9
    return {"avg_launch_ms": round(ms, 5), "bytes": nbytes, "GB/s": round(gbs, 1), "frac_of_8TB/s": round(gbs / 8000.0, 4),
            "note": f"standalone, {copies} rotating state pairs ({2 * copies * state / 2**20:.0f} MiB)"}


class SensorSampler:
    """Core clock and socket power of GPU 0 from sysfs while a region runs (a thread polling every
    few milliseconds).  Returns None for what the box does not expose."""

    def __init__(self, period_s=0.01):
        import glob
        self.period = period_s
        self.power = (glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_input") +
                      glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_average") + [None])[0]
        self.sclk = (glob.glob("/sys/class/drm/card*/device/pp_dpm_sclk") + [None])[0]
        self.cap = (glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_cap") + [None])[0]
        self.w, self.mhz = [], []
        self._stop = False
        self._thread = None

    def _read(self):
        try:
            if self.power:
                self.w.append(int(open(self.power).read()) / 1e6)
            if self.sclk:
                for line in open(self.sclk):
                    if line.rstrip().endswith("*"):
                        self.mhz.append(float(line.split(":")[1].lower().replace("mhz", "").replace("*", "")))
        except (OSError, ValueError, IndexError):
            pass

    def __enter__(self):
        import threading

        def loop():
            while not self._stop:
                self._read()
                time.sleep(self.period)
        self._thread = threading.Thread(target=loop, daemon=True)
        self._thread.start()
        return self

    def __exit__(self, *exc):
        self._stop = True
        self._thread.join()

    def summary(self):
        import statistics
        med = lambda v: round(statistics.median(v), 1) if v else None
        cap = None
        try:
            cap = int(open(self.cap).read()) / 1e6 if self.cap else None
        except (OSError, ValueError):
            pass
        return {"core_clock_mhz_median": med(self.mhz), "core_clock_mhz_max": max(self.mhz) if self.mhz else None,
                "socket_power_w_median": med(self.w), "socket_power_w_max": max(self.w) if self.w else None,
                "socket_power_cap_w": cap, "samples": max(len(self.w), len(self.mhz)), "nominal_clock_mhz": 2400}


def mfma_ceiling_measurement(dev, iters=40000):
    """What the matrix cores sustain with nothing else in the loop (burst_probe_mfma: 256 workgroups,
    16 independent-by-four v_mfma_f32_32x32x16_bf16 per iteration), on operands distributed like the
    workload's (N(0,1) rounded to bf16) and on constant ones; operands in registers, or the A operand
    read fresh from LDS for every MFMA / every second MFMA, which is how the attention kernels are
    fed (dK/dV: every MFMA; forward and dQ: every second).  TFLOP/s."""
    import torch
    from paper_2403_09347_amd import binding as B
    gen = torch.Generator(device=dev)
    gen.manual_seed(4242)
    normal = torch.randn(32768, generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
    ones = torch.ones(32768, device=dev, dtype=torch.bfloat16)
    sink = torch.empty(256 * 512, device=dev, dtype=torch.float32)

    def rate(lds, wps, data):
        B.burst_probe_mfma(lds, wps, data, sink, 2000)
        a, b = B.Event(), B.Event()
        a.record()
        B.burst_probe_mfma(lds, wps, data, sink, iters)
        b.record()
        return round(256 * 4 * wps * iters * 16 * 32768.0 / a.elapsed_ms_until(b) / 1e9, 1)
    out = {"unit": "TFLOP/s", "nominal_peak": PEAK_BF16_TFLOPS}
    for wps in (1, 2):
        key = f"{wps}_wavefront{'s' if wps > 1 else ''}_per_simd"
        out[key] = {
            "constant_operands_in_registers": rate(0, wps, ones),
            "normal_operands_in_registers": rate(0, wps, normal),
            "normal_operands_A_from_lds_every_2nd_mfma": rate(2, wps, normal),
            "normal_operands_A_from_lds_every_mfma": rate(1, wps, normal),
        }
    return out


def fused_backward_floor_measurement(w, dev):
    """Lower bound for a backward that computes each block pair once (five contractions instead of the
    seven of the two-kernel form): with the keys stationary its dQ partial sums leave every
    128-key workgroup through fp32 atomic adds, B*H*Nq*d*(Nc/128) of them per block pair.
    burst_probe_atomic_dq issues exactly those adds and nothing else; also the same pattern as plain
    stores and as plain load-add-store (what workgroups that took turns on a tile under a lock would
    issue: the memory time alone, without the locks, and not reproducible bit for bit)."""
    import torch
    from paper_2403_09347_amd import binding as B
    heads = (w.B * w.H + 7) // 8 * 8
    dq = torch.zeros(heads * w.Nq * 128, device=dev, dtype=torch.float32)
    out = {}
    for name, atomic in (("atomic_adds_ms", 1), ("plain_stores_same_pattern_ms", 0),
                         ("plain_read_modify_write_same_pattern_ms", 2)):
        B.burst_probe_atomic_dq(dq, heads, w.Nq, w.Nc // 128, atomic)
        best = 1e30
        for _ in range(3):
            a, b = B.Event(), B.Event()
            a.record()
            B.burst_probe_atomic_dq(dq, heads, w.Nq, w.Nc // 128, atomic)
            b.record()
            best = min(best, a.elapsed_ms_until(b))
        out[name] = round(best, 4)
    n = heads * w.Nq * 128 * (w.Nc // 128)
    out["adds_per_block_pair"] = n
    out["atomic_rate_G_per_s"] = round(n / out["atomic_adds_ms"] / 1e6, 1)
    return out


def block_sparse_measurement(w, inp, dev):
    """Sec. 2.6 on the headline block pair: one forward, dQ and dK/dV launch each (first chunk of the
    workload) under seeded random block flags, ms per launch (best of 3 rounds of 8 launches), dense
    through the same entry points beside them.  Time that follows the density is the point: tiles
    that the flags hide are skipped, not masked."""
    import torch
    from paper_2403_09347_amd import binding as B
    from paper_2403_09347_amd import workloads
    Q, K, V, dO = inp["Q"], inp["K"][0], inp["V"][0], inp["dO"]
    lse = torch.full((w.B, w.H, w.Nq), 8.0, device=dev)
    D = torch.zeros((w.B, w.H, w.Nq), device=dev)
    dQ = torch.zeros((w.B, w.H, w.Nq, w.d), device=dev)
    dK = torch.empty((w.B, w.H, w.Nc, w.d), device=dev)
    dV = torch.empty_like(dK)
    O = torch.zeros_like(dQ)
    m = torch.full((w.B, w.H, w.Nq), -float("inf"), device=dev)
    l = torch.zeros((w.B, w.H, w.Nq), device=dev)

    def launches(p):
        return {"fwd_ms": lambda: B.burst_local_fwd(Q, K, V, O, m, l, p),
                "dq_ms": lambda: B.burst_local_bwd_dq(Q, K, V, dO, lse, D, dQ, p, False),
                "dkv_ms": lambda: B.burst_local_bwd_dkv(Q, K, V, dO, lse, D, dK, dV, p)}

    def timed(fn):
        for _ in range(4):
            fn()
        best = 1e30
        for _ in range(3):
            a, b = B.Event(), B.Event()
            a.record()
            for _ in range(8):
                fn()
            b.record()
            best = min(best, a.elapsed_ms_until(b) / 8)
        return round(best, 4)

    out = {"note": "per launch, first chunk of the workload; random block flags, seed 3",
           "dense": {k: timed(fn) for k, fn in launches(
               B.params(w.B, w.H, w.Nq, w.Nc, w.d, torch.bfloat16, w.scale)).items()}}
    for block, density in ((64, 0.5), (64, 0.25), (256, 0.5)):
        flags = workloads.block_flags(w.Nq // block, w.Nc // block, "random", density=density, seed=3)
        mask = torch.from_numpy(flags).to(dev).contiguous()
        p = B.params(w.B, w.H, w.Nq, w.Nc, w.d, torch.bfloat16, w.scale, block_mask=mask, block=block)
        r = {k: timed(fn) for k, fn in launches(p).items()}
        r["density"] = round(float(flags.mean()), 3)
        out[f"block{block}_density{density}"] = r
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


def measure_workload(w, dev, steps, warmup, detailed, zero_inputs=False):
    """Times `steps` steps of workload w (after `warmup` untimed ones).  Returns the figures of the
    JSON line; with `detailed` also the inputs and the walk for the follow-up measurements.
    zero_inputs: the same launches on all-zero Q, K, V, dO (a diagnostic: the instruction stream is
    the same, the matrix cores' operands toggle no bits)."""
    import statistics
    import torch
    from paper_2403_09347_amd import binding as B
    from paper_2403_09347_amd import workloads
    from paper_2403_09347_amd.harness import RingWalk

    inp = workloads.make_inputs(w, dev)
    Q, Ks, Vs, dO = inp["Q"], inp["K"], inp["V"], inp["dO"]
    if zero_inputs:
        for t in [Q, dO] + Ks + Vs:
            t.zero_()
    k_offs = [w.k_off(j) for j in range(w.G)]
    walk = RingWalk(Q, w.scale, w.causal, w.q_off)
    dQ = torch.zeros((w.B, w.H, w.Nq, w.d), device=dev, dtype=torch.float32)
    dKs = [torch.empty((w.B, w.H, w.Nc, w.d), device=dev, dtype=torch.float32) for _ in range(w.G)]
    dVs = [torch.empty_like(x) for x in dKs]

    names = ("init", "fwd", "finalize", "prepare", "zero_dq", "dq", "dkv")
    ev = {k: [] for k in names}
    step_ev = []

    def step(timed):
        # Every launch of a timed step lies between two events on the launch stream; consecutive
        # launches share one (the end of one is the start of the next), so the stream is never idle
        # between them and a step records 5 + 3 G events.
        def mark():
            e = B.Event()
            e.record()
            return e

        def after(kind, prev):
            if not timed:
                return None
            cur = mark()
            ev[kind].append((prev, cur))
            return cur
        first = prev = mark() if timed else None
        walk.init()
        prev = after("init", prev)
        for j in range(w.G):
            walk.step(Ks[j], Vs[j], k_offs[j])
            prev = after("fwd", prev)
        walk.finalize()
        prev = after("finalize", prev)
        walk.prepare(dO)
        prev = after("prepare", prev)
        dQ.zero_()
        prev = after("zero_dq", prev)
        for j in range(w.G):
            p = walk.params(w.Nc, k_offs[j])
            B.burst_local_bwd_dq(Q, Ks[j], Vs[j], dO, walk.lse, walk.D, dQ, p, True)
            prev = after("dq", prev)
            B.burst_local_bwd_dkv(Q, Ks[j], Vs[j], dO, walk.lse, walk.D, dKs[j], dVs[j], p, False)
            prev = after("dkv", prev)
        if timed:
            step_ev.append((first, prev))

    for _ in range(warmup):
        step(False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step(True)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / steps
    step_ms = [a.elapsed_ms_until(b) for a, b in step_ev]

    avg = {k: sum(a.elapsed_ms_until(b) for a, b in v) / len(v) for k, v in ev.items()}
    res = {"w": w, "ms_per_step": ms_per_step, "step_ms_median": statistics.median(step_ms), "step_ms_min": min(step_ms),
           "avg": avg, "value": (w.fwd_flops() + w.bwd_flops()) / (ms_per_step * 1e-3) / 1e12}
    if detailed:
        res.update(inp=inp, walk=walk, step=step)
    return res


def brief(res):
    """One workload's figures for the 'other_workloads' list."""
    w, avg = res["w"], res["avg"]
    fwd_ms, bwd_ms = avg["fwd"] * w.G, (avg["dq"] + avg["dkv"]) * w.G
    return {"workload": w.name, "ms_per_step": round(res["ms_per_step"], 3),
            "ms_per_step_median": round(res["step_ms_median"], 3), "ms_per_step_min": round(res["step_ms_min"], 3),
            "tflops": round(res["value"], 1), "pct_of_bf16_peak": round(100.0 * res["value"] / PEAK_BF16_TFLOPS, 2),
            "fwd_tflops": round(w.fwd_flops() / (fwd_ms * 1e-3) / 1e12, 1),
            "bwd_tflops": round(w.bwd_flops() / (bwd_ms * 1e-3) / 1e12, 1)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="llama7b_32k_G8")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--brief", action="store_true",
                    help="only the timed steps of --workload: no ceiling probes, no other workloads, no overlap "
                         "measurement, no oracle timing (for profiler runs)")
    ap.add_argument("--overlap", choices=["hbm", "pinned_host"], default="hbm",
                    help="source pool of the double-buffered chunk walk's copies (paper Sec. 2.5): chunks are copied "
                         "from a pool of that kind into two receive buffers on a second stream while the previous "
                         "chunk computes; reported as the 'overlap' object of the JSON line")
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

    B.load()                                   # fails loudly if the HIP library is missing
    dev = "cuda:0"
    torch.cuda.set_device(0)
    w = workloads.by_name(args.workload)
    if args.calibration_copy:
        src = torch.ones(64 * 1024 * 1024, device=dev, dtype=torch.float32)
        for _ in range(3):
            dst = src * 1.0                    # one elementwise kernel: reads 256 MiB, writes 256 MiB
        del src, dst

    res = measure_workload(w, dev, args.steps, args.warmup, detailed=True)
    avg, walk, inp = res["avg"], res["walk"], res["inp"]
    ms_per_step, value = res["ms_per_step"], res["value"]
    pairs_launch = float(w.visible_pairs_per_head()) / w.G * w.H * w.B      # per chunk call (non-causal: equal)
    gemm_flop = 2.0 * pairs_launch * w.d                                    # one contraction of a block pair
    # contractions each kernel executes per launch: fwd 2, dq 3 (S, dP, dQ), dkv 4 (S, dP, dV, dK);
    # Alg. 2 counts five for the pair (S and dP once), so the two backward kernels together are
    # credited 5 of the 7 they execute.
    gemms = {"fwd": 2, "dq": 3, "dkv": 4}
    kern = {k: {"avg_ms": avg[k], "tflops": gemms[k] * gemm_flop / (avg[k] * 1e-3) / 1e12} for k in gemms}
    dom = max(gemms, key=lambda k: avg[k])
    names = {"fwd": "burst_fwd_mfma_kernel", "dq": "burst_bwd_dq_kernel", "dkv": "burst_bwd_dkv_kernel"}
    if w.d == 64:
        names = {"fwd": "d64::burst_fwd_d64_kernel", "dq": "d64::burst_bwd_dq_d64_kernel", "dkv": "d64::burst_bwd_dkv_d64_kernel"}
    elif B.burst_kernel_family_for(walk.params(w.Nc, 0)) == 2:     # the 128-row kernels serve this shape
        names.update(fwd="d128p::burst_fwd_d64_kernel", dq="d128p::burst_bwd_dq_d64_kernel")
    pair_ms = avg["dq"] + avg["dkv"]
    pair_counted = 5 * gemm_flop / (pair_ms * 1e-3) / 1e12
    roofline = {"bound": "mfma", "kernel": names[dom], "achieved": kern[dom]["tflops"], "peak": PEAK_BF16_TFLOPS,
                "unit": "TFLOP/s", "frac": kern[dom]["tflops"] / PEAK_BF16_TFLOPS,
                "frac_note": "executed contractions of that kernel (S and dP are computed in both backward kernels); "
                             "frac_counted credits the backward pair with Alg. 2's five contractions",
                "frac_counted": pair_counted / PEAK_BF16_TFLOPS,
                "backward_pair": {"kernels": [names["dq"], names["dkv"]], "avg_ms": round(pair_ms, 4),
                                  "executed_tflops": round(7 * gemm_flop / (pair_ms * 1e-3) / 1e12, 1),
                                  "counted_tflops": round(pair_counted, 1),
                                  "frac_counted": round(pair_counted / PEAK_BF16_TFLOPS, 4)},
                "step_frac_counted": value / PEAK_BF16_TFLOPS,
                "traffic": measured_traffic(names[dom], w.name),
                "avg_launch_ms": avg[dom],
                "all_kernels": {names[k]: {"avg_launch_ms": round(kern[k]["avg_ms"], 4),
                                           "tflops": round(kern[k]["tflops"], 1),
                                           "frac": round(kern[k]["tflops"] / PEAK_BF16_TFLOPS, 4)} for k in kern}}

    fwd_ms = avg["fwd"] * w.G
    bwd_ms = (avg["dq"] + avg["dkv"]) * w.G
    out = {
        "metric": "local-attn fwd+bwd TFLOP/s & % bf16 MFMA peak, 7B-shape 32K/G=8 share",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "ms_per_step_median": res["step_ms_median"], "ms_per_step_min": res["step_ms_min"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if w.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"{w.name}: B={w.B} H={w.H} d={w.d} Nq={w.Nq} G={w.G} Nc={w.Nc} "
                               f"{w.dtype} {'causal' if w.causal else 'non-causal'}, fp32 accumulate"},
        "pct_of_bf16_peak": 100.0 * value / PEAK_BF16_TFLOPS,
        "fwd_tflops": w.fwd_flops() / (fwd_ms * 1e-3) / 1e12,
        "bwd_tflops": w.bwd_flops() / (bwd_ms * 1e-3) / 1e12,
        "fwd_kernels_ms": fwd_ms, "bwd_kernels_ms": bwd_ms,
        "roofline": roofline,
    }
    # the HBM-bound steps, as they ran inside the timed steps (one launch each per step)
    es = 2 if w.dtype == "bf16" else 4
    rows = w.B * w.H * w.Nq
    state = rows * (4 * w.d + 8)
    hbm_bytes = {"init": ("state_init", state), "finalize": ("finalize", state + rows * (es * w.d + 4)),
                 "prepare": ("bwd_prepare", rows * (2 * es * w.d + 4)), "zero_dq": ("zero_fill_dQ", rows * 4 * w.d)}
    out["hbm_steps"] = {"timing": "events around each launch inside the timed steps"}
    for k, (name, nbytes) in hbm_bytes.items():
        gbs = nbytes / (avg[k] * 1e-3) / 1e9
        out["hbm_steps"][name] = {"avg_launch_ms": round(avg[k], 5), "bytes": nbytes, "GB/s": round(gbs, 1),
                                  "frac_of_8TB/s": round(gbs / 8000.0, 4)}
    if not args.brief:
        out["hbm_steps"]["merge_state"] = merge_state_measurement(w, walk)
        # clock and power while the same steps keep running (untimed), about one second
        with SensorSampler() as sensors:
            t_end = time.perf_counter() + 1.0
            while time.perf_counter() < t_end:
                res["step"](False)
                torch.cuda.synchronize()
        out["sensors_under_load"] = sensors.summary()
        out["mfma_ceiling"] = mfma_ceiling_measurement(dev)
        ceil1 = out["mfma_ceiling"]["1_wavefront_per_simd"]
        out["mfma_ceiling"]["executed_vs_ceiling"] = {
            names[k]: round(kern[k]["tflops"] / ceil1["normal_operands_A_from_lds_every_mfma" if k == "dkv" else
                                                       "normal_operands_A_from_lds_every_2nd_mfma"], 3) for k in kern}
        if w.d == 128 and w.Nq % 64 == 0 and w.Nc % 128 == 0:
            floor = fused_backward_floor_measurement(w, dev)
            floor["two_kernel_backward_ms"] = round(pair_ms, 4)
            floor["two_kernel_minus_recomputed_contractions_ms"] = round(pair_ms * 5.0 / 7.0, 4)
            out["fused_backward_floor"] = floor
        out["overlap"] = overlap_measurement(w, inp, args.overlap, max(3, args.steps // 2))
        if w.d == 128 and not w.causal and w.Nq % 256 == 0 and w.Nc % 256 == 0:
            out["block_sparse"] = block_sparse_measurement(w, inp, dev)
    if args.graph:
        out["graph"] = graph_measurement(w, inp, max(20, args.steps))
    if args.ablation:
        out["ablation"] = ablation_measurement(w, inp, max(3, args.steps // 2))
    if not args.no_cpu_baseline and not args.brief:
        out["cpu_baseline"] = cpu_baseline(w, inp)
    del res, walk, inp
    torch.cuda.empty_cache()
    if not args.brief:
        # the same steps on all-zero inputs: same instruction stream, operands that toggle no bits
        # (how much of the step time is the power limit's, i.e. the clock the data allows)
        r = measure_workload(w, dev, 5, 2, detailed=False, zero_inputs=True)
        out["same_steps_on_zero_inputs"] = {"ms_per_step_median": round(r["step_ms_median"], 3),
                                            "speedup_over_normal_inputs": round(out["ms_per_step_median"] / r["step_ms_median"], 3),
                                            "kernels_avg_launch_ms": {k: round(r["avg"][k], 4) for k in ("fwd", "dq", "dkv")}}
        del r
        torch.cuda.empty_cache()
    if not args.brief and args.workload == "llama7b_32k_G8":
        # the benchmark's other configurations, a few steps each (same step definition)
        out["other_workloads"] = []
        for other, n in ((workloads.WORKLOADS[2], 5), (workloads.WORKLOADS[3], 3), (workloads.WORKLOADS[4], 2)):
            r = measure_workload(other, dev, n, 1, detailed=False)
            out["other_workloads"].append(brief(r))
            del r
            torch.cuda.empty_cache()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
