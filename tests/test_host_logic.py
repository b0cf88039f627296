"""Host-side logic that needs no GPU: workload table, FLOP accounting, bench argument handling."""
import json
import math
import os
import subprocess
import sys

import numpy as np
import pytest

from paper_2403_09347_amd import workloads

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_workload_table_matches_the_benchmark_configurations():
    names = [w.name for w in workloads.WORKLOADS]
    assert len(names) == 5 and len(set(names)) == 5
    w0, w1, w2, w3, w4 = workloads.WORKLOADS
    assert (w0.H, w0.d, w0.Nq, w0.G, w0.Nc, w0.dtype, w0.causal) == (1, 64, 256, 4, 256, "f32", False)
    assert (w1.H, w1.d, w1.Nq, w1.G, w1.Nc, w1.dtype, w1.causal) == (32, 128, 4096, 8, 4096, "bf16", False)
    assert (w2.G, w2.causal, w2.q_off) == (32, True, 31 * 4096)
    assert (w3.H, w3.Nq, w3.G * w3.Nc) == (40, 16384, 131072)
    assert (w4.Nq, w4.G * w4.Nc) == (32768, 1 << 20)
    assert all(abs(w.scale - 1 / math.sqrt(w.d)) < 1e-12 for w in workloads.WORKLOADS)


def test_flop_accounting():
    w1 = workloads.by_name("llama7b_32k_G8")
    assert w1.visible_pairs_per_head() == 4096 * 32768
    assert abs(w1.fwd_flops() - 2.199e12) / 2.199e12 < 1e-3
    assert abs(w1.fwd_flops() + w1.bwd_flops() - 7.697e12) / 7.697e12 < 1e-3
    w2 = workloads.by_name("llama7b_128k_G32_rank31_causal")
    # rank 31 sees 31 full chunks plus the lower triangle (diagonal included) of its own
    assert w2.visible_pairs_per_head() == 4096 * 126976 + 4096 * 4097 // 2
    # brute force on a small causal case
    small = workloads.Workload("s", 1, 1, 8, 5, 2, 4, "f32", True, 2, 0)
    vis = sum(1 for r in range(5) for c in range(8) if c <= 2 + r)
    assert small.visible_pairs_per_head() == vis


def test_inputs_are_seeded_and_rounded_once():
    w0 = workloads.WORKLOADS[0]
    a = workloads.make_inputs(w0, "cpu")
    b = workloads.make_inputs(w0, "cpu")
    assert all((x == y).all() for x, y in zip(a["K"], b["K"])) and (a["Q"] == b["Q"]).all()
    c = workloads.make_case(1, 2, 128, 10, [3, 4], "bf16", seed=1)
    assert c["Q"].dtype.__str__() == "torch.bfloat16" and c["k_offs"] == [0, 3]
    assert abs(float(a["Q"].double().std()) - 1.0) < 0.05


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in r.stderr


def test_bench_reads_measured_traffic_from_profiles():
    sys.path.insert(0, ROOT)
    import bench
    assert bench.measured_traffic("no_such_kernel", "llama7b_32k_G8") is None
    v = bench.measured_traffic("burst_bwd_dkv_kernel", "llama7b_32k_G8")
    assert v is None or v > 100e6


def test_zigzag_assignment_balances_causal_work():
    N, G = 131072, 32
    contiguous = [workloads.causal_pairs(workloads.contiguous_spans(N, G, r), N) for r in range(G)]
    zigzag = [workloads.causal_pairs(workloads.zigzag_spans(N, G, r), N) for r in range(G)]
    assert sum(contiguous) == sum(zigzag) == N * (N + 1) // 2
    assert max(contiguous) > 60 * min(contiguous)              # rank 31 does 63x the work of rank 0
    assert max(zigzag) == min(zigzag)                          # every rank does the same
    # the spans tile the sequence exactly once
    covered = sorted(span for r in range(G) for span in workloads.zigzag_spans(N, G, r))
    assert covered == [(i * (N // (2 * G)), N // (2 * G)) for i in range(2 * G)]
    # brute-force count on a small case
    spans = workloads.zigzag_spans(64, 4, 1)
    brute = sum(1 for first, rows in spans for q in range(first, first + rows) for k in range(64) if k <= q)
    assert workloads.causal_pairs(spans, 64) == brute


def test_block_flag_generators_are_seeded_and_shaped():
    a = workloads.block_flags(5, 9, "random", density=0.3, seed=4)
    b = workloads.block_flags(5, 9, "random", density=0.3, seed=4)
    assert a.shape == (5, 9) and a.dtype == np.uint8 and np.array_equal(a, b)
    assert not np.array_equal(a, workloads.block_flags(5, 9, "random", density=0.3, seed=5))
    assert workloads.block_flags(4, 4, "random", density=0.0).sum() == 0
    band = workloads.block_flags(6, 6, "band")
    assert all(band[i, j] == (abs(i - j) <= 1) for i in range(6) for j in range(6))
    shifted = workloads.block_flags(3, 8, "band", diag_shift=4)         # the diagonal sits 4 blocks to the right
    assert all(shifted[i, j] == (abs(j - 4 - i) <= 1) for i in range(3) for j in range(8))
    bg = workloads.block_flags(5, 7, "band_global")
    assert bg[:, 0].all() and bg[0].all() and bg[4, 2] == 0
    with pytest.raises(ValueError):
        workloads.block_flags(2, 2, "nope")


def test_cases_with_block_flags_and_fewer_kv_heads():
    case = workloads.make_case(B=1, H=4, d=16, Nq=100, chunk_rows=[70, 130], dtype="f32", seed=3,
                               block=64, pattern="random", density=0.5, kv_heads=2)
    assert case["K"][0].shape == (1, 2, 70, 16) and case["Q"].shape == (1, 4, 100, 16)
    assert [f.shape for f in case["flags"]] == [(2, 2), (2, 3)]
    assert all(np.array_equal(m.numpy(), f) for m, f in zip(case["masks"], case["flags"]))
    again = workloads.make_case(B=1, H=4, d=16, Nq=100, chunk_rows=[70, 130], dtype="f32", seed=3,
                                block=64, pattern="random", density=0.5, kv_heads=2)
    assert all(np.array_equal(a, b) for a, b in zip(case["flags"], again["flags"]))
    per_head = workloads.make_case(B=2, H=4, d=16, Nq=100, chunk_rows=[70, 130], dtype="f32", seed=3,
                                   block=64, pattern="random", density=0.5, kv_heads=2, per_head_flags=True)
    assert [f.shape for f in per_head["flags"]] == [(2, 4, 2, 2), (2, 4, 2, 3)]
    assert np.array_equal(per_head["flags"][0][0, 0], case["flags"][0])         # head 0 keeps the shared pattern
    assert not np.array_equal(per_head["flags"][1][0, 1], per_head["flags"][1][1, 3])
    assert per_head["masks"][1].shape == (2, 4, 2, 3)


def test_layouts_keep_the_values_and_binding_reads_their_strides():
    import torch
    from paper_2403_09347_amd import binding
    head = workloads.make_case(B=2, H=3, d=16, Nq=10, chunk_rows=[7], dtype="f32", seed=5)
    for layout, q_strides, k_strides in (("seq", (480, 16, 48), (336, 16, 48)),
                                         ("packed", (1440, 16, 144), (1008, 16, 144))):
        case = workloads.make_case(B=2, H=3, d=16, Nq=10, chunk_rows=[7], dtype="f32", seed=5, layout=layout)
        assert torch.equal(case["Q"], head["Q"]) and torch.equal(case["V"][0], head["V"][0])
        assert binding.strides_of(case["Q"]) == q_strides and binding.strides_of(case["K"][0]) == k_strides
    assert binding.strides_of(head["Q"]) is None
    one = torch.zeros((1, 1, 5, 16)).transpose(1, 2).transpose(1, 2)
    assert binding.strides_of(one) is None
    with pytest.raises(ValueError):
        binding.strides_of(torch.zeros((2, 3, 4, 16)).transpose(2, 3))          # last dimension not contiguous
    p = binding.params(2, 3, 10, 7, 16, "f32", 0.25, q_strides=(480, 16, 48))
    assert tuple(p.q_strides) == (480, 16, 48) and tuple(p.kv_strides) == (0, 0, 0)


def test_binding_rejects_host_masks_and_wrong_shapes():
    import torch
    from paper_2403_09347_amd import binding
    with pytest.raises(ValueError):
        binding.params(1, 1, 128, 128, 128, "bf16", 0.1, block_mask=torch.ones((2, 2), dtype=torch.uint8), block=64)
