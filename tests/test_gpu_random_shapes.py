"""A seeded sweep over call shapes: sizes, chunk lists with gaps, masks of all three kinds, head
dimension, grouped heads, per-head flags, memory layouts, tiled and stored-matrix walks, every output
against the oracle.  The specifications come from one numpy generator, so the sweep is the same
on every run."""
import numpy as np
import pytest
import torch

from paper_2403_09347_amd import workloads
from paper_2403_09347_amd.harness import MaterializedWalk, RingWalk
from gpu_util import compare_all_heads

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def specs(seed, n):
    rng = np.random.default_rng(seed)
    out = []
    for it in range(n):
        H, Nq, G = int(rng.integers(1, 4)), int(rng.integers(1, 700)), int(rng.integers(1, 4))
        rows = [int(rng.integers(1, 600)) for _ in range(G)]
        spec = dict(B=int(rng.integers(1, 3)), H=H, d=int(rng.choice([64, 128, 32])), Nq=Nq, chunk_rows=rows,
                    causal=bool(rng.integers(0, 2)), q_off=int(rng.integers(-50, sum(rows) + 50)),
                    window=int(rng.choice([0, 0, 1, 7, 64, 100, 300, 1000])))
        if rng.integers(0, 4) == 0:                 # gaps between the chunks' positions
            k_offs, s = [], 0
            for r in rows:
                s += int(rng.integers(0, 80))
                k_offs.append(s)
                s += r
            spec["k_offs"] = k_offs
        if rng.integers(0, 2):
            spec.update(block=int(rng.choice([64, 128, 256])), pattern=str(rng.choice(["random", "band", "band_global"])),
                        density=float(rng.choice([0.1, 0.4, 0.8])), per_head_flags=bool(rng.integers(0, 2)))
        if rng.integers(0, 3) == 0:
            g = int(rng.choice([2, 3, 4]))
            spec.update(H=H * g, kv_heads=H)
            if rng.integers(0, 2):
                spec["Nq"] = 64 * int(rng.integers(1, 10))
        spec["layout"] = str(rng.choice(["head", "seq", "packed"]))
        out.append((it, "f32" if spec["d"] == 32 else "bf16", bool(rng.integers(0, 4) == 0), spec))
    return out


@pytest.mark.parametrize("it,dtype,stored,spec", specs(2024, 48), ids=lambda v: str(v) if isinstance(v, int) else "")
def test_seeded_random_call(it, dtype, stored, spec):
    case = workloads.make_case(dtype=dtype, seed=5000 + it, device=DEV, **spec)
    cls = MaterializedWalk if stored else RingWalk
    walk = cls(case["Q"], case["scale"], case["causal"], case["q_off"], case["window"],
               block=case.get("block", 0), kv_heads=case.get("kv_heads", 0))
    O, lse = walk.forward(case["K"], case["V"], case["k_offs"], masks=case.get("masks"))
    dQ, dKs, dVs = walk.backward(case["K"], case["V"], case["k_offs"], case["dO"], masks=case.get("masks"))
    torch.cuda.synchronize()
    compare_all_heads(case, dtype, O, lse, dQ, dKs, dVs)


def narrow_flag_specs(seed, n):
    """bf16, d = 128, 64-wide block flags on every call: the shapes that send the dK/dV half to the
    hand-scheduled kernel's 64-key workgroups."""
    rng = np.random.default_rng(seed)
    out = []
    for it in range(n):
        H, G = int(rng.integers(1, 4)), int(rng.integers(1, 4))
        rows = [int(rng.integers(64, 700)) for _ in range(G)]
        spec = dict(B=int(rng.integers(1, 3)), H=H, d=128, Nq=int(rng.integers(1, 900)), chunk_rows=rows,
                    causal=bool(rng.integers(0, 2)), q_off=int(rng.integers(0, sum(rows) + 50)),
                    window=int(rng.choice([0, 0, 0, 200, 1000])), block=64,
                    pattern=str(rng.choice(["random", "band", "band_global"])), density=float(rng.choice([0.3, 0.6, 0.9])),
                    per_head_flags=bool(rng.integers(0, 2)), layout=str(rng.choice(["head", "seq", "packed"])))
        if rng.integers(0, 3) == 0:
            g = int(rng.choice([2, 3]))
            spec.update(H=H * g, kv_heads=H, Nq=64 * int(rng.integers(1, 12)))
        out.append((it, spec))
    return out


@pytest.mark.parametrize("it,spec", narrow_flag_specs(2025, 24), ids=lambda v: str(v) if isinstance(v, int) else "")
def test_seeded_random_call_with_narrow_block_flags(it, spec):
    case = workloads.make_case(dtype="bf16", seed=7000 + it, device=DEV, **spec)
    walk = RingWalk(case["Q"], case["scale"], case["causal"], case["q_off"], case["window"],
                    block=64, kv_heads=case.get("kv_heads", 0))
    O, lse = walk.forward(case["K"], case["V"], case["k_offs"], masks=case["masks"])
    dQ, dKs, dVs = walk.backward(case["K"], case["V"], case["k_offs"], case["dO"], masks=case["masks"])
    torch.cuda.synchronize()
    compare_all_heads(case, "bf16", O, lse, dQ, dKs, dVs)
