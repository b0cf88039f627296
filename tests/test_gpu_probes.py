"""The measurement probes of the library do what bench.py says they do."""
import pytest
import torch

from paper_2403_09347_amd import binding as B

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def test_atomic_dq_probe_issues_one_add_per_key_block_and_element():
    heads, nq, key_blocks = 8, 256, 5
    dq = torch.zeros(heads * nq * 128, device=DEV, dtype=torch.float32)
    B.burst_probe_atomic_dq(dq, heads, nq, key_blocks, 1)
    torch.cuda.synchronize()
    assert bool((dq == float(key_blocks)).all())          # every element: one add of 1.0 per key block
    B.burst_probe_atomic_dq(dq, heads, nq, key_blocks, 0)
    torch.cuda.synchronize()
    assert bool((dq == 1.0).all())                         # the same pattern as plain stores
    with pytest.raises(B.BurstError):
        B.burst_probe_atomic_dq(dq, 7, nq, key_blocks, 1)  # heads must be a multiple of 8
    with pytest.raises(B.BurstError):
        B.burst_probe_atomic_dq(dq, heads, 100, 1, 1)      # Nq must be a multiple of 64


def test_mfma_probe_runs_every_feeding_mode_and_accumulates():
    ones = torch.ones(32768, device=DEV, dtype=torch.bfloat16)
    sink = torch.zeros(256 * 512, device=DEV, dtype=torch.float32)
    iters = 3
    for wps in (1, 2):
        for lds in (0, 1, 2):
            sink.zero_()
            B.burst_probe_mfma(lds, wps, ones, sink, iters)
            torch.cuda.synchronize()
            used = sink[: 256 * 256 * wps]
            # all-ones operands: every MFMA adds 16 to each of its 1024 accumulator entries, a lane
            # holds 16 entries of each of 4 accumulators, 4 MFMAs per accumulator and iteration
            assert bool((used == 16.0 * 16 * 4 * 4 * iters).all()), (wps, lds, used[:4])
    with pytest.raises(B.BurstError):
        B.burst_probe_mfma(3, 1, ones, sink, 1)
    with pytest.raises(B.BurstError):
        B.burst_probe_mfma(0, 4, ones, sink, 1)
