"""burst_local_bwd_static (the entry point that allocates nothing) against burst_local_bwd.

Both compute D = rowsum(dO o O) themselves; one into an allocated buffer, the other into the
library's static device scratch.  Same kernels, same arithmetic: every gradient must agree bit for
bit, and with the oracle within the usual bounds.  Two calls in a row, the second on a smaller
input, which finds a stale-scratch or stale-size mistake; then an over-sized call that must be
rejected with nothing written.
"""
import ctypes

import pytest
import torch

from paper_2403_09347_amd import binding as B
from paper_2403_09347_amd import workloads
from paper_2403_09347_amd.harness import RingWalk
from gpu_util import compare_all_heads

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _raw(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else ctypes.c_void_p(0)


def _backward_through_the_c_abi(entry, case, O, lse, with_D_arg):
    """One walk over the case's chunks through the raw C entry point (ctypes, hand-made pointers)."""
    lib = B.load()
    Q, dO = case["Q"], case["dO"]
    Bt, H, Nq, d = Q.shape
    dQ = torch.zeros((Bt, H, Nq, d), dtype=torch.float32, device=DEV)
    dKs, dVs = [], []
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    for K, V, k_off in zip(case["K"], case["V"], case["k_offs"]):
        p = B.params(Bt, H, Nq, K.shape[2], d, "bf16", case["scale"], case["causal"], case["q_off"], k_off)
        dK = torch.full(K.shape, 7.0, dtype=torch.float32, device=DEV)      # overwritten (accumulate_dkv = 0)
        dV = torch.full(V.shape, 7.0, dtype=torch.float32, device=DEV)
        args = [_raw(Q), _raw(K), _raw(V), _raw(O), _raw(dO), _raw(lse)]
        if with_D_arg:
            args.append(ctypes.c_void_p(0))                                   # D = NULL
        args += [_raw(dQ), _raw(dK), _raw(dV), 1, 0, ctypes.byref(p), stream]
        st = getattr(lib, entry)(*args)
        assert st == 0, (entry, st, B.strerror(st))
        dKs.append(dK)
        dVs.append(dV)
    torch.cuda.synchronize()
    return dQ, dKs, dVs


def _one_case(**kw):
    case = workloads.make_case(dtype="bf16", device=DEV, **kw)
    walk = RingWalk(case["Q"], case["scale"], case["causal"], case["q_off"])
    O, lse = walk.forward(case["K"], case["V"], case["k_offs"])
    torch.cuda.synchronize()
    ref = _backward_through_the_c_abi("burst_local_bwd", case, O, lse, with_D_arg=True)
    got = _backward_through_the_c_abi("burst_local_bwd_static", case, O, lse, with_D_arg=False)
    assert torch.equal(got[0], ref[0]), "dQ differs from burst_local_bwd"
    for a, b in zip(got[1] + got[2], ref[1] + ref[2]):
        assert torch.equal(a, b), "dK / dV differ from burst_local_bwd"
    compare_all_heads(case, "bf16", O, lse, *got)


def test_static_scratch_backward_matches_the_allocating_one_twice_in_a_row():
    # first a larger input (several query blocks, ragged tails, two chunks) ...
    _one_case(B=1, H=3, d=128, Nq=704, chunk_rows=[320, 448], seed=61, causal=True, q_off=200)
    # ... then a smaller one: the scratch still holds the first call's D beyond what this one writes
    _one_case(B=1, H=2, d=128, Nq=200, chunk_rows=[150], seed=62)
    # and the d = 64 and generic (fp32 is not bf16: d = 96) kernel families
    _one_case(B=2, H=2, d=64, Nq=160, chunk_rows=[96, 64], seed=63, causal=True, q_off=64)
    _one_case(B=1, H=2, d=96, Nq=70, chunk_rows=[50], seed=64)


def test_static_scratch_backward_rejects_oversized_calls_and_writes_nothing():
    lib = B.load()
    rows = B.BURST_STATIC_MAX_ROWS
    H = 32
    Nq = rows // H + 64                                   # B*H*Nq just above the limit
    p = B.params(1, H, Nq, 64, 128, "bf16", 0.1)
    small = torch.zeros(64, dtype=torch.float32, device=DEV)
    canary = torch.full((1024,), 3.0, dtype=torch.float32, device=DEV)
    ptr = ctypes.c_void_p(small.data_ptr())               # never dereferenced: the call is rejected first
    out = ctypes.c_void_p(canary.data_ptr())
    st = lib.burst_local_bwd_static(ptr, ptr, ptr, ptr, ptr, ptr, out, out, out, 1, 0, ctypes.byref(p),
                                    ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    torch.cuda.synchronize()
    assert st == -8 and b"static scratch" in lib.burst_strerror(st)
    assert bool((canary == 3.0).all())
    # exactly at the limit the parameter block is accepted (not run here: 8 MiB of D needs real inputs)
    assert B.params(1, H, rows // H, 64, 128, "bf16", 0.1).Nq * H == rows
