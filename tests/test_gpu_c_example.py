"""The library driven from a plain host program (no Python, no PyTorch on the path): the example
built from paper_2403_09347_amd/examples/ring_walk.cpp walks a ring share through the C ABI with
hipMalloc'ed buffers, backward through burst_local_bwd_static, and dumps inputs and results; this
test holds the results against the oracle, every head and every element."""
import os
import subprocess

import numpy as np
import pytest

from oracle import burst_oracle as orc
from gpu_util import check

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
EXE = os.path.join(ROOT, "paper_2403_09347_amd", "_build", "ring_walk")


def bf16_to_f64(raw):
    return (raw.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


@pytest.mark.parametrize("H,Nq,Nc,G,causal", [(3, 320, 200, 3, 0), (2, 256, 256, 2, 1)])
def test_plain_host_program_matches_the_oracle(tmp_path, H, Nq, Nc, G, causal):
    assert os.path.exists(EXE), "examples/ring_walk is not built: run __graft_entry__.build() first"
    out = str(tmp_path / "walk.bin")
    r = subprocess.run([EXE, str(H), str(Nq), str(Nc), str(G), str(causal), "7", out], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode == 0, r.stdout + r.stderr
    raw = open(out, "rb").read()
    head = np.frombuffer(raw, np.int32, 5)
    assert tuple(head) == (H, Nq, Nc, G, causal)
    scale = float(np.frombuffer(raw, np.float32, 1, 20)[0])
    pos, d = 24, 128

    def take(dtype, shape):
        nonlocal pos
        n = int(np.prod(shape))
        a = np.frombuffer(raw, dtype, n, pos).reshape(shape)
        pos += n * np.dtype(dtype).itemsize
        return a
    Q = bf16_to_f64(take(np.uint16, (H, Nq, d)))
    K = bf16_to_f64(take(np.uint16, (G, H, Nc, d)))
    V = bf16_to_f64(take(np.uint16, (G, H, Nc, d)))
    dO = bf16_to_f64(take(np.uint16, (H, Nq, d)))
    O = bf16_to_f64(take(np.uint16, (H, Nq, d)))
    lse = take(np.float32, (H, Nq)).astype(np.float64)
    dQ = take(np.float32, (H, Nq, d)).astype(np.float64)
    dK = take(np.float32, (G, H, Nc, d)).astype(np.float64)
    dV = take(np.float32, (G, H, Nc, d)).astype(np.float64)
    assert pos == len(raw)
    assert abs(float(Q.std()) - 1.0) < 0.05                       # the program's inputs are about N(0,1)
    q_pos = (G - 1) * Nc * (1 if causal else 0) + np.arange(Nq)
    k_pos = np.arange(G * Nc)
    for h in range(H):
        Kh = K[:, h].reshape(G * Nc, d)
        Vh = V[:, h].reshape(G * Nc, d)
        O_ref, lse_ref = orc.full_forward(Q[h], Kh, Vh, scale, bool(causal), q_pos, k_pos)
        dQ_ref, dK_ref, dV_ref = orc.full_backward(Q[h], Kh, Vh, dO[h], scale, bool(causal), q_pos, k_pos)
        check(f"O[{h}]", O[h], O_ref, "bf16")
        check(f"lse[{h}]", lse[h], lse_ref, "bf16", "lse")
        check(f"dQ[{h}]", dQ[h], dQ_ref, "bf16")
        check(f"dK[{h}]", dK[:, h].reshape(G * Nc, d), dK_ref, "bf16")
        check(f"dV[{h}]", dV[:, h].reshape(G * Nc, d), dV_ref, "bf16")
