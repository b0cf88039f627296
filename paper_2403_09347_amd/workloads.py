"""Seeded synthetic workloads: shapes, seeds and random tensors only.

This module holds none of the method's arithmetic.  It is the one module that
both the HIP path's callers and the CPU oracle's callers may use, so that the
two sides see bit-identical stored inputs.

Each workload is one device's share of a sequence-parallel ring (paper Sec. 2.2):
a resident query slice of `Nq` rows per head and `G` key/value chunks of `Nc`
rows that arrive one at a time.  Values are i.i.d. N(0,1) drawn in fp32 from a
seeded generator and rounded once to the storage dtype; the softmax scale is
1/sqrt(d).  They stand in for LLaMA-7B / 13B attention activations at the
paper's sequence lengths (Sec. 4.1), which need model weights and text that
are not available offline.
"""
import math
from dataclasses import dataclass

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    H: int
    d: int
    Nq: int
    G: int
    Nc: int
    dtype: str          # "bf16" | "f32": storage type of Q, K, V, O, dO
    causal: bool
    q_off: int          # global position of query row 0
    seed: int
    window: int = 0     # sliding window (0 = none): keys at positions <= query position - window are hidden

    @property
    def scale(self):
        return 1.0 / math.sqrt(self.d)

    def k_off(self, j):
        return j * self.Nc

    @property
    def torch_dtype(self):
        return torch.bfloat16 if self.dtype == "bf16" else torch.float32

    def visible_pairs_per_head(self):
        """Number of (query, key) pairs that are not masked, per head."""
        if not self.causal and not self.window:
            return self.Nq * self.G * self.Nc
        total = 0
        nk = self.G * self.Nc
        for r in range(self.Nq):
            hi = min(nk, self.q_off + r + 1) if self.causal else nk          # keys [lo, hi) are visible
            lo = max(0, self.q_off + r - self.window + 1) if self.window else 0
            total += max(0, hi - lo)
        return total

    def fwd_flops(self):
        return 4.0 * self.visible_pairs_per_head() * self.d * self.H * self.B

    def bwd_flops(self):
        return 2.5 * self.fwd_flops()


# Index = position in the benchmark's list of configurations.
WORKLOADS = [
    Workload("tiny_f32_G4", 1, 1, 64, 256, 4, 256, "f32", False, 0, 1000),
    Workload("llama7b_32k_G8", 1, 32, 128, 4096, 8, 4096, "bf16", False, 0, 1001),
    Workload("llama7b_128k_G32_rank31_causal", 1, 32, 128, 4096, 32, 4096, "bf16", True, 31 * 4096, 1002),
    Workload("llama13b_128k_G8", 1, 40, 128, 16384, 8, 16384, "bf16", False, 0, 1003),
    Workload("llama7b_1m_G32", 1, 32, 128, 32768, 32, 32768, "bf16", False, 0, 1004),
]


# Further shapes of the paper's experiments (not in the benchmark's list of configurations).
EXTRA_WORKLOADS = [
    # the single-device point of the latency-vs-devices experiment (Sec. 4, batch 1, 65,536 tokens,
    # LLaMA-13B): with G = 1 there is one chunk and the method is plain tiled attention (Sec. 2.4)
    Workload("llama13b_64k_G1", 1, 40, 128, 65536, 1, 65536, "bf16", False, 0, 1005),
    # LLaMA-13B heads at the 32K / G = 8 share (the 13B counterpart of configuration 1): 40 heads x 16
    # blocks of 256 rows = 640 forward workgroups, two and a half rounds on 256 CUs
    Workload("llama13b_32k_G8", 1, 40, 128, 4096, 8, 4096, "bf16", False, 0, 1006),
]


def contiguous_spans(N, G, rank):
    """The paper's assignment (Sec. 2.2): rank r owns positions [r N/G, (r+1) N/G).
    Returns a list of (first position, rows)."""
    n = N // G
    return [(rank * n, n)]


def zigzag_spans(N, G, rank):
    """Load-balanced causal assignment: the sequence is cut into 2G stripes of N/(2G) positions and
    rank r owns stripes r and 2G-1-r, so that every rank sees the same number of causal
    (query, key) pairs.  Returns a list of (first position, rows)."""
    n = N // (2 * G)
    return [(rank * n, n), ((2 * G - 1 - rank) * n, n)]


def causal_pairs(spans, N):
    """Unmasked (query, key) pairs of query spans against keys 0..N-1 under the causal mask."""
    total = 0
    for first, rows in spans:
        lo, hi = min(first, N), min(first + rows, N)          # rows at positions >= N see all N keys
        total += (hi * (hi + 1) - lo * (lo + 1)) // 2 + (first + rows - hi) * N
    return total


def by_name(name):
    for w in WORKLOADS + EXTRA_WORKLOADS:
        if w.name == name:
            return w
    raise KeyError(name)


def _randn(shape, gen, device, dtype):
    return torch.randn(shape, generator=gen, device=device, dtype=torch.float32).to(dtype)


def make_inputs(w, device="cpu", seed=None):
    """Returns dict(Q, K=[G chunks], V=[G chunks], dO); tensors are [B,H,rows,d]."""
    gen = torch.Generator(device=device)
    gen.manual_seed(w.seed if seed is None else seed)
    dt = w.torch_dtype
    Q = _randn((w.B, w.H, w.Nq, w.d), gen, device, dt)
    K = [_randn((w.B, w.H, w.Nc, w.d), gen, device, dt) for _ in range(w.G)]
    V = [_randn((w.B, w.H, w.Nc, w.d), gen, device, dt) for _ in range(w.G)]
    dO = _randn((w.B, w.H, w.Nq, w.d), gen, device, dt)
    return {"Q": Q, "K": K, "V": V, "dO": dO}


def block_flags(n_row_blocks, n_col_blocks, kind="random", density=0.4, seed=0, diag_shift=0):
    """Seeded block-sparse patterns as a uint8 matrix of block flags (1 = the block pair is
    computed).  kind: "random" (each flag set with probability `density`), "band" (blocks on and
    next to the diagonal, which sits `diag_shift` column blocks to the right), "band_global"
    (band, plus the first column block for every row block and the first row block complete: the
    shape of global-plus-local patterns for long documents)."""
    import numpy as np
    rng = np.random.default_rng(seed)
    i, j = np.arange(n_row_blocks)[:, None], np.arange(n_col_blocks)[None, :]
    if kind == "random":
        f = rng.random((n_row_blocks, n_col_blocks)) < density
    elif kind in ("band", "band_global"):
        f = np.abs(j - diag_shift - i) <= 1
        if kind == "band_global":
            f = f | (j == 0) | (i == 0)
    else:
        raise ValueError(kind)
    return f.astype(np.uint8)


def relayout(x, layout):
    """The same [B, H, rows, d] values in another memory layout: "head" (contiguous), "seq" (a
    transposed view of a contiguous [B, rows, H, d] tensor: the layout of the backward messages
    in paper Sec. 2.2) or "packed" (a view into slot 1 of a [B, rows, 3, H, d] tensor, as a fused
    query/key/value projection leaves its output)."""
    if layout == "head":
        return x
    if layout == "seq":
        return x.transpose(1, 2).contiguous().transpose(1, 2)
    if layout == "packed":
        B, H, rows, d = x.shape
        big = torch.zeros((B, rows, 3, H, d), dtype=x.dtype, device=x.device)
        big[:, :, 1] = x.transpose(1, 2)
        return big[:, :, 1].transpose(1, 2)
    raise ValueError(layout)


def make_case(B, H, d, Nq, chunk_rows, dtype="bf16", seed=0, device="cpu",
              causal=False, q_off=0, k_offs=None, window=0, block=0, pattern="random", density=0.4, kv_heads=0,
              per_head_flags=False, layout="head"):
    """Free-form case for parity tests: `chunk_rows` lists the rows of each chunk.  With
    block > 0 the case carries one block-flag matrix per chunk ("flags": numpy, "masks": the
    same on the device), blocks counted from the first row of the slice / of each chunk.  With
    kv_heads > 0 the K / V chunks have that many heads (grouped-query attention).  With
    per_head_flags every (batch, query head) has a flag matrix of its own: [B, H, blocks, blocks].
    layout: how Q, K, V, dO lie in memory (see relayout; the values do not depend on it)."""
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    dt = torch.bfloat16 if dtype == "bf16" else torch.float32
    Q = _randn((B, H, Nq, d), gen, device, dt)
    Hkv = kv_heads or H
    K = [_randn((B, Hkv, n, d), gen, device, dt) for n in chunk_rows]
    V = [_randn((B, Hkv, n, d), gen, device, dt) for n in chunk_rows]
    dO = _randn((B, H, Nq, d), gen, device, dt)
    Q, dO = relayout(Q, layout), relayout(dO, layout)
    K, V = [relayout(x, layout) for x in K], [relayout(x, layout) for x in V]
    if k_offs is None:
        k_offs, s = [], 0
        for n in chunk_rows:
            k_offs.append(s)
            s += n
    case = {"Q": Q, "K": K, "V": V, "dO": dO, "k_offs": list(k_offs),
            "q_off": q_off, "causal": causal, "window": window, "scale": 1.0 / math.sqrt(d)}
    if kv_heads:
        case["kv_heads"] = kv_heads
    if block:
        nrb = -(-Nq // block)
        case["block"] = block
        import numpy as np

        def one(j, n, bh):
            return block_flags(nrb, -(-n // block), pattern, density, seed + 101 * j + 7919 * bh,
                               diag_shift=(q_off - k_offs[j]) // block if pattern != "random" else 0)
        if per_head_flags:
            case["flags"] = [np.stack([one(j, n, bh) for bh in range(B * H)]).reshape(B, H, nrb, -1)
                             for j, n in enumerate(chunk_rows)]
        else:
            case["flags"] = [one(j, n, 0) for j, n in enumerate(chunk_rows)]
        case["masks"] = [torch.from_numpy(f).to(device).contiguous() for f in case["flags"]]
    return case
