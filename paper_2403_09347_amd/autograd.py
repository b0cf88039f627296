"""torch.autograd wrapper around the chunk walk: attention of a query slice against a list of
key/value chunks (paper Alg. 1 for the forward, Alg. 2 for the backward) as one differentiable
call.  Argument marshalling and buffer management only: every arithmetic step is a library call
through `harness.RingWalk`.  On one GPU the chunks are simply all resident; in a ring the same
calls are made once per received chunk."""
import torch

from .harness import RingWalk


class _BurstAttention(torch.autograd.Function):
    @staticmethod
    def forward(ctx, q, scale, causal, q_off, window, kv_heads, n_chunks, *kv):
        ks, vs = list(kv[:n_chunks]), list(kv[n_chunks:])
        k_offs, s = [], 0
        for k in ks:
            k_offs.append(s)
            s += k.shape[2]
        walk = RingWalk(q.contiguous(), scale, causal, q_off, window, 0, kv_heads)
        ks, vs = [k.contiguous() for k in ks], [v.contiguous() for v in vs]
        O, lse = walk.forward(ks, vs, k_offs)
        ctx.walk, ctx.ks, ctx.vs, ctx.k_offs = walk, ks, vs, k_offs
        ctx.mark_non_differentiable(lse)
        return O, lse

    @staticmethod
    def backward(ctx, dO, _dlse):
        walk = ctx.walk
        dQ, dKs, dVs = walk.backward(ctx.ks, ctx.vs, ctx.k_offs, dO.contiguous().to(walk.Q.dtype))
        dt = walk.Q.dtype
        return (dQ.to(dt), None, None, None, None, None, None,
                *[g.to(dt) for g in dKs], *[g.to(dt) for g in dVs])


def burst_attention(q, k_chunks, v_chunks, scale=None, causal=False, q_off=0, window=0):
    """q [B, H, Nq, d]; k_chunks / v_chunks: lists of [B, Hkv, Nc_j, d] (Hkv divides H), chunk j
    starting at global key position sum(Nc_0..Nc_{j-1}); q_off = global position of query row 0.
    Returns (O [B, H, Nq, d] in q's dtype, lse [B, H, Nq] fp32).  Gradients flow to q and to
    every chunk (rounded to the input dtype)."""
    if isinstance(k_chunks, torch.Tensor):
        k_chunks, v_chunks = [k_chunks], [v_chunks]
    assert len(k_chunks) == len(v_chunks) and len(k_chunks) > 0
    d = q.shape[-1]
    scale = float(scale) if scale is not None else d ** -0.5
    Hkv = k_chunks[0].shape[1]
    kv_heads = Hkv if Hkv != q.shape[1] else 0
    return _BurstAttention.apply(q, scale, bool(causal), int(q_off), int(window), kv_heads, len(k_chunks),
                                 *k_chunks, *v_chunks)
