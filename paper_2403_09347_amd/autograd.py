"""torch.autograd wrapper around the chunk walk: attention of a query slice against a list of
key/value chunks (paper Alg. 1 for the forward, Alg. 2 for the backward) as one differentiable
call.  Argument marshalling and buffer management only: every arithmetic step is a library call
through `harness.RingWalk`.  On one GPU the chunks are simply all resident; in a ring the same
calls are made once per received chunk."""
import torch

from .harness import RingWalk


def _addressable(t):
    """True if the library can read the [B, H, rows, d] tensor where it lies: last dimension
    contiguous, the other strides and the base address multiples of 16 bytes, rows not overlapping."""
    unit = 16 // t.element_size()
    return (t.dim() == 4 and (t.shape[3] == 1 or t.stride(3) == 1) and t.data_ptr() % 16 == 0 and
            all(t.shape[i] == 1 or (t.stride(i) > 0 and t.stride(i) % unit == 0) for i in range(3)) and
            (t.shape[2] == 1 or t.stride(2) >= t.shape[3]))


def _pair_in_place(k, v):
    """K and V of a chunk as they are if the library can address both with one set of strides,
    else contiguous copies."""
    same = all(k.shape[i] == 1 or k.stride(i) == v.stride(i) for i in range(3))
    if _addressable(k) and _addressable(v) and same and k.is_contiguous() == v.is_contiguous():
        return k, v
    return k.contiguous(), v.contiguous()


class _BurstAttention(torch.autograd.Function):
    @staticmethod
    def forward(ctx, q, scale, causal, q_off, window, kv_heads, block, masks, n_chunks, *kv):
        ks, vs = list(kv[:n_chunks]), list(kv[n_chunks:])
        k_offs, s = [], 0
        for k in ks:
            k_offs.append(s)
            s += k.shape[2]
        walk = RingWalk(q if _addressable(q) else q.contiguous(), scale, causal, q_off, window, block, kv_heads)
        pairs = [_pair_in_place(k, v) for k, v in zip(ks, vs)]
        ks, vs = [p[0] for p in pairs], [p[1] for p in pairs]
        O, lse = walk.forward(ks, vs, k_offs, masks=masks)
        ctx.walk, ctx.ks, ctx.vs, ctx.k_offs, ctx.masks = walk, ks, vs, k_offs, masks
        ctx.mark_non_differentiable(lse)
        return O, lse

    @staticmethod
    def backward(ctx, dO, _dlse):
        walk = ctx.walk
        dQ, dKs, dVs = walk.backward(ctx.ks, ctx.vs, ctx.k_offs, dO.to(walk.Q.dtype), masks=ctx.masks)
        dt = walk.Q.dtype
        return (dQ.to(dt), None, None, None, None, None, None, None, None,
                *[g.to(dt) for g in dKs], *[g.to(dt) for g in dVs])


def burst_attention(q, k_chunks, v_chunks, scale=None, causal=False, q_off=0, window=0, block_masks=None, block=0):
    """q [B, H, Nq, d]; k_chunks / v_chunks: lists of [B, Hkv, Nc_j, d] (Hkv divides H), chunk j
    starting at global key position sum(Nc_0..Nc_{j-1}); q_off = global position of query row 0.
    Returns (O [B, H, Nq, d] in q's dtype and memory layout, lse [B, H, Nq] fp32).  Gradients flow
    to q and to every chunk (rounded to the input dtype).  Views with a contiguous last dimension
    (sequence-major tensors, slices of a packed projection) are read in place, without a copy.
    block_masks: one uint8 device tensor of block flags per chunk (see binding.params) with blocks
    of `block` rows / keys, or None."""
    if isinstance(k_chunks, torch.Tensor):
        k_chunks, v_chunks = [k_chunks], [v_chunks]
    assert len(k_chunks) == len(v_chunks) and len(k_chunks) > 0
    d = q.shape[-1]
    scale = float(scale) if scale is not None else d ** -0.5
    Hkv = k_chunks[0].shape[1]
    kv_heads = Hkv if Hkv != q.shape[1] else 0
    if block_masks is not None:
        assert len(block_masks) == len(k_chunks) and block > 0
        block_masks = list(block_masks)
    return _BurstAttention.apply(q, scale, bool(causal), int(q_off), int(window), kv_heads,
                                 int(block) if block_masks is not None else 0, block_masks, len(k_chunks),
                                 *k_chunks, *v_chunks)
