"""Single-GPU harness: walks G key/value chunks, one library call per chunk, in the order a
device of the ring would receive them (paper Alg. 1 / Alg. 2 loops with the ring step replaced
by taking the next chunk).  Two walks: chunks already resident (plain), and chunks fetched from
a source pool through two receive buffers on a second stream while the previous chunk is being
computed (the double buffer of paper Sec. 2.5 / Alg. 3, with a copy standing in for the ring
transfer).  Host-side orchestration only: every arithmetic step is a library call."""
import torch

from . import binding as B


class RingWalk:
    """Buffers and call sequence for one query slice against a list of chunks."""

    def __init__(self, Q, scale, causal=False, q_off=0, window=0, block=0, kv_heads=0):
        assert Q.dim() == 4
        self.Q = Q
        self.kv_heads = int(kv_heads)    # heads of K / V when fewer than Q's (0 = the same)
        self.block = int(block)          # edge of the blocks of per-chunk block masks (0 = no masks)
        self.Bt, self.H, self.Nq, self.d = Q.shape
        self.scale, self.causal, self.q_off, self.window = float(scale), bool(causal), int(q_off), int(window)
        dev = Q.device
        self.O_acc = torch.empty((self.Bt, self.H, self.Nq, self.d), device=dev, dtype=torch.float32)
        self.m = torch.empty((self.Bt, self.H, self.Nq), device=dev, dtype=torch.float32)
        self.l = torch.empty_like(self.m)
        self.O = torch.empty_strided(Q.shape, Q.stride(), device=dev, dtype=Q.dtype)   # O and dO lie in memory like Q
        self.lse = torch.empty_like(self.m)
        self.D = torch.empty_like(self.m)

    def params(self, Nc, k_off, mask=None, K_c=None):
        """K_c: the chunk the call is about (its strides go into the parameter block; Q's always do)."""
        return B.params(self.Bt, self.H, self.Nq, Nc, self.d, self.Q.dtype, self.scale,
                        self.causal, self.q_off, k_off, self.window, mask, self.block, self.kv_heads,
                        q_strides=B.strides_of(self.Q), kv_strides=None if K_c is None else B.strides_of(K_c))

    # ---- forward (Alg. 1)
    def init(self):
        B.burst_state_init(self.O_acc, self.m, self.l, self.params(0, 0))

    def step(self, K_c, V_c, k_off, mask=None):
        B.burst_local_fwd(self.Q, K_c, V_c, self.O_acc, self.m, self.l, self.params(K_c.shape[2], k_off, mask, K_c))

    def finalize(self):
        B.burst_finalize(self.O_acc, self.m, self.l, self.O, self.lse, self.params(0, 0))
        return self.O, self.lse

    def forward(self, Ks, Vs, k_offs, order=None, masks=None):
        """masks: optional list of per-chunk block masks (uint8 device tensors, see binding.params)."""
        self.init()
        for j in (range(len(Ks)) if order is None else order):
            self.step(Ks[j], Vs[j], k_offs[j], None if masks is None else masks[j])
        return self.finalize()

    # ---- backward (Alg. 2), query slice pinned, chunks walked
    def prepare(self, dO):
        B.burst_bwd_prepare(self.O, dO, self.D, self.params(0, 0))

    def backward(self, Ks, Vs, k_offs, dO, dQ=None, dKs=None, dVs=None, use_D=True, masks=None):
        dev = self.Q.device
        if dQ is None:
            dQ = torch.zeros((self.Bt, self.H, self.Nq, self.d), device=dev, dtype=torch.float32)
        if dKs is None:
            dKs = [torch.empty(K.shape, device=dev, dtype=torch.float32) for K in Ks]
            dVs = [torch.empty(V.shape, device=dev, dtype=torch.float32) for V in Vs]
        if dO.stride() != self.Q.stride():         # dO and O lie in memory like Q
            dO = torch.empty_strided(self.Q.shape, self.Q.stride(), device=dev, dtype=self.Q.dtype).copy_(dO)
        if use_D:
            self.prepare(dO)
        for j in range(len(Ks)):
            B.burst_local_bwd(self.Q, Ks[j], Vs[j], self.O, dO, self.lse, self.D if use_D else None,
                              dQ, dKs[j], dVs[j],
                              self.params(Ks[j].shape[2], k_offs[j], None if masks is None else masks[j], Ks[j]),
                              accumulate_dq=True, accumulate_dkv=False)
        return dQ, dKs, dVs


class MaterializedWalk(RingWalk):
    """The forward walk with the chunk step that stores S_ij and P_ij in HBM (the paper's
    "w/o LAO" ablation): same state, same finalize, one workspace sized for the largest chunk."""

    def __init__(self, Q, scale, causal=False, q_off=0, window=0, max_chunk_rows=0, block=0, kv_heads=0):
        super().__init__(Q, scale, causal, q_off, window, block, kv_heads)
        self.workspace = None
        if max_chunk_rows:
            self._reserve(max_chunk_rows)

    def _reserve(self, rows):
        need = B.burst_materialized_workspace_bytes(self.params(rows, 0))
        if self.workspace is None or self.workspace.numel() < need:
            self.workspace = torch.empty(max(need, 256), device=self.Q.device, dtype=torch.uint8)
        return need

    def step(self, K_c, V_c, k_off, mask=None):
        self._reserve(K_c.shape[2])
        B.burst_local_fwd_materialized(self.Q, K_c, V_c, self.O_acc, self.m, self.l, self.workspace,
                                       self.params(K_c.shape[2], k_off, mask, K_c))

    def backward(self, Ks, Vs, k_offs, dO, dQ=None, dKs=None, dVs=None, use_D=True, masks=None):
        """Alg. 2 with every matrix of a block pair stored in HBM (D is always computed first)."""
        dev = self.Q.device
        if dQ is None:
            dQ = torch.zeros((self.Bt, self.H, self.Nq, self.d), device=dev, dtype=torch.float32)
        if dKs is None:
            dKs = [torch.empty(K.shape, device=dev, dtype=torch.float32) for K in Ks]
            dVs = [torch.empty(V.shape, device=dev, dtype=torch.float32) for V in Vs]
        if dO.stride() != self.Q.stride():
            dO = torch.empty_strided(self.Q.shape, self.Q.stride(), device=dev, dtype=self.Q.dtype).copy_(dO)
        self.prepare(dO)
        for j in range(len(Ks)):
            p = self.params(Ks[j].shape[2], k_offs[j], None if masks is None else masks[j], Ks[j])
            need = B.burst_materialized_bwd_workspace_bytes(p)
            if self.workspace is None or self.workspace.numel() < need:
                self.workspace = torch.empty(max(need, 256), device=dev, dtype=torch.uint8)
            B.burst_local_bwd_materialized(self.Q, Ks[j], Vs[j], dO, self.lse, self.D, dQ, dKs[j], dVs[j],
                                           self.workspace, p, accumulate_dq=True, accumulate_dkv=False)
        return dQ, dKs, dVs

    def stored_gradients(self, Nc):
        """Views of dP_ij (fp32), P_ij and dS_ij (input type) of the last backward step: [B, H, Nq, Nc]."""
        ncp = (Nc + 7) // 8 * 8
        rows = self.Bt * self.H * self.Nq
        es = self.Q.element_size()
        a = (rows * ncp * 4 + 255) // 256 * 256
        b = a + (rows * ncp * es + 255) // 256 * 256
        shape = (self.Bt, self.H, self.Nq, ncp)
        dP = self.workspace[: rows * ncp * 4].view(torch.float32).view(shape)
        P = self.workspace[a: a + rows * ncp * es].view(self.Q.dtype).view(shape)
        dS = self.workspace[b: b + rows * ncp * es].view(self.Q.dtype).view(shape)
        return dP[..., :Nc], P[..., :Nc], dS[..., :Nc]

    def stored_scores(self, Nc):
        """Views of S_ij (fp32) and P_ij (input type) of the last step: [B, H, Nq, Nc]."""
        ncp = (Nc + 7) // 8 * 8
        rows = self.Bt * self.H * self.Nq
        s_bytes = (rows * ncp * 4 + 255) // 256 * 256
        S = self.workspace[: rows * ncp * 4].view(torch.float32).view(self.Bt, self.H, self.Nq, ncp)
        P = self.workspace[s_bytes: s_bytes + rows * ncp * self.Q.element_size()].view(self.Q.dtype) \
            .view(self.Bt, self.H, self.Nq, ncp)
        return S[..., :Nc], P[..., :Nc]


class DoubleBufferedWalk(RingWalk):
    """Paper Sec. 2.5 / Alg. 3 on one GPU: chunk j+1 is copied from its source (another HBM
    allocation, or pinned host memory as a slow link) into the alternate receive buffer on a
    copy stream while chunk j is computed on the caller's stream.  The copy of chunk j+1
    starts when the local attention of chunk j starts and may only overwrite a buffer whose
    chunk (j-1) has been consumed; the computation of chunk j waits for its copy.  All streams
    have the default priority."""

    def __init__(self, Q, scale, causal=False, q_off=0, max_chunk_rows=None, window=0):
        super().__init__(Q, scale, causal, q_off, window)
        self.copy_stream = torch.cuda.Stream(device=Q.device)
        self.max_rows = max_chunk_rows
        self._bufs = None

    def _buffers(self, rows):
        n = self.Bt * self.H * rows * self.d
        if self._bufs is None or self._bufs[0][0].numel() < n:
            mk = lambda: torch.empty(n, device=self.Q.device, dtype=self.Q.dtype)
            self._bufs = [(mk(), mk()), (mk(), mk())]
        return self._bufs

    def _view(self, flat, rows):
        return flat[: self.Bt * self.H * rows * self.d].view(self.Bt, self.H, rows, self.d)

    def _fetch(self, j, src_Ks, src_Vs, ready, done):
        rows = src_Ks[j].shape[2]
        kb, vb = self._bufs[j % 2]
        with torch.cuda.stream(self.copy_stream):
            if j >= 2:
                self.copy_stream.wait_event(done[j - 2])       # the buffer's previous chunk is consumed
            self._view(kb, rows).copy_(src_Ks[j], non_blocking=True)
            self._view(vb, rows).copy_(src_Vs[j], non_blocking=True)
            ready[j].record(self.copy_stream)
        return self._view(kb, rows), self._view(vb, rows)

    def forward(self, src_Ks, src_Vs, k_offs, order=None):
        idx = list(range(len(src_Ks))) if order is None else list(order)
        Ks, Vs, offs = [src_Ks[j] for j in idx], [src_Vs[j] for j in idx], [k_offs[j] for j in idx]
        G = len(Ks)
        main = torch.cuda.current_stream(self.Q.device)
        self._buffers(self.max_rows or max(k.shape[2] for k in Ks))
        ready = [torch.cuda.Event() for _ in range(G)]
        done = [torch.cuda.Event() for _ in range(G)]
        self.copy_stream.wait_stream(main)                       # sources are complete
        self.init()
        nxt = self._fetch(0, Ks, Vs, ready, done) if G else None
        for j in range(G):
            cur = nxt
            if j + 1 < G:
                nxt = self._fetch(j + 1, Ks, Vs, ready, done)    # issued as chunk j's attention starts
            main.wait_event(ready[j])
            self.step(cur[0], cur[1], offs[j])
            done[j].record(main)
        return self.finalize()

    def backward(self, src_Ks, src_Vs, k_offs, dO, dQ=None, dKs=None, dVs=None, use_D=True):
        """Same pipeline for Alg. 2 with the query slice pinned: K/V chunks stream in, each
        chunk's dK/dV is written to its destination as soon as it is complete."""
        dev = self.Q.device
        G = len(src_Ks)
        main = torch.cuda.current_stream(dev)
        if dQ is None:
            dQ = torch.zeros((self.Bt, self.H, self.Nq, self.d), device=dev, dtype=torch.float32)
        if dKs is None:
            dKs = [torch.empty(tuple(K.shape), device=dev, dtype=torch.float32) for K in src_Ks]
            dVs = [torch.empty(tuple(V.shape), device=dev, dtype=torch.float32) for V in src_Vs]
        self._buffers(self.max_rows or max(k.shape[2] for k in src_Ks))
        ready = [torch.cuda.Event() for _ in range(G)]
        done = [torch.cuda.Event() for _ in range(G)]
        self.copy_stream.wait_stream(main)
        if use_D:
            self.prepare(dO)
        nxt = self._fetch(0, src_Ks, src_Vs, ready, done) if G else None
        for j in range(G):
            cur = nxt
            if j + 1 < G:
                nxt = self._fetch(j + 1, src_Ks, src_Vs, ready, done)
            main.wait_event(ready[j])
            B.burst_local_bwd(self.Q, cur[0], cur[1], self.O, dO, self.lse, self.D if use_D else None,
                              dQ, dKs[j], dVs[j], self.params(cur[0].shape[2], k_offs[j]),
                              accumulate_dq=True, accumulate_dkv=False)
            done[j].record(main)
        return dQ, dKs, dVs

    def copies_only(self, src_Ks, src_Vs):
        """The transfers alone, back to back on the copy stream (for the overlap measurement)."""
        G = len(src_Ks)
        self._buffers(self.max_rows or max(k.shape[2] for k in src_Ks))
        ready = [torch.cuda.Event() for _ in range(G)]
        self.copy_stream.wait_stream(torch.cuda.current_stream(self.Q.device))
        for j in range(G):
            rows = src_Ks[j].shape[2]
            kb, vb = self._bufs[j % 2]
            with torch.cuda.stream(self.copy_stream):
                self._view(kb, rows).copy_(src_Ks[j], non_blocking=True)
                self._view(vb, rows).copy_(src_Vs[j], non_blocking=True)
        torch.cuda.current_stream(self.Q.device).wait_stream(self.copy_stream)



class GraphedStep:
    """One whole step (Alg. 1 walk, then Alg. 2 walk) of a fixed shape recorded once as a HIP
    graph and replayed with a single launch: for chunks short enough that the launches, not
    the kernels, set the pace.  The graph reads and writes the tensors it was recorded on: new
    inputs are copied INTO `walk.Q`, the chunk tensors and `dO`, results are read from
    `walk.O`, `walk.lse`, `dQ`, `dKs`, `dVs`.  Every node is a kernel (the gradient buffer is
    cleared by a fill kernel, nothing is allocated or memset while recording)."""

    def __init__(self, walk, Ks, Vs, k_offs, dO, masks=None):
        assert type(walk) is RingWalk
        dev = walk.Q.device
        self.walk, self.Ks, self.Vs, self.k_offs, self.masks = walk, list(Ks), list(Vs), list(k_offs), masks
        self.dO = dO if dO.stride() == walk.Q.stride() else \
            torch.empty_strided(walk.Q.shape, walk.Q.stride(), device=dev, dtype=walk.Q.dtype).copy_(dO)
        self.dQ = torch.zeros((walk.Bt, walk.H, walk.Nq, walk.d), device=dev, dtype=torch.float32)
        self.dKs = [torch.empty(K.shape, device=dev, dtype=torch.float32) for K in Ks]
        self.dVs = [torch.empty(V.shape, device=dev, dtype=torch.float32) for V in Vs]
        # eager once on a side stream: first calls set kernel attributes, which a recording cannot hold
        side = torch.cuda.Stream(device=dev)
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            self._run()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        self.graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(self.graph):
            self._run()

    def _run(self):
        w = self.walk
        w.forward(self.Ks, self.Vs, self.k_offs, masks=self.masks)
        self.dQ.zero_()
        w.backward(self.Ks, self.Vs, self.k_offs, self.dO, self.dQ, self.dKs, self.dVs, masks=self.masks)

    def replay(self):
        self.graph.replay()
        return self.walk.O, self.walk.lse, self.dQ, self.dKs, self.dVs


class SpanWalk:
    """A device whose query rows are several contiguous spans of the sequence, each its own tensor
    with its own global offset -- e.g. the two stripes of a load-balanced ("zig-zag") causal
    assignment (workloads.zigzag_spans).  Every span keeps its own running state; dK / dV of a
    chunk accumulate over the spans.  Chunks a span cannot see cost a kernel launch that returns
    at once (whole-chunk skipping, paper Sec. 2.6)."""

    def __init__(self, Q_spans, q_offs, scale, causal=True, window=0):
        self.walks = [RingWalk(Q, scale, causal, off, window) for Q, off in zip(Q_spans, q_offs)]

    def forward(self, Ks, Vs, k_offs):
        return [w.forward(Ks, Vs, k_offs) for w in self.walks]

    def backward(self, Ks, Vs, k_offs, dO_spans):
        dev = Ks[0].device
        dKs = [torch.empty(tuple(K.shape), device=dev, dtype=torch.float32) for K in Ks]
        dVs = [torch.empty(tuple(V.shape), device=dev, dtype=torch.float32) for V in Vs]
        dQs = []
        for i, (w, dO) in enumerate(zip(self.walks, dO_spans)):
            dQ = torch.zeros((w.Bt, w.H, w.Nq, w.d), device=dev, dtype=torch.float32)
            w.prepare(dO)
            for j in range(len(Ks)):
                B.burst_local_bwd(w.Q, Ks[j], Vs[j], w.O, dO, w.lse, w.D, dQ, dKs[j], dVs[j],
                                  w.params(Ks[j].shape[2], k_offs[j]), accumulate_dq=True, accumulate_dkv=(i > 0))
            dQs.append(dQ)
        return dQs, dKs, dVs


class KeyPinnedBackward:
    """Alg. 2 in the orientation the paper prints (Sec. 2.3; double buffer of Sec. 2.5 / Alg. 4): this
    device keeps K_i, V_i and accumulates dK_i, dV_i while the query-side payloads
    (Q_j, dO_j, D_j, lse_j, dQ_j) of all devices pass through.  Each payload is copied from its
    source (another HBM allocation or pinned host memory: the stand-in for the ring neighbour)
    into one of two receive buffers on a copy stream while the previous one is processed; its
    dQ_j gets this device's contribution added and is copied back (the "send")."""

    def __init__(self, K_i, V_i, scale, causal=False, k_off=0, window=0):
        self.K, self.V = K_i, V_i
        self.Bt, self.Hkv, self.Nc, self.d = K_i.shape
        self.scale, self.causal, self.k_off, self.window = float(scale), bool(causal), int(k_off), int(window)
        dev = K_i.device
        self.dK = torch.empty(tuple(K_i.shape), device=dev, dtype=torch.float32)
        self.dV = torch.empty_like(self.dK)
        self.copy_stream = torch.cuda.Stream(device=dev)

    def backward(self, payloads):
        """payloads: list of dicts with Q, dO [B,H,Nq_j,d], D, lse [B,H,Nq_j], dQ [B,H,Nq_j,d] fp32
        (read, updated and written back) and q_off.  Returns (dK_i, dV_i)."""
        dev = self.K.device
        main = torch.cuda.current_stream(dev)
        n = len(payloads)
        bufs = [None, None]
        ready = [torch.cuda.Event() for _ in range(n)]
        done = [torch.cuda.Event() for _ in range(n)]
        names = ("Q", "dO", "D", "lse", "dQ")

        def fetch(j):
            with torch.cuda.stream(self.copy_stream):
                if j >= 2:
                    self.copy_stream.wait_event(done[j - 2])      # the buffer's previous payload went back
                src = payloads[j]
                if bufs[j % 2] is None or any(bufs[j % 2][k].shape != src[k].shape for k in names):
                    bufs[j % 2] = {k: torch.empty(tuple(src[k].shape), device=dev, dtype=src[k].dtype) for k in names}
                for k in names:
                    bufs[j % 2][k].copy_(src[k], non_blocking=True)
                ready[j].record(self.copy_stream)

        self.copy_stream.wait_stream(main)
        if n:
            fetch(0)
        for j in range(n):
            if j + 1 < n:
                fetch(j + 1)
            main.wait_event(ready[j])
            b = bufs[j % 2]
            H, Nq = b["Q"].shape[1], b["Q"].shape[2]
            p = B.params(self.Bt, H, Nq, self.Nc, self.d, b["Q"].dtype, self.scale, self.causal,
                         payloads[j]["q_off"], self.k_off, self.window, None, 0, self.Hkv if self.Hkv != H else 0)
            B.burst_local_bwd(b["Q"], self.K, self.V, None, b["dO"], b["lse"], b["D"], b["dQ"], self.dK, self.dV, p,
                              accumulate_dq=True, accumulate_dkv=(j > 0))
            payloads[j]["dQ"].copy_(b["dQ"], non_blocking=True)  # on the compute stream, after the kernels
            done[j].record(main)
        return self.dK, self.dV

