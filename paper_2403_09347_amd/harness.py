"""Single-GPU harness: walks G key/value chunks resident in HBM, one library call per chunk,
in the order a device of the ring would receive them (paper Alg. 1 / Alg. 2 loops with the
ring step replaced by taking the next resident chunk).  Host-side orchestration only."""
import torch

from . import binding as B


class RingWalk:
    """Buffers and call sequence for one query slice against a list of chunks."""

    def __init__(self, Q, scale, causal=False, q_off=0):
        assert Q.dim() == 4
        self.Q = Q
        self.Bt, self.H, self.Nq, self.d = Q.shape
        self.scale, self.causal, self.q_off = float(scale), bool(causal), int(q_off)
        dev = Q.device
        self.O_acc = torch.empty((self.Bt, self.H, self.Nq, self.d), device=dev, dtype=torch.float32)
        self.m = torch.empty((self.Bt, self.H, self.Nq), device=dev, dtype=torch.float32)
        self.l = torch.empty_like(self.m)
        self.O = torch.empty_like(Q)
        self.lse = torch.empty_like(self.m)
        self.D = torch.empty_like(self.m)

    def params(self, Nc, k_off):
        return B.params(self.Bt, self.H, self.Nq, Nc, self.d, self.Q.dtype, self.scale,
                        self.causal, self.q_off, k_off)

    # ---- forward (Alg. 1)
    def init(self):
        B.burst_state_init(self.O_acc, self.m, self.l, self.params(0, 0))

    def step(self, K_c, V_c, k_off):
        B.burst_local_fwd(self.Q, K_c, V_c, self.O_acc, self.m, self.l, self.params(K_c.shape[2], k_off))

    def finalize(self):
        B.burst_finalize(self.O_acc, self.m, self.l, self.O, self.lse, self.params(0, 0))
        return self.O, self.lse

    def forward(self, Ks, Vs, k_offs, order=None):
        self.init()
        for j in (range(len(Ks)) if order is None else order):
            self.step(Ks[j], Vs[j], k_offs[j])
        return self.finalize()

    # ---- backward (Alg. 2), query slice pinned, chunks walked
    def prepare(self, dO):
        B.burst_bwd_prepare(self.O, dO, self.D, self.params(0, 0))

    def backward(self, Ks, Vs, k_offs, dO, dQ=None, dKs=None, dVs=None, use_D=True):
        dev = self.Q.device
        if dQ is None:
            dQ = torch.zeros((self.Bt, self.H, self.Nq, self.d), device=dev, dtype=torch.float32)
        if dKs is None:
            dKs = [torch.empty(K.shape, device=dev, dtype=torch.float32) for K in Ks]
            dVs = [torch.empty(V.shape, device=dev, dtype=torch.float32) for V in Vs]
        if use_D:
            self.prepare(dO)
        for j in range(len(Ks)):
            B.burst_local_bwd(self.Q, Ks[j], Vs[j], self.O, dO, self.lse, self.D if use_D else None,
                              dQ, dKs[j], dVs[j], self.params(Ks[j].shape[2], k_offs[j]),
                              accumulate_dq=True, accumulate_dkv=False)
        return dQ, dKs, dVs
