"""fp64 CPU oracle for one device's share of the BurstAttention ring.

THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  Only the test-suite, the smoke
check and the benchmark's `cpu_baseline` leg may import it.  It shares no code
with the HIP path and never calls it; it is plain numpy in float64, slow and
written so that it can be checked against the paper by eye.

Two independent routines live here:

* `full_*`    -- the definition (paper Eq. 1): S = scale * Q K^T over ALL keys,
                 P = softmax(S) row-wise, O = P V, and the textbook gradient of
                 that map (softmax Jacobian).  No chunks, no running state.
* `gao_*`     -- the paper's algorithm done naively: Alg. 1 (forward of global
                 attention optimisation: per-chunk S, rowmax, exp, rowsum, PV,
                 then the online-softmax merge and the final normalisation)
                 and Alg. 2 (backward that recomputes S and P from the saved
                 lse and D = rowsum(dO o O)).  Each S_ij / P_ij is stored in
                 full, one chunk at a time, with no tiling or fusion.

Readings of the paper taken here (the paper is silent or inconsistent):

* The 1/sqrt(d) of Eq. 1 / Eq. 2 is missing from the listings of Alg. 1 and
  Alg. 2.  Here S = scale * Q K^T everywhere and therefore
  dQ = scale * dS K and dK = scale * dS^T Q.  `scale` is an argument.
* Masking is not part of the paper.  A key at global position kp is visible to
  a query at global position qp iff kp <= qp when `causal` is set; masked
  scores are -inf.
* Sec. 2.6 lets local attention skip the similarities a sparse pattern does not
  need.  The one pattern taken here is a sliding window: with `window` = w > 0
  a key is visible only if kp > qp - w (the query itself and its w - 1
  predecessors when combined with `causal`); w = 0 means no window.  Skipped
  pairs behave exactly like masked ones (score -inf).  Any other pattern is
  given as a boolean matrix `pattern` [Nq, Nk] that is ANDed with the above;
  `block_visibility` expands a matrix of block flags (one flag per
  block x block square of the query-slice x chunk pair) into such a matrix.
* Alg. 1 initialises m = -inf.  When m_new = -inf (a row sees no key of the
  chunk and has seen none before) both rescale factors are taken as 0, so a
  fully masked chunk leaves the state unchanged.  Finalising a row with l = 0
  gives O = 0 and lse = -inf; the backward treats exp(S - (-inf)) of such a
  row as 0.

All per-head functions take 2-D arrays (rows x d).  `q_pos` / `k_pos` are the
global positions (int64) of the query rows / key rows; they default to
`q_off + arange` and `k_off + arange`.
"""
import numpy as np

F64 = np.float64


def _f64(x):
    return np.ascontiguousarray(np.asarray(x, dtype=F64))


def visibility(q_pos, k_pos, causal, window=0):
    """Boolean [Nq, Nk]: True where the key may be attended to."""
    q_pos = np.asarray(q_pos, dtype=np.int64)
    k_pos = np.asarray(k_pos, dtype=np.int64)
    vis = np.ones((q_pos.shape[0], k_pos.shape[0]), dtype=bool)
    if causal:
        vis &= k_pos[None, :] <= q_pos[:, None]
    if window:
        vis &= k_pos[None, :] > q_pos[:, None] - int(window)
    return vis


def block_visibility(nq, nk, flags, block):
    """Boolean [nq, nk]: entry (r, c) is flags[r // block, c // block] != 0."""
    flags = np.asarray(flags)
    assert flags.shape == (-(-nq // block), -(-nk // block)), (flags.shape, nq, nk, block)
    return flags[np.arange(nq) // block][:, np.arange(nk) // block] != 0


# --------------------------------------------------------------------------
# The definition: Eq. 1 and its gradient
# --------------------------------------------------------------------------
def full_forward(Q, K, V, scale, causal=False, q_pos=None, k_pos=None,
                 return_p=False, window=0, pattern=None):
    """Eq. 1 on one head.  Returns O [Nq,d], lse [Nq] (and P if asked)."""
    Q, K, V = _f64(Q), _f64(K), _f64(V)
    nq, nk = Q.shape[0], K.shape[0]
    q_pos = np.arange(nq) if q_pos is None else q_pos
    k_pos = np.arange(nk) if k_pos is None else k_pos
    S = scale * (Q @ K.T)
    vis = visibility(q_pos, k_pos, causal, window)
    if pattern is not None:
        vis &= np.asarray(pattern, dtype=bool)
    S = np.where(vis, S, -np.inf)
    if nk == 0:
        row_max = np.full(nq, -np.inf)
    else:
        row_max = S.max(axis=1)
    safe_max = np.where(np.isfinite(row_max), row_max, 0.0)
    E = np.exp(S - safe_max[:, None])          # masked entries: exp(-inf) = 0
    denom = E.sum(axis=1)
    with np.errstate(divide="ignore", invalid="ignore"):
        P = np.where(denom[:, None] > 0, E / denom[:, None], 0.0)
        lse = np.where(denom > 0, safe_max + np.log(denom), -np.inf)
    O = P @ V
    if return_p:
        return O, lse, P
    return O, lse


def full_backward(Q, K, V, dO, scale, causal=False, q_pos=None, k_pos=None,
                  return_ds=False, window=0, pattern=None):
    """Gradient of L = sum(O o dO) w.r.t. Q, K, V from the softmax Jacobian.

    dV = P^T dO;  dP = dO V^T;  dS = P o (dP - rowsum(P o dP));
    dQ = scale dS K;  dK = scale dS^T Q.
    """
    Q, K, V, dO = _f64(Q), _f64(K), _f64(V), _f64(dO)
    _, _, P = full_forward(Q, K, V, scale, causal, q_pos, k_pos, return_p=True, window=window, pattern=pattern)
    dV = P.T @ dO
    dP = dO @ V.T
    dS = P * (dP - (P * dP).sum(axis=1, keepdims=True))
    dQ = scale * (dS @ K)
    dK = scale * (dS.T @ Q)
    if return_ds:
        return dQ, dK, dV, dS
    return dQ, dK, dV


# --------------------------------------------------------------------------
# The algorithm: Alg. 1 (forward) step by step
# --------------------------------------------------------------------------
def gao_state_init(nq, d):
    """Alg. 1, initialisation: O_i = 0, l_i = 0, m_i = -inf."""
    return np.zeros((nq, d), F64), np.full(nq, -np.inf, F64), np.zeros(nq, F64)


def gao_local_forward(Q, K_j, V_j, scale, vis=None):
    """Alg. 1, local attention of one chunk (no LAO): returns O_ij, m_ij, l_ij.

    S_ij = scale Q K_j^T; m_ij = rowmax; P_ij = exp(S_ij - m_ij);
    l_ij = rowsum(P_ij); O_ij = P_ij V_j  (unnormalised partial result).
    """
    S_ij, m_ij, P_ij = gao_local_scores(Q, K_j, scale, vis)
    l_ij = P_ij.sum(axis=1)
    O_ij = P_ij @ _f64(V_j)
    return O_ij, m_ij, l_ij


def gao_local_scores(Q, K_j, scale, vis=None):
    """Alg. 1, the first three steps of the local attention of one chunk, with their
    intermediate matrices returned: S_ij = scale Q K_j^T (hidden entries -inf),
    m_ij = rowmax(S_ij), P_ij = exp(S_ij - m_ij)."""
    Q, K_j = _f64(Q), _f64(K_j)
    S_ij = scale * (Q @ K_j.T)
    if vis is not None:
        S_ij = np.where(vis, S_ij, -np.inf)
    if S_ij.shape[1] == 0:
        m_ij = np.full(Q.shape[0], -np.inf)
    else:
        m_ij = S_ij.max(axis=1)
    shift = np.where(np.isfinite(m_ij), m_ij, 0.0)   # rows with no visible key
    P_ij = np.exp(S_ij - shift[:, None])
    return S_ij, m_ij, P_ij


def gao_merge(O_i, m_i, l_i, O_ij, m_ij, l_ij):
    """Alg. 1, online-softmax merge of a partial result into the running state.

    m_new = max(m_i, m_ij); l_i = e^{m_i-m_new} l_i + e^{m_ij-m_new} l_ij;
    O_i likewise; m_i = m_new.  With m_new = -inf both factors are 0.
    """
    m_new = np.maximum(m_i, m_ij)
    finite = np.isfinite(m_new)
    ref = np.where(finite, m_new, 0.0)
    with np.errstate(invalid="ignore"):
        a = np.where(finite, np.exp(m_i - ref), 0.0)     # exp(-inf - x) = 0
        b = np.where(finite, np.exp(m_ij - ref), 0.0)
    l_out = a * l_i + b * l_ij
    O_out = a[:, None] * O_i + b[:, None] * O_ij
    return O_out, m_new, l_out


def gao_finalize(O_i, m_i, l_i):
    """Alg. 1, last two steps: O_i = diag(l_i)^-1 O_i; lse_i = m_i + log l_i."""
    with np.errstate(divide="ignore", invalid="ignore"):
        O = np.where(l_i[:, None] > 0, O_i / l_i[:, None], 0.0)
        lse = np.where(l_i > 0, m_i + np.log(l_i), -np.inf)
    return O, lse


def gao_forward(Q, K_chunks, V_chunks, scale, causal=False, q_pos=None,
                k_pos_chunks=None, order=None, window=0, pattern_chunks=None):
    """Alg. 1 on one head over a list of K/V chunks, visited in `order`.
    pattern_chunks: optional list of boolean [Nq, Nc_j] matrices (Sec. 2.6 patterns)."""
    Q = _f64(Q)
    nq, d = Q.shape
    q_pos = np.arange(nq) if q_pos is None else q_pos
    if k_pos_chunks is None:
        k_pos_chunks, start = [], 0
        for K_j in K_chunks:
            k_pos_chunks.append(np.arange(start, start + len(K_j)))
            start += len(K_j)
    order = range(len(K_chunks)) if order is None else order
    O_i, m_i, l_i = gao_state_init(nq, d)
    for j in order:
        vis = visibility(q_pos, k_pos_chunks[j], causal, window) if (causal or window) else None
        if pattern_chunks is not None:
            vis = np.asarray(pattern_chunks[j], dtype=bool) & (True if vis is None else vis)
        O_ij, m_ij, l_ij = gao_local_forward(Q, K_chunks[j], V_chunks[j], scale, vis)
        O_i, m_i, l_i = gao_merge(O_i, m_i, l_i, O_ij, m_ij, l_ij)
    return gao_finalize(O_i, m_i, l_i)


# --------------------------------------------------------------------------
# The algorithm: Alg. 2 (backward) step by step
# --------------------------------------------------------------------------
def gao_bwd_prepare(O, dO):
    """Alg. 2, pre-step: D = rowsum(dO o O)."""
    return (_f64(dO) * _f64(O)).sum(axis=1)


def gao_local_backward_matrices(Q, K_c, V_c, dO, lse, D, scale, vis=None):
    """Alg. 2, one block pair, the matrices of the loop body: S = scale Q K_c^T;
    P = exp(S - lse); dP = dO V_c^T; dS = P o (dP - D).  Returns (P, dP, dS)."""
    Q, K_c, V_c, dO = _f64(Q), _f64(K_c), _f64(V_c), _f64(dO)
    lse, D = _f64(lse), _f64(D)
    S = scale * (Q @ K_c.T)
    if vis is not None:
        S = np.where(vis, S, -np.inf)
    live = np.isfinite(lse)                      # rows that saw at least one key
    ref = np.where(live, lse, 0.0)
    P = np.where(live[:, None], np.exp(S - ref[:, None]), 0.0)
    dP = dO @ V_c.T
    dS = P * (dP - D[:, None])
    return P, dP, dS


def gao_local_backward(Q, K_c, V_c, dO, lse, D, scale, vis=None):
    """Alg. 2, one block pair: returns (dQ contribution, dK_c, dV_c).

    With P, dP, dS as above: dV = P^T dO; dK = scale dS^T Q; dQ = scale dS K_c.
    """
    P, _, dS = gao_local_backward_matrices(Q, K_c, V_c, dO, lse, D, scale, vis)
    Q, K_c, dO = _f64(Q), _f64(K_c), _f64(dO)
    dV = P.T @ dO
    dK = scale * (dS.T @ Q)
    dQ = scale * (dS @ K_c)
    return dQ, dK, dV


def gao_backward(Q, K_chunks, V_chunks, O, dO, lse, scale, causal=False,
                 q_pos=None, k_pos_chunks=None, window=0, pattern_chunks=None):
    """Alg. 2 on one head with Q pinned and the K/V chunks walked in order.

    Returns dQ [Nq,d] and lists dK_chunks, dV_chunks.
    """
    Q = _f64(Q)
    nq = Q.shape[0]
    q_pos = np.arange(nq) if q_pos is None else q_pos
    if k_pos_chunks is None:
        k_pos_chunks, start = [], 0
        for K_j in K_chunks:
            k_pos_chunks.append(np.arange(start, start + len(K_j)))
            start += len(K_j)
    D = gao_bwd_prepare(O, dO)
    dQ = np.zeros_like(Q)
    dKs, dVs = [], []
    for j in range(len(K_chunks)):
        vis = visibility(q_pos, k_pos_chunks[j], causal, window) if (causal or window) else None
        if pattern_chunks is not None:
            vis = np.asarray(pattern_chunks[j], dtype=bool) & (True if vis is None else vis)
        dq, dk, dv = gao_local_backward(Q, K_chunks[j], V_chunks[j], dO, lse, D, scale, vis)
        dQ += dq
        dKs.append(dk)
        dVs.append(dv)
    return dQ, dKs, dVs


# --------------------------------------------------------------------------
# Multi-head helpers (plain loops over batch and head)
# --------------------------------------------------------------------------
def full_forward_bh(Q, K, V, scale, causal=False, q_off=0, k_off=0, window=0):
    """Q [B,H,Nq,d], K,V [B,H,Nk,d] -> O [B,H,Nq,d], lse [B,H,Nq]."""
    B, H, nq, d = Q.shape
    nk = K.shape[2]
    O = np.empty((B, H, nq, d), F64)
    lse = np.empty((B, H, nq), F64)
    qp, kp = q_off + np.arange(nq), k_off + np.arange(nk)
    for b in range(B):
        for h in range(H):
            O[b, h], lse[b, h] = full_forward(Q[b, h], K[b, h], V[b, h], scale, causal, qp, kp, window=window)
    return O, lse


def full_backward_bh(Q, K, V, dO, scale, causal=False, q_off=0, k_off=0, window=0):
    B, H, nq, d = Q.shape
    nk = K.shape[2]
    dQ = np.empty((B, H, nq, d), F64)
    dK = np.empty((B, H, nk, d), F64)
    dV = np.empty((B, H, nk, d), F64)
    qp, kp = q_off + np.arange(nq), k_off + np.arange(nk)
    for b in range(B):
        for h in range(H):
            dQ[b, h], dK[b, h], dV[b, h] = full_backward(
                Q[b, h], K[b, h], V[b, h], dO[b, h], scale, causal, qp, kp, window=window)
    return dQ, dK, dV
