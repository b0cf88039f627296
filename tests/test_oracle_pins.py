"""Pins for the fp64 oracle: closed forms, invariants, finite differences, brute force.

None of these re-type the oracle's own formula: each checks it against something the
mathematics fixes independently (paper Eq. 1 for the definition, Alg. 1 / Alg. 2 for the
chunked algorithm, whose results must equal the definition's).
"""
import json
import math
import os

import numpy as np
import pytest

from oracle import burst_oracle as orc

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def rng(seed):
    return np.random.default_rng(seed)


def split(X, sizes):
    out, s = [], 0
    for n in sizes:
        out.append(X[s:s + n])
        s += n
    return out


# ---------------------------------------------------------------- hand example
def test_hand_example_forward_backward():
    g = json.load(open(os.path.join(GOLD, "hand_example.json")))
    q = np.array(g["q"])
    K = np.log(np.array(g["K_exp"])).reshape(-1, 1)    # keys are stored as exp(K): [1, 3] -> [0, ln 3]
    V = np.array(g["V"])
    dO = np.array(g["dO"])
    O, lse, P = orc.full_forward(q, K, V, g["scale"], return_p=True)
    assert np.allclose(O, g["O"], atol=1e-14)
    assert np.allclose(np.exp(lse), g["lse_exp"], atol=1e-13)
    assert np.allclose(P, g["P"], atol=1e-15)
    dQ, dK, dV, dS = orc.full_backward(q, K, V, dO, g["scale"], return_ds=True)
    assert np.allclose(dV, g["dV"], atol=1e-15)
    assert np.allclose(dS, g["dS"], atol=1e-15)
    assert np.allclose(dQ, np.array(g["dQ_over_ln3"]) * math.log(3.0), atol=1e-15)
    assert np.allclose(dK, g["dK"], atol=1e-15)
    # same scores through scale=2, q=1/2: dQ doubles, dK unchanged (scale enters dQ, dK once each)
    dQ2, dK2, dV2 = orc.full_backward(q / 2, K, V, dO, 2.0)
    assert np.allclose(dQ2, 2 * dQ, atol=1e-15) and np.allclose(dK2, dK, atol=1e-15)
    assert np.allclose(dV2, dV, atol=1e-15)
    # and the chunked algorithm (one key per chunk) gives the same numbers
    Oc, lsec = orc.gao_forward(q, [K[:1], K[1:]], [V[:1], V[1:]], g["scale"])
    assert np.allclose(Oc, g["O"], atol=1e-14) and np.allclose(np.exp(lsec), g["lse_exp"], atol=1e-13)
    dQc, dKs, dVs = orc.gao_backward(q, [K[:1], K[1:]], [V[:1], V[1:]], Oc, dO, lsec, g["scale"])
    assert np.allclose(dQc, dQ, atol=1e-15)
    assert np.allclose(np.concatenate(dKs), g["dK"], atol=1e-15)
    assert np.allclose(np.concatenate(dVs), g["dV"], atol=1e-15)


# ---------------------------------------------------------------- brute force
def brute_force(Q, K, V, dO, scale, causal, q_pos, k_pos):
    """Scalar loops in extended precision, written from Eq. 1 and the chain rule."""
    LD = np.longdouble
    nq, d = Q.shape
    nk = K.shape[0]
    O = np.zeros((nq, d), LD)
    lse = np.zeros(nq, LD)
    dQ = np.zeros((nq, d), LD)
    dK = np.zeros((nk, d), LD)
    dV = np.zeros((nk, d), LD)
    for r in range(nq):
        cols = [c for c in range(nk) if (not causal) or k_pos[c] <= q_pos[r]]
        s = {}
        for c in cols:
            acc = LD(0)
            for t in range(d):
                acc += LD(Q[r, t]) * LD(K[c, t])
            s[c] = acc * LD(scale)
        mx = max(s.values())
        z = sum(np.exp(s[c] - mx) for c in cols)
        lse[r] = mx + np.log(z)
        p = {c: np.exp(s[c] - mx) / z for c in cols}
        for t in range(d):
            O[r, t] = sum(p[c] * LD(V[c, t]) for c in cols)
        # dL/dp_c = dO_r . V_c ; softmax Jacobian: ds_c = p_c (dp_c - sum_k p_k dp_k)
        dp = {c: sum(LD(dO[r, t]) * LD(V[c, t]) for t in range(d)) for c in cols}
        avg = sum(p[c] * dp[c] for c in cols)
        for c in cols:
            ds = p[c] * (dp[c] - avg)
            for t in range(d):
                dV[c, t] += p[c] * LD(dO[r, t])
                dQ[r, t] += LD(scale) * ds * LD(K[c, t])
                dK[c, t] += LD(scale) * ds * LD(Q[r, t])
    return [np.asarray(x, np.float64) for x in (O, lse, dQ, dK, dV)]


@pytest.mark.parametrize("causal", [False, True])
def test_full_and_chunked_match_brute_force(causal):
    r = rng(11)
    nq, nk, d = 13, 16, 8
    Q, K, V, dO = r.normal(size=(nq, d)), r.normal(size=(nk, d)), r.normal(size=(nk, d)), r.normal(size=(nq, d))
    scale = 0.37
    q_pos = 5 + np.arange(nq)            # first query sees keys 0..5, last sees all 16
    k_pos = np.arange(nk)
    O, lse, dQ, dK, dV = brute_force(Q, K, V, dO, scale, causal, q_pos, k_pos)
    Of, lsef = orc.full_forward(Q, K, V, scale, causal, q_pos, k_pos)
    dQf, dKf, dVf = orc.full_backward(Q, K, V, dO, scale, causal, q_pos, k_pos)
    for a, b in ((O, Of), (lse, lsef), (dQ, dQf), (dK, dKf), (dV, dVf)):
        assert np.max(np.abs(a - b)) < 1e-13
    sizes = [5, 1, 7, 3]
    kp = split(k_pos, sizes)
    Oc, lsec = orc.gao_forward(Q, split(K, sizes), split(V, sizes), scale, causal, q_pos, kp)
    dQc, dKs, dVs = orc.gao_backward(Q, split(K, sizes), split(V, sizes), Oc, dO, lsec, scale, causal, q_pos, kp)
    for a, b in ((O, Oc), (lse, lsec), (dQ, dQc), (dK, np.concatenate(dKs)), (dV, np.concatenate(dVs))):
        assert np.max(np.abs(a - b)) < 1e-13


# ---------------------------------------------------------------- definition <-> algorithm
@pytest.mark.parametrize("sizes", [[96], [48, 48], [24, 24, 24, 24], [10, 20, 5, 30, 1, 17, 13]])
@pytest.mark.parametrize("causal", [False, True])
def test_chunked_equals_full(sizes, causal):
    r = rng(3 + len(sizes))
    nk, nq, d = sum(sizes), 40, 16
    Q, K, V, dO = r.normal(size=(nq, d)), r.normal(size=(nk, d)), r.normal(size=(nk, d)), r.normal(size=(nq, d))
    scale = 1 / math.sqrt(d)
    q_pos = (nk - nq) + np.arange(nq)
    k_pos = np.arange(nk)
    Of, lsef = orc.full_forward(Q, K, V, scale, causal, q_pos, k_pos)
    dQf, dKf, dVf = orc.full_backward(Q, K, V, dO, scale, causal, q_pos, k_pos)
    Ks, Vs, kp = split(K, sizes), split(V, sizes), split(k_pos, sizes)
    G = len(sizes)
    for order in (list(range(G)), list(range(G))[::-1], [(j + 2) % G for j in range(G)]):
        Oc, lsec = orc.gao_forward(Q, Ks, Vs, scale, causal, q_pos, kp, order=order)
        assert np.max(np.abs(Oc - Of)) < 1e-12 and np.max(np.abs(lsec - lsef)) < 1e-12
    dQc, dKs, dVs = orc.gao_backward(Q, Ks, Vs, Of, dO, lsef, scale, causal, q_pos, kp)
    assert np.max(np.abs(dQc - dQf)) < 1e-12
    assert np.max(np.abs(np.concatenate(dKs) - dKf)) < 1e-12
    assert np.max(np.abs(np.concatenate(dVs) - dVf)) < 1e-12


# ---------------------------------------------------------------- closed forms
def test_zero_query_gives_mean_of_values():
    r = rng(5)
    nk, d = 37, 12
    K, V = r.normal(size=(nk, d)), r.normal(size=(nk, d))
    Q = np.zeros((6, d))
    for fwd in (lambda: orc.full_forward(Q, K, V, 0.3),
                lambda: orc.gao_forward(Q, split(K, [10, 27]), split(V, [10, 27]), 0.3)):
        O, lse = fwd()
        assert np.allclose(O, V.mean(axis=0)[None, :], atol=1e-14)
        assert np.allclose(lse, math.log(nk), atol=1e-14)


def test_zero_query_causal_gives_prefix_means():
    r = rng(6)
    nk, d = 20, 5
    K, V = r.normal(size=(nk, d)), r.normal(size=(nk, d))
    Q = np.zeros((nk, d))
    prefix = np.cumsum(V, axis=0) / np.arange(1, nk + 1)[:, None]
    O, lse = orc.full_forward(Q, K, V, 1.0, causal=True)
    assert np.allclose(O, prefix, atol=1e-14)
    assert np.allclose(lse, np.log(np.arange(1, nk + 1)), atol=1e-14)
    sizes = [7, 7, 6]
    O, lse = orc.gao_forward(Q, split(K, sizes), split(V, sizes), 1.0, causal=True)
    assert np.allclose(O, prefix, atol=1e-14)
    assert np.allclose(lse, np.log(np.arange(1, nk + 1)), atol=1e-14)
    # offset queries: row r at global position 3+r sees 4+r keys
    O, lse = orc.full_forward(Q[:10], K, V, 1.0, causal=True, q_pos=3 + np.arange(10))
    assert np.allclose(O, prefix[3:13], atol=1e-14)


def test_single_key():
    r = rng(7)
    d = 9
    Q, dO = r.normal(size=(4, d)), r.normal(size=(4, d))
    K, V = r.normal(size=(1, d)), r.normal(size=(1, d))
    O, lse = orc.full_forward(Q, K, V, 0.5)
    assert np.allclose(O, np.repeat(V, 4, axis=0), atol=1e-15)
    assert np.allclose(lse, 0.5 * (Q @ K.T)[:, 0], atol=1e-14)
    dQ, dK, dV = orc.full_backward(Q, K, V, dO, 0.5)
    assert np.allclose(dQ, 0, atol=1e-15) and np.allclose(dK, 0, atol=1e-15)
    assert np.allclose(dV, dO.sum(axis=0, keepdims=True), atol=1e-14)
    dQc, dKs, dVs = orc.gao_backward(Q, [K], [V], O, dO, lse, 0.5)
    assert np.allclose(dQc, 0, atol=1e-15) and np.allclose(dKs[0], 0, atol=1e-15)
    assert np.allclose(dVs[0], dO.sum(axis=0, keepdims=True), atol=1e-14)


def test_equal_value_rows_and_key_shift():
    r = rng(8)
    nq, nk, d = 7, 19, 6
    Q, K = r.normal(size=(nq, d)), r.normal(size=(nk, d))
    v = r.normal(size=(1, d))
    O, _ = orc.full_forward(Q, K, np.repeat(v, nk, axis=0), 0.4)
    assert np.allclose(O, np.repeat(v, nq, axis=0), atol=1e-14)
    V = r.normal(size=(nk, d))
    c = r.normal(size=(1, d))
    O0, lse0 = orc.full_forward(Q, K, V, 0.4)
    O1, lse1 = orc.gao_forward(Q, split(K + c, [9, 10]), split(V, [9, 10]), 0.4)
    assert np.allclose(O0, O1, atol=1e-13)
    assert np.allclose(lse1 - lse0, 0.4 * (Q @ c.T)[:, 0], atol=1e-13)


def test_two_keys_sigmoid():
    # two keys: p_1 = sigmoid(s_1 - s_0), a textbook special case of softmax
    q = np.array([[0.7, -1.2]])
    K = np.array([[0.3, 0.9], [-0.5, 0.2]])
    V = np.array([[1.0, 0.0], [0.0, 1.0]])
    scale = 1.3
    s = scale * (K @ q[0])
    p1 = 1.0 / (1.0 + math.exp(-(s[1] - s[0])))
    O, lse = orc.full_forward(q, K, V, scale)
    assert np.allclose(O, [[1 - p1, p1]], atol=1e-15)
    assert abs(lse[0] - math.log(math.exp(s[0]) + math.exp(s[1]))) < 1e-15


# ---------------------------------------------------------------- invariants
@pytest.mark.parametrize("causal", [False, True])
def test_invariants(causal):
    r = rng(9)
    nq, nk, d = 24, 24, 10
    Q, K, V, dO = (r.normal(size=(n, d)) for n in (nq, nk, nk, nq))
    scale = 0.31
    O, lse, P = orc.full_forward(Q, K, V, scale, causal, return_p=True)
    assert np.allclose(P.sum(axis=1), 1.0, atol=1e-14)
    vis = orc.visibility(np.arange(nq), np.arange(nk), causal)
    S = scale * Q @ K.T
    assert np.allclose(np.where(vis, np.exp(S - lse[:, None]), 0.0).sum(axis=1), 1.0, atol=1e-13)
    assert np.all(P[~vis] == 0.0)
    dQ, dK, dV, dS = orc.full_backward(Q, K, V, dO, scale, causal, return_ds=True)
    assert np.allclose(dS.sum(axis=1), 0.0, atol=1e-14)
    # Alg. 2's D = rowsum(dO o O) equals the Jacobian's rowsum(P o dP)
    assert np.allclose(orc.gao_bwd_prepare(O, dO), (P * (dO @ V.T)).sum(axis=1), atol=1e-13)
    assert np.allclose(dV.sum(axis=0), dO.sum(axis=0), atol=1e-12)      # columns of P^T sum rows of dO
    assert abs((Q * dQ).sum() - (K * dK).sum()) < 1e-12                  # L invariant under Q->aQ, K->K/a


def test_merge_identity_and_split_merge():
    r = rng(10)
    nq, d = 9, 7
    Q = r.normal(size=(nq, d))
    Ks = [r.normal(size=(n, d)) for n in (5, 8, 3, 6)]
    Vs = [r.normal(size=(n, d)) for n in (5, 8, 3, 6)]
    scale = 0.5
    st = orc.gao_state_init(nq, d)
    for j in range(4):
        st = orc.gao_merge(*st, *orc.gao_local_forward(Q, Ks[j], Vs[j], scale))
    # merging an empty chunk or a fully masked chunk is the identity
    empty = orc.gao_local_forward(Q, np.zeros((0, d)), np.zeros((0, d)), scale)
    masked = orc.gao_local_forward(Q, Ks[0], Vs[0], scale, vis=np.zeros((nq, 5), bool))
    for part in (empty, masked):
        st2 = orc.gao_merge(*st, *part)
        assert all(np.array_equal(a, b) for a, b in zip(st, st2))
        st3 = orc.gao_merge(*orc.gao_state_init(nq, d), *part)   # into a fresh state: still fresh
        assert np.all(st3[0] == 0) and np.all(st3[2] == 0) and np.all(np.isneginf(st3[1]))
    # two half walks merged == straight walk
    a = orc.gao_state_init(nq, d)
    b = orc.gao_state_init(nq, d)
    for j in (0, 1):
        a = orc.gao_merge(*a, *orc.gao_local_forward(Q, Ks[j], Vs[j], scale))
    for j in (2, 3):
        b = orc.gao_merge(*b, *orc.gao_local_forward(Q, Ks[j], Vs[j], scale))
    O1, lse1 = orc.gao_finalize(*orc.gao_merge(*a, *b))
    O0, lse0 = orc.gao_finalize(*st)
    assert np.allclose(O0, O1, atol=1e-14) and np.allclose(lse0, lse1, atol=1e-14)
    # finalising a fresh state: O = 0, lse = -inf (a row that saw nothing)
    Oz, lsez = orc.gao_finalize(*orc.gao_state_init(nq, d))
    assert np.all(Oz == 0) and np.all(np.isneginf(lsez))


def test_rows_that_see_nothing_contribute_nothing_in_backward():
    r = rng(12)
    nq, nk, d = 6, 4, 5
    Q, K, V, dO = (r.normal(size=(n, d)) for n in (nq, nk, nk, nq))
    q_pos = np.array([-3, -1, 0, 1, 2, 9])       # rows 0,1 see no key at all
    k_pos = np.arange(nk)
    O, lse = orc.full_forward(Q, K, V, 1.0, True, q_pos, k_pos)
    assert np.all(O[:2] == 0) and np.all(np.isneginf(lse[:2])) and np.all(np.isfinite(lse[2:]))
    dQ, dK, dV = orc.full_backward(Q, K, V, dO, 1.0, True, q_pos, k_pos)
    dQc, dKs, dVs = orc.gao_backward(Q, [K], [V], O, dO, lse, 1.0, True, q_pos, [k_pos])
    assert np.all(dQ[:2] == 0) and np.all(dQc[:2] == 0)
    assert np.allclose(dQ, dQc, atol=1e-14) and np.allclose(dK, dKs[0], atol=1e-14) and np.allclose(dV, dVs[0], atol=1e-14)


# ---------------------------------------------------------------- finite differences
@pytest.mark.parametrize("causal", [False, True])
def test_backward_matches_central_differences(causal):
    r = rng(13)
    nq, nk, d = 6, 9, 4
    Q, K, V, dO = (r.normal(size=(n, d)) for n in (nq, nk, nk, nq))
    scale = 0.45
    sizes = [4, 5]
    q_pos = 3 + np.arange(nq)
    k_pos = np.arange(nk)

    def loss(Q_, K_, V_):
        O, _ = orc.full_forward(Q_, K_, V_, scale, causal, q_pos, k_pos)
        return (O * dO).sum()

    O, lse = orc.gao_forward(Q, split(K, sizes), split(V, sizes), scale, causal, q_pos, split(k_pos, sizes))
    dQ, dKs, dVs = orc.gao_backward(Q, split(K, sizes), split(V, sizes), O, dO, lse, scale, causal,
                                    q_pos, split(k_pos, sizes))
    dK, dV = np.concatenate(dKs), np.concatenate(dVs)
    dQf, dKf, dVf = orc.full_backward(Q, K, V, dO, scale, causal, q_pos, k_pos)
    h = 1e-5
    for X, g_alg, g_def, idx in ((Q, dQ, dQf, 0), (K, dK, dKf, 1), (V, dV, dVf, 2)):
        for (i, t) in [(0, 0), (X.shape[0] - 1, d - 1), (X.shape[0] // 2, 1), (1, 2)]:
            args = [Q.copy(), K.copy(), V.copy()]
            args[idx][i, t] += h
            up = loss(*args)
            args[idx][i, t] -= 2 * h
            dn = loss(*args)
            fd = (up - dn) / (2 * h)
            assert abs(fd - g_alg[i, t]) < 1e-8 * max(1.0, abs(fd)), (idx, i, t)
            assert abs(fd - g_def[i, t]) < 1e-8 * max(1.0, abs(fd)), (idx, i, t)


def test_multihead_helpers_loop_over_heads():
    r = rng(14)
    B, H, nq, nk, d = 2, 3, 5, 7, 4
    Q, K, V, dO = (r.normal(size=(B, H, n, d)) for n in (nq, nk, nk, nq))
    O, lse = orc.full_forward_bh(Q, K, V, 0.5, True, q_off=4, k_off=2)
    dQ, dK, dV = orc.full_backward_bh(Q, K, V, dO, 0.5, True, q_off=4, k_off=2)
    o, l = orc.full_forward(Q[1, 2], K[1, 2], V[1, 2], 0.5, True, 4 + np.arange(nq), 2 + np.arange(nk))
    assert np.array_equal(O[1, 2], o) and np.array_equal(lse[1, 2], l)
    dq, dk, dv = orc.full_backward(Q[0, 1], K[0, 1], V[0, 1], dO[0, 1], 0.5, True, 4 + np.arange(nq), 2 + np.arange(nk))
    assert np.array_equal(dQ[0, 1], dq) and np.array_equal(dK[0, 1], dk) and np.array_equal(dV[0, 1], dv)


# ---------------------------------------------------------------- sliding window (Sec. 2.6: skipped similarities)
def test_window_zero_query_gives_means_over_the_window():
    r = rng(21)
    nk, d, w = 23, 4, 5
    K, V = r.normal(size=(nk, d)), r.normal(size=(nk, d))
    Q = np.zeros((nk, d))
    csum = np.vstack([np.zeros((1, d)), np.cumsum(V, axis=0)])
    # causal + window: row r sees keys max(0, r-w+1) .. r
    lo = np.maximum(0, np.arange(nk) - w + 1)
    cnt = np.arange(nk) + 1 - lo
    want = (csum[np.arange(nk) + 1] - csum[lo]) / cnt[:, None]
    O, lse = orc.full_forward(Q, K, V, 1.0, causal=True, window=w)
    assert np.allclose(O, want, atol=1e-14) and np.allclose(lse, np.log(cnt), atol=1e-14)
    O, lse = orc.gao_forward(Q, split(K, [6, 9, 8]), split(V, [6, 9, 8]), 1.0, causal=True, window=w)
    assert np.allclose(O, want, atol=1e-14) and np.allclose(lse, np.log(cnt), atol=1e-14)
    # window without causal: row r sees keys max(0, r-w+1) .. nk-1
    cnt2 = nk - lo
    want2 = (csum[nk] - csum[lo]) / cnt2[:, None]
    O, lse = orc.full_forward(Q, K, V, 1.0, causal=False, window=w)
    assert np.allclose(O, want2, atol=1e-14) and np.allclose(lse, np.log(cnt2), atol=1e-14)


@pytest.mark.parametrize("causal", [False, True])
def test_window_equals_unwindowed_attention_on_the_visible_keys(causal):
    """Row by row: attention with a window = plain attention (no window argument at all) over
    exactly the keys the window leaves visible; the gradients scatter back accordingly."""
    r = rng(22)
    nq, nk, d, w = 11, 17, 6, 4
    Q, K, V, dO = (r.normal(size=(n, d)) for n in (nq, nk, nk, nq))
    scale = 0.3
    q_pos, k_pos = 4 + np.arange(nq), np.arange(nk)
    O, lse = orc.full_forward(Q, K, V, scale, causal, q_pos, k_pos, window=w)
    dQ, dK, dV = orc.full_backward(Q, K, V, dO, scale, causal, q_pos, k_pos, window=w)
    dK2, dV2 = np.zeros_like(K), np.zeros_like(V)
    for i in range(nq):
        keep = [c for c in range(nk) if k_pos[c] > q_pos[i] - w and (not causal or k_pos[c] <= q_pos[i])]
        Oi, lsei = orc.full_forward(Q[i:i + 1], K[keep], V[keep], scale)
        dqi, dki, dvi = orc.full_backward(Q[i:i + 1], K[keep], V[keep], dO[i:i + 1], scale)
        assert np.allclose(O[i], Oi[0], atol=1e-14) and abs(lse[i] - lsei[0]) < 1e-14
        assert np.allclose(dQ[i], dqi[0], atol=1e-14)
        dK2[keep] += dki
        dV2[keep] += dvi
    assert np.allclose(dK, dK2, atol=1e-13) and np.allclose(dV, dV2, atol=1e-13)
    # the chunked algorithm agrees, including chunks that some or all rows cannot see
    sizes = [3, 6, 1, 7]
    kp = split(k_pos, sizes)
    Oc, lsec = orc.gao_forward(Q, split(K, sizes), split(V, sizes), scale, causal, q_pos, kp, window=w)
    dQc, dKs, dVs = orc.gao_backward(Q, split(K, sizes), split(V, sizes), Oc, dO, lsec, scale, causal, q_pos, kp,
                                     window=w)
    for a, b in ((O, Oc), (lse, lsec), (dQ, dQc), (dK, np.concatenate(dKs)), (dV, np.concatenate(dVs))):
        assert np.max(np.abs(a - b)) < 1e-13


def test_window_wider_than_everything_changes_nothing_and_window_one_copies_values():
    r = rng(23)
    nq, nk, d = 7, 12, 5
    Q, K, V, dO = (r.normal(size=(n, d)) for n in (nq, nk, nk, nq))
    q_pos, k_pos = 5 + np.arange(nq), np.arange(nk)
    for causal in (False, True):
        a = orc.full_forward(Q, K, V, 0.5, causal, q_pos, k_pos)
        b = orc.full_forward(Q, K, V, 0.5, causal, q_pos, k_pos, window=10 ** 6)
        assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    # causal, window 1: each query sees only the key at its own position
    O, lse = orc.full_forward(Q, K, V, 0.5, True, q_pos, k_pos, window=1)
    assert np.allclose(O, V[5:12], atol=1e-15)
    assert np.allclose(lse, 0.5 * np.einsum("rd,rd->r", Q, K[5:12]), atol=1e-14)
    dQ, dK, dV = orc.full_backward(Q, K, V, dO, 0.5, True, q_pos, k_pos, window=1)
    assert np.allclose(dQ, 0) and np.allclose(dK, 0)
    assert np.allclose(dV[5:12], dO, atol=1e-15) and np.allclose(dV[:5], 0)


def test_window_backward_matches_central_differences():
    r = rng(24)
    nq, nk, d, w = 6, 10, 3, 4
    Q, K, V, dO = (r.normal(size=(n, d)) for n in (nq, nk, nk, nq))
    scale, q_pos, k_pos = 0.6, 3 + np.arange(nq), np.arange(nk)

    def loss(Q_, K_, V_):
        O, _ = orc.full_forward(Q_, K_, V_, scale, True, q_pos, k_pos, window=w)
        return (O * dO).sum()
    sizes = [4, 6]
    O, lse = orc.gao_forward(Q, split(K, sizes), split(V, sizes), scale, True, q_pos, split(k_pos, sizes), window=w)
    dQ, dKs, dVs = orc.gao_backward(Q, split(K, sizes), split(V, sizes), O, dO, lse, scale, True, q_pos,
                                    split(k_pos, sizes), window=w)
    grads = (dQ, np.concatenate(dKs), np.concatenate(dVs))
    h = 1e-5
    for idx, X in enumerate((Q, K, V)):
        for (i, t) in [(0, 0), (X.shape[0] - 1, d - 1), (X.shape[0] // 2, 1)]:
            args = [Q.copy(), K.copy(), V.copy()]
            args[idx][i, t] += h
            up = loss(*args)
            args[idx][i, t] -= 2 * h
            fd = (up - loss(*args)) / (2 * h)
            assert abs(fd - grads[idx][i, t]) < 1e-8 * max(1.0, abs(fd)), (idx, i, t)


# ---------------------------------------------------------------- block patterns (Sec. 2.6: skipped block pairs)
def test_block_visibility_expands_flags_blockwise():
    flags = np.array([[1, 0, 1], [0, 0, 2]])
    vis = orc.block_visibility(5, 7, flags, 3)          # rows 0-2 / 3-4, columns 0-2 / 3-5 / 6
    assert vis.shape == (5, 7) and vis.dtype == bool
    for r in range(5):
        for c in range(7):
            assert vis[r, c] == (flags[r // 3, c // 3] != 0)
    assert vis.sum() == 3 * 3 + 3 * 1 + 2 * 1


@pytest.mark.parametrize("causal", [False, True])
def test_block_pattern_equals_plain_attention_on_the_visible_keys(causal):
    """Row by row: attention under a block pattern = plain attention (no pattern argument) over
    exactly the keys of the row's visible blocks; gradients scatter back accordingly.  Also the
    chunked algorithm with one flag matrix per chunk, some chunks fully hidden for some rows."""
    r = rng(31)
    nq, nk, d, blk = 10, 16, 5, 4
    Q, K, V, dO = (r.normal(size=(n, d)) for n in (nq, nk, nk, nq))
    scale = 0.4
    q_pos, k_pos = 6 + np.arange(nq), np.arange(nk)
    flags = np.array([[1, 0, 0, 1], [0, 1, 0, 0], [1, 1, 0, 1]])       # 3 row blocks x 4 key blocks
    pattern = orc.block_visibility(nq, nk, flags, blk)
    O, lse = orc.full_forward(Q, K, V, scale, causal, q_pos, k_pos, pattern=pattern)
    dQ, dK, dV = orc.full_backward(Q, K, V, dO, scale, causal, q_pos, k_pos, pattern=pattern)
    dK2, dV2 = np.zeros_like(K), np.zeros_like(V)
    for i in range(nq):
        keep = [c for c in range(nk) if flags[i // blk, c // blk] and (not causal or k_pos[c] <= q_pos[i])]
        assert keep, "every row of this pattern sees something"
        Oi, lsei = orc.full_forward(Q[i:i + 1], K[keep], V[keep], scale)
        dqi, dki, dvi = orc.full_backward(Q[i:i + 1], K[keep], V[keep], dO[i:i + 1], scale)
        assert np.allclose(O[i], Oi[0], atol=1e-14) and abs(lse[i] - lsei[0]) < 1e-14
        assert np.allclose(dQ[i], dqi[0], atol=1e-14)
        dK2[keep] += dki
        dV2[keep] += dvi
    assert np.allclose(dK, dK2, atol=1e-13) and np.allclose(dV, dV2, atol=1e-13)
    sizes = [8, 4, 4]                                   # chunk boundaries on block boundaries
    cols = np.cumsum([0] + sizes)
    pats = [pattern[:, cols[j]:cols[j + 1]] for j in range(3)]
    for j in range(3):                                  # the same thing from per-chunk flag matrices
        fj = flags[:, cols[j] // blk: cols[j + 1] // blk]
        assert np.array_equal(pats[j], orc.block_visibility(nq, sizes[j], fj, blk))
    kp = split(k_pos, sizes)
    Oc, lsec = orc.gao_forward(Q, split(K, sizes), split(V, sizes), scale, causal, q_pos, kp, pattern_chunks=pats)
    dQc, dKs, dVs = orc.gao_backward(Q, split(K, sizes), split(V, sizes), Oc, dO, lsec, scale, causal, q_pos, kp,
                                     pattern_chunks=pats)
    for a, b in ((O, Oc), (lse, lsec), (dQ, dQc), (dK, np.concatenate(dKs)), (dV, np.concatenate(dVs))):
        assert np.max(np.abs(a - b)) < 1e-13


def test_block_pattern_all_ones_is_no_pattern_and_hidden_rows_get_nothing():
    r = rng(32)
    nq, nk, d = 6, 9, 4
    Q, K, V, dO = (r.normal(size=(n, d)) for n in (nq, nk, nk, nq))
    ones = orc.block_visibility(nq, nk, np.ones((2, 3)), 3)
    a, b = orc.full_forward(Q, K, V, 0.5), orc.full_forward(Q, K, V, 0.5, pattern=ones)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    flags = np.array([[0, 0, 0], [1, 0, 1]])            # rows 0-2 see nothing
    pat = orc.block_visibility(nq, nk, flags, 3)
    O, lse = orc.full_forward(Q, K, V, 0.5, pattern=pat)
    assert np.all(O[:3] == 0) and np.all(np.isneginf(lse[:3])) and np.all(np.isfinite(lse[3:]))
    dQ, dK, dV = orc.full_backward(Q, K, V, dO, 0.5, pattern=pat)
    assert np.all(dQ[:3] == 0) and np.all(dK[3:6] == 0) and np.all(dV[3:6] == 0)
    assert np.allclose(dV.sum(axis=0), dO[3:].sum(axis=0), atol=1e-13)      # visible rows of P sum to 1


def test_block_pair_gradient_matrices_brute_force_and_row_identities():
    """Alg. 2's P, dP, dS of one block pair: every entry against scalar loops with math.exp on a
    tiny causal case; with one chunk holding all keys, rows of P sum to 1 and rows of dS to 0
    (sum_c P (dP - D) = D - D), and the three products of the loop body rebuild the gradients."""
    rng = np.random.default_rng(77)
    nq, nk, d, scale = 5, 7, 3, 0.6
    Q, K, V, dO = (rng.standard_normal(s) for s in ((nq, d), (nk, d), (nk, d), (nq, d)))
    qp, kp = 2 + np.arange(nq), np.arange(nk)
    vis = orc.visibility(qp, kp, True)
    O, lse = orc.full_forward(Q, K, V, scale, True, qp, kp)
    D = orc.gao_bwd_prepare(O, dO)
    P, dP, dS = orc.gao_local_backward_matrices(Q, K, V, dO, lse, D, scale, vis)
    for r in range(nq):
        for c in range(nk):
            s = scale * sum(Q[r, t] * K[c, t] for t in range(d))
            p = math.exp(s - lse[r]) if kp[c] <= qp[r] else 0.0
            dp = sum(dO[r, t] * V[c, t] for t in range(d))
            assert abs(P[r, c] - p) < 1e-13 and abs(dP[r, c] - dp) < 1e-13
            assert abs(dS[r, c] - p * (dp - D[r])) < 1e-13
    assert np.allclose(P.sum(axis=1), 1.0, atol=1e-13) and np.allclose(dS.sum(axis=1), 0.0, atol=1e-13)
    dQ, dK, dV = orc.gao_local_backward(Q, K, V, dO, lse, D, scale, vis)
    assert np.allclose(dV, P.T @ dO) and np.allclose(dQ, scale * dS @ K) and np.allclose(dK, scale * dS.T @ Q)
    ref = orc.full_backward(Q, K, V, dO, scale, True, qp, kp)
    for got, want in zip((dQ, dK, dV), ref):
        assert np.max(np.abs(got - want)) < 1e-12
