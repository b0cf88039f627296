"""Parity at the benchmark's full sizes, in the launch configuration bench.py times.

The oracle cannot evaluate these shapes completely in reasonable time, so it computes
(i) complete heads where a head fits (forward + backward, every output element), and
(ii) sampled query rows on other heads: O, lse and dQ of a row depend only on that row of Q
and dO, so the oracle evaluates them one by one over the full key range.  dK / dV of the
largest shapes are additionally pinned by two identities that hold at any size:
sum_c dV_c = sum_r dO_r (columns of P sum to one per row) and <Q, dQ> = <K, dK>.
"""
import numpy as np
import pytest
import torch

from oracle import burst_oracle as orc
from paper_2403_09347_amd import workloads
from paper_2403_09347_amd.harness import RingWalk
from gpu_util import check, f64

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def run_workload(w, backward=True):
    inp = workloads.make_inputs(w, DEV)
    k_offs = [w.k_off(j) for j in range(w.G)]
    walk = RingWalk(inp["Q"], w.scale, w.causal, w.q_off, w.window)
    O, lse = walk.forward(inp["K"], inp["V"], k_offs)
    dQ = dKs = dVs = None
    if backward:
        # one (dK, dV) pair per chunk is kept only where it is checked; others reuse a scratch pair
        dQ, dKs, dVs = walk.backward(inp["K"], inp["V"], k_offs, inp["dO"])
    torch.cuda.synchronize()
    return inp, k_offs, walk, O, lse, dQ, dKs, dVs


def head_arrays(inp, h):
    K = np.concatenate([f64(k[0, h]) for k in inp["K"]])
    V = np.concatenate([f64(v[0, h]) for v in inp["V"]])
    return f64(inp["Q"][0, h]), K, V, f64(inp["dO"][0, h])


def check_complete_head(w, inp, h, O, lse, dQ, dKs, dVs):
    Q, K, V, dO = head_arrays(inp, h)
    qp, kp = w.q_off + np.arange(w.Nq), np.arange(K.shape[0])
    O_ref, lse_ref = orc.full_forward(Q, K, V, w.scale, w.causal, qp, kp, window=w.window)
    check(f"O[h{h}]", f64(O[0, h]), O_ref, w.dtype)
    check(f"lse[h{h}]", f64(lse[0, h]), lse_ref, w.dtype, "lse")
    dQ_ref, dK_ref, dV_ref = orc.full_backward(Q, K, V, dO, w.scale, w.causal, qp, kp, window=w.window)
    check(f"dQ[h{h}]", f64(dQ[0, h]), dQ_ref, w.dtype)
    check(f"dK[h{h}]", np.concatenate([f64(x[0, h]) for x in dKs]), dK_ref, w.dtype)
    check(f"dV[h{h}]", np.concatenate([f64(x[0, h]) for x in dVs]), dV_ref, w.dtype)


def check_sampled_rows(w, inp, h, O, lse, dQ, n_rows=64, seed=0, pattern=None):
    Q, K, V, dO = head_arrays(inp, h)
    rows = np.sort(np.random.default_rng(seed + h).choice(w.Nq, size=n_rows, replace=False))
    rows[0], rows[-1] = 0, w.Nq - 1                      # always include the first and last row
    qp, kp = w.q_off + rows, np.arange(K.shape[0])
    pat = None if pattern is None else pattern[rows]
    O_ref, lse_ref = orc.full_forward(Q[rows], K, V, w.scale, w.causal, qp, kp, window=w.window, pattern=pat)
    check(f"O[h{h},rows]", f64(O[0, h])[rows], O_ref, w.dtype)
    check(f"lse[h{h},rows]", f64(lse[0, h])[rows], lse_ref, w.dtype, "lse")
    if dQ is not None:
        dQ_ref, _, _ = orc.full_backward(Q[rows], K, V, dO[rows], w.scale, w.causal, qp, kp, window=w.window,
                                         pattern=pat)
        check(f"dQ[h{h},rows]", f64(dQ[0, h])[rows], dQ_ref, w.dtype)


def check_complete_head_by_row_slabs(w, inp, h, O, lse, dQ, dKs, dVs, slab=512, workers=4, forward_every=4):
    """A complete head where the score matrix of the whole head does not fit in host memory: the
    oracle runs on slabs of query rows against all keys.  dQ (like O and lse) of a row depends on
    that row alone; dK and dV are sums over query rows, so the slabs' dK / dV are added up.  Only
    oracle calls; slabs run on a few threads (numpy releases the interpreter lock)."""
    from concurrent.futures import ThreadPoolExecutor
    Q, K, V, dO = head_arrays(inp, h)
    kp = np.arange(K.shape[0])
    n_slabs = -(-w.Nq // slab)

    def one(i):
        rows = slice(i * slab, min(w.Nq, (i + 1) * slab))
        qp = w.q_off + np.arange(rows.start, rows.stop)
        fwd = orc.full_forward(Q[rows], K, V, w.scale, w.causal, qp, kp, window=w.window) \
            if i % forward_every == 0 or i == n_slabs - 1 else None
        return rows, fwd, orc.full_backward(Q[rows], K, V, dO[rows], w.scale, w.causal, qp, kp, window=w.window)

    dQ_ref = np.zeros_like(Q)
    dK_ref, dV_ref = np.zeros_like(K), np.zeros_like(V)
    O_got, lse_got = f64(O[0, h]), f64(lse[0, h])
    with ThreadPoolExecutor(workers) as pool:
        for rows, fwd, (dq, dk, dv) in pool.map(one, range(n_slabs)):
            dQ_ref[rows] = dq
            dK_ref += dk
            dV_ref += dv
            if fwd is not None:
                check(f"O[h{h},{rows.start}:{rows.stop}]", O_got[rows], fwd[0], w.dtype)
                check(f"lse[h{h},{rows.start}:{rows.stop}]", lse_got[rows], fwd[1], w.dtype, "lse")
    check(f"dQ[h{h}]", f64(dQ[0, h]), dQ_ref, w.dtype)
    check(f"dK[h{h}]", np.concatenate([f64(x[0, h]) for x in dKs]), dK_ref, w.dtype)
    check(f"dV[h{h}]", np.concatenate([f64(x[0, h]) for x in dVs]), dV_ref, w.dtype)


def check_identities(w, inp, h, dQ, dKs, dVs):
    Q, K, V, dO = head_arrays(inp, h)
    dV_sum = sum(f64(x[0, h]).sum(axis=0) for x in dVs)
    dO_sum = dO.sum(axis=0)
    # every query row of these workloads sees at least one key, so each row of P sums to one
    assert np.max(np.abs(dV_sum - dO_sum)) <= 2e-2 * max(1.0, np.max(np.abs(dO_sum)))
    qdq = float((Q * f64(dQ[0, h])).sum())
    kdk = float(sum((f64(k[0, h]) * f64(dk[0, h])).sum() for k, dk in zip(inp["K"], dKs)))
    scale = float(np.abs(Q * f64(dQ[0, h])).sum())
    assert abs(qdq - kdk) <= 1e-2 * scale, (qdq, kdk, scale)


def test_llama7b_32k_G8_two_complete_heads_and_sampled_rows():
    w = workloads.by_name("llama7b_32k_G8")
    inp, k_offs, walk, O, lse, dQ, dKs, dVs = run_workload(w)
    for h in (0, w.H - 1):
        check_complete_head(w, inp, h, O, lse, dQ, dKs, dVs)
    for h in (1, 7, 8, 15, 16, 30):
        check_sampled_rows(w, inp, h, O, lse, dQ)
    for h in (3, 12):
        check_identities(w, inp, h, dQ, dKs, dVs)


def test_llama7b_128k_rank31_causal_complete_head_and_sampled_rows():
    w = workloads.by_name("llama7b_128k_G32_rank31_causal")
    inp, k_offs, walk, O, lse, dQ, dKs, dVs = run_workload(w)
    check_complete_head(w, inp, w.H - 1, O, lse, dQ, dKs, dVs)
    for h in (0, 9, 17):
        check_sampled_rows(w, inp, h, O, lse, dQ)
    check_identities(w, inp, 5, dQ, dKs, dVs)


def test_llama13b_128k_G8_sampled_rows_and_identities():
    w = workloads.by_name("llama13b_128k_G8")
    inp, k_offs, walk, O, lse, dQ, dKs, dVs = run_workload(w)
    for h in (0, 21, w.H - 1):
        check_sampled_rows(w, inp, h, O, lse, dQ)
    for h in (0, w.H - 1):
        check_identities(w, inp, h, dQ, dKs, dVs)
    # one complete head at the full 16384 x 131072 size: dQ, dK, dV element by element (O and lse on
    # every fourth slab of rows), the oracle evaluated on slabs of query rows
    check_complete_head_by_row_slabs(w, inp, 23, O, lse, dQ, dKs, dVs)
    del inp, O, lse, dQ, dKs, dVs
    # and the first 256 query rows against all 128K keys, complete oracle on one head
    small = workloads.Workload("llama13b_128k_G8_nq256", 1, 2, 128, 256, w.G, w.Nc, "bf16", False, 0, 2003)
    inp, k_offs, walk, O, lse, dQ, dKs, dVs = run_workload(small)
    check_complete_head(small, inp, 1, O, lse, dQ, dKs, dVs)


def test_llama7b_1m_G32_streaming_sampled_rows_and_identities():
    w = workloads.by_name("llama7b_1m_G32")
    inp, k_offs, walk, O, lse, dQ, dKs, dVs = run_workload(w)
    for h in (0, w.H - 1):
        check_sampled_rows(w, inp, h, O, lse, dQ, n_rows=32)
    check_identities(w, inp, 0, dQ, dKs, dVs)
    del inp, O, lse, dQ, dKs, dVs
    # the same kernels on a reduced query slice: 256 query rows against all 32 chunks of 32768 keys,
    # complete oracle on both heads, all five outputs (dK and dV of every one of the 1M keys)
    small = workloads.Workload("llama7b_1m_G32_nq256", 1, 2, 128, 256, w.G, w.Nc, "bf16", False, 0, 2004)
    inp, k_offs, walk, O, lse, dQ, dKs, dVs = run_workload(small)
    for h in (0, 1):
        check_complete_head(small, inp, h, O, lse, dQ, dKs, dVs)


def test_llama13b_64k_single_device_point():
    """G = 1: one chunk of 65,536 keys, the single-device point of the paper's latency experiment;
    the walk is then plain tiled attention (Sec. 2.4, last paragraph)."""
    w = workloads.by_name("llama13b_64k_G1")
    inp, k_offs, walk, O, lse, dQ, dKs, dVs = run_workload(w)
    for h in (0, 21, 39):
        check_sampled_rows(w, inp, h, O, lse, dQ, n_rows=32)
    check_identities(w, inp, 17, dQ, dKs, dVs)


def test_llama7b_32k_last_rank_causal_sliding_window():
    """Sec. 2.6 at full shape: the 7B slice of the last rank of a 32K ring, causal, window 6000:
    five of the eight chunks lie outside every row's window and are skipped, the others are cut
    by the window's far edge and by the diagonal."""
    w = workloads.Workload("llama7b_32k_G8_rank7_causal_window6000", 1, 32, 128, 4096, 8, 4096, "bf16", True,
                           7 * 4096, 2011, window=6000)
    assert w.visible_pairs_per_head() == sum(min(6000, 7 * 4096 + r + 1) for r in range(4096))
    inp, k_offs, walk, O, lse, dQ, dKs, dVs = run_workload(w)
    check_complete_head(w, inp, w.H - 1, O, lse, dQ, dKs, dVs)
    for h in (0, 13):
        check_sampled_rows(w, inp, h, O, lse, dQ)
    check_identities(w, inp, 6, dQ, dKs, dVs)
    for j in range(5):                                     # chunks 0..4 are out of every window
        assert float(dKs[j].abs().max()) == 0.0 and float(dVs[j].abs().max()) == 0.0


def test_llama7b_32k_G8_with_scores_stored_in_hbm():
    """The chunk step without the Sec. 2.4 tiling (S_ij, P_ij in HBM: 3 GiB of workspace for this
    shape) at the benchmark's full size: sampled rows of several heads against the oracle."""
    from paper_2403_09347_amd.harness import MaterializedWalk
    w = workloads.by_name("llama7b_32k_G8")
    inp = workloads.make_inputs(w, DEV)
    k_offs = [w.k_off(j) for j in range(w.G)]
    walk = MaterializedWalk(inp["Q"], w.scale, w.causal, w.q_off, w.window, max_chunk_rows=w.Nc)
    assert walk.workspace.numel() >= w.B * w.H * w.Nq * w.Nc * 6
    O, lse = walk.forward(inp["K"], inp["V"], k_offs)
    torch.cuda.synchronize()
    for h in (0, 13, w.H - 1):
        check_sampled_rows(w, inp, h, O, lse, None)


@pytest.mark.parametrize("block", [128, 64])
def test_llama7b_32k_G8_block_sparse_band_plus_global(block):
    """Block flags (Sec. 2.6) at the benchmark's full size: a band of blocks around the diagonal of
    rank 3's slice plus global first blocks, one flag matrix per chunk.  Lists of visible tiles are
    longer than one round of the list builder for every kernel.  One complete head (all five
    outputs) and sampled rows of others against the oracle.  With 64-wide blocks the forward and
    dQ calls go to the 128-row kernels and the dK/dV call to the kernel with 64-key workgroups."""
    w = workloads.by_name("llama7b_32k_G8")
    inp = workloads.make_inputs(w, DEV)
    k_offs = [w.k_off(j) for j in range(w.G)]
    q_off = 3 * w.Nq
    nrb, ncb = w.Nq // block, w.Nc // block
    flags = [workloads.block_flags(nrb, ncb, "band_global", seed=7 + j, diag_shift=(q_off - k_offs[j]) // block)
             for j in range(w.G)]
    flags[5] |= workloads.block_flags(nrb, ncb, "random", density=0.2, seed=99)     # one chunk with scattered blocks
    flags[6][0, 1:] = 0                                                             # only the global column block left
    flags[7][:] = 0                                                                 # a chunk nobody sees
    masks = [torch.from_numpy(f).to(DEV).contiguous() for f in flags]
    walk = RingWalk(inp["Q"], w.scale, False, q_off, 0, block)
    O, lse = walk.forward(inp["K"], inp["V"], k_offs, masks=masks)
    dQ, dKs, dVs = walk.backward(inp["K"], inp["V"], k_offs, inp["dO"], masks=masks)
    torch.cuda.synchronize()
    pattern = np.concatenate([orc.block_visibility(w.Nq, w.Nc, f, block) for f in flags], axis=1)
    h = 11
    Q, K, V, dO = head_arrays(inp, h)
    qp, kp = q_off + np.arange(w.Nq), np.arange(K.shape[0])
    O_ref, lse_ref = orc.full_forward(Q, K, V, w.scale, False, qp, kp, pattern=pattern)
    dQ_ref, dK_ref, dV_ref = orc.full_backward(Q, K, V, dO, w.scale, False, qp, kp, pattern=pattern)
    check("O", f64(O[0, h]), O_ref, w.dtype)
    check("lse", f64(lse[0, h]), lse_ref, w.dtype, "lse")
    check("dQ", f64(dQ[0, h]), dQ_ref, w.dtype)
    check("dK", np.concatenate([f64(x[0, h]) for x in dKs]), dK_ref, w.dtype)
    check("dV", np.concatenate([f64(x[0, h]) for x in dVs]), dV_ref, w.dtype)
    for h in (0, 31):
        check_sampled_rows(w, inp, h, O, lse, dQ, pattern=pattern)
    # key blocks no row block sees get exactly zero gradients
    for j in (6, 7):
        hidden = np.repeat(flags[j].sum(axis=0) == 0, block)
        assert hidden.any()
        assert torch.count_nonzero(dKs[j][0, :, torch.from_numpy(hidden).to(DEV)]) == 0
        assert torch.count_nonzero(dVs[j][0, :, torch.from_numpy(hidden).to(DEV)]) == 0


def test_d64_heads_at_the_benchmark_sequence_shape():
    """The d = 64 kernels at 32 heads, 4096 rows against 4 chunks of 4096 keys, causal at the last rank:
    sampled rows of several heads, identities on another."""
    w = workloads.Workload("d64_16k_G4_rank3_causal", 1, 32, 64, 4096, 4, 4096, "bf16", True, 3 * 4096, 1006)
    inp, k_offs, walk, O, lse, dQ, dKs, dVs = run_workload(w)
    for h in (0, 14, 31):
        check_sampled_rows(w, inp, h, O, lse, dQ)
    check_identities(w, inp, 7, dQ, dKs, dVs)


def test_llama7b_32k_G8_sequence_major_tensors_match_the_contiguous_run_bitwise():
    """The benchmark workload with Q, K, V, dO as views of [B, rows, H, d] tensors (the layout a
    projection leaves them in): same kernels, same arithmetic, other addresses: every output equals
    that of the contiguous run (which the tests above hold against the oracle) bit for bit."""
    w = workloads.WORKLOADS[1]
    inp, k_offs, _, O, lse, dQ, dKs, dVs = run_workload(w)
    seq = {"Q": workloads.relayout(inp["Q"], "seq"), "dO": workloads.relayout(inp["dO"], "seq"),
           "K": [workloads.relayout(k, "seq") for k in inp["K"]], "V": [workloads.relayout(v, "seq") for v in inp["V"]]}
    assert seq["Q"].stride() == (w.Nq * w.H * w.d, w.d, w.H * w.d, 1)
    walk = RingWalk(seq["Q"], w.scale, w.causal, w.q_off, w.window)
    O2, lse2 = walk.forward(seq["K"], seq["V"], k_offs)
    dQ2, dKs2, dVs2 = walk.backward(seq["K"], seq["V"], k_offs, seq["dO"])
    torch.cuda.synchronize()
    assert O2.stride() == seq["Q"].stride()
    assert torch.equal(O, O2) and torch.equal(lse, lse2) and torch.equal(dQ, dQ2)
    assert all(torch.equal(a, b) for a, b in zip(dKs + dVs, dKs2 + dVs2))


def test_llama13b_32k_G8_share_runs_on_the_128_row_kernels():
    """40 heads x 4096 rows give the 256-row forward / dQ kernels 640 workgroups, a last round half
    empty: the call is served by the 128-row kernels (automatic choice).  One complete head, sampled
    rows elsewhere, the size-independent identities."""
    from paper_2403_09347_amd import binding
    w = workloads.by_name("llama13b_32k_G8")
    assert binding.burst_kernel_family_for(binding.params(w.B, w.H, w.Nq, w.Nc, w.d, "bf16", w.scale)) == 2
    inp, k_offs, walk, O, lse, dQ, dKs, dVs = run_workload(w)
    check_complete_head(w, inp, 39, O, lse, dQ, dKs, dVs)
    for h in (0, 20):
        check_sampled_rows(w, inp, h, O, lse, dQ)
    check_identities(w, inp, 7, dQ, dKs, dVs)


MAX_MFMA_ROWS = 4 * 1024 * 1024        # slices or chunks up to this many rows are served by the MFMA kernels


@pytest.mark.parametrize("long_side", ["queries", "keys", "queries_at_the_limit"])
def test_slices_and_chunks_around_the_largest_size_the_tiled_kernels_take(long_side):
    """More than 4 Mi rows on either side of a block pair (the tiled kernels address a head through
    32-bit byte offsets and hand such calls to the generic kernels), and exactly 4 Mi query rows
    (the largest slice the tiled kernels take: 16384 workgroups per head), against few rows on the
    other side so that the oracle can evaluate the whole pair: all five outputs, every element."""
    from gpu_util import compare_all_heads
    from paper_2403_09347_amd import binding
    if long_side == "queries":
        spec = dict(B=1, H=1, d=128, Nq=MAX_MFMA_ROWS + 70, chunk_rows=[40], causal=False)
    elif long_side == "keys":
        spec = dict(B=1, H=1, d=128, Nq=40, chunk_rows=[MAX_MFMA_ROWS + 70], causal=True, q_off=MAX_MFMA_ROWS - 500)
    else:
        spec = dict(B=1, H=1, d=128, Nq=MAX_MFMA_ROWS, chunk_rows=[64], causal=False)
    case = workloads.make_case(dtype="bf16", seed=2100, device=DEV, **spec)
    p = binding.params(1, 1, spec["Nq"], spec["chunk_rows"][0], 128, "bf16", case["scale"])
    assert binding.burst_kernel_family_for(p) == (1 if long_side == "queries_at_the_limit" else 0)
    walk = RingWalk(case["Q"], case["scale"], case["causal"], case["q_off"])
    O, lse = walk.forward(case["K"], case["V"], case["k_offs"])
    dQ, dKs, dVs = walk.backward(case["K"], case["V"], case["k_offs"], case["dO"])
    torch.cuda.synchronize()
    # dK, dV of the long-query cases sum 4 Mi rows into 40 / 64 keys and reach the hundreds: they are
    # held to 1e-2 of the largest reference entry, not to the absolute 2e-2 (see gpu_util.check)
    compare_all_heads(case, "bf16", O, lse, dQ, dKs, dVs, dkv_kind="abs" if long_side == "keys" else "rel")


@pytest.mark.parametrize("tiles", [2048, 2049])
def test_narrow_block_flags_around_the_longest_tile_list_of_the_64_key_workgroups(tiles):
    """64-wide block flags (Sec. 2.6): the dK/dV half runs with 64-key workgroups whose tile lists
    hold 2048 query tiles of 64 rows; one tile more and the call goes to the 128-key workgroups.
    Few keys, so that the oracle evaluates the whole pair: all five outputs, every element."""
    from gpu_util import compare_all_heads
    spec = dict(B=1, H=2, d=128, Nq=64 * tiles, chunk_rows=[322, 200], block=64, pattern="random", density=0.7)
    case = workloads.make_case(dtype="bf16", seed=2200 + tiles, device=DEV, **spec)
    walk = RingWalk(case["Q"], case["scale"], case["causal"], case["q_off"], 0, 64)
    O, lse = walk.forward(case["K"], case["V"], case["k_offs"], masks=case["masks"])
    dQ, dKs, dVs = walk.backward(case["K"], case["V"], case["k_offs"], case["dO"], masks=case["masks"])
    torch.cuda.synchronize()
    compare_all_heads(case, "bf16", O, lse, dQ, dKs, dVs, dkv_kind="rel")
