"""GPU parity: the HIP path (through the C ABI) against the fp64 oracle, element by element."""
import numpy as np
import pytest
import torch

from oracle import burst_oracle as orc
from paper_2403_09347_amd import binding as B
from paper_2403_09347_amd import workloads
from paper_2403_09347_amd.harness import DoubleBufferedWalk, KeyPinnedBackward, RingWalk, SpanWalk
from gpu_util import check, compare_all_heads, f64, head_inputs

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(autouse=True, params=[1, 2], ids=["hand-scheduled", "plain"])
def kernel_family(request):
    """Every test of this file runs once with each of the two kernel families for dense bf16,
    d = 128 calls (the automatic choice would give these small shapes to one of them only)."""
    B.burst_set_kernel_family(request.param)
    yield request.param
    B.burst_set_kernel_family(0)


def run_case(case, dtype, backward=True, use_D=True, order=None):
    walk = RingWalk(case["Q"], case["scale"], case["causal"], case["q_off"], case.get("window", 0),
                    case.get("block", 0), case.get("kv_heads", 0))
    masks = case.get("masks")
    O, lse = walk.forward(case["K"], case["V"], case["k_offs"], order=order, masks=masks)
    res = (O, lse, None, None, None)
    if backward:
        dQ, dKs, dVs = walk.backward(case["K"], case["V"], case["k_offs"], case["dO"], use_D=use_D, masks=masks)
        res = (O, lse, dQ, dKs, dVs)
    torch.cuda.synchronize()
    return walk, res


# MFMA path: sizes span several 256-row workgroups, 64-key tiles and ragged tails on both sides.
BF16_CASES = [
    dict(B=1, H=2, d=128, Nq=64, chunk_rows=[64]),
    dict(B=1, H=3, d=128, Nq=300, chunk_rows=[200, 64, 331]),
    dict(B=2, H=2, d=128, Nq=517, chunk_rows=[256, 1, 390]),
    dict(B=1, H=9, d=128, Nq=256, chunk_rows=[512]),                       # more heads than XCDs
    dict(B=1, H=2, d=128, Nq=300, chunk_rows=[256, 192], causal=True, q_off=148),
    dict(B=1, H=2, d=128, Nq=384, chunk_rows=[128, 128, 128], causal=True, q_off=0),   # self-attention diagonal
    dict(B=1, H=1, d=128, Nq=200, chunk_rows=[300, 300], causal=True, q_off=250),       # second chunk partly masked
    dict(B=1, H=2, d=128, Nq=130, chunk_rows=[100, 260], causal=True, q_off=50,
         k_offs=[0, 400]),                                                 # second chunk fully masked
    dict(B=1, H=1, d=128, Nq=100, chunk_rows=[64, 64], causal=True, q_off=-30),         # rows that see nothing
    # sliding window (Sec. 2.6): band narrower than a tile, wider than a workgroup, chunks fully outside it
    dict(B=1, H=2, d=128, Nq=600, chunk_rows=[256, 200, 344], causal=True, q_off=200, window=40),
    dict(B=1, H=2, d=128, Nq=700, chunk_rows=[512, 512], causal=True, q_off=324, window=300),
    dict(B=1, H=1, d=128, Nq=520, chunk_rows=[300, 300, 300], causal=False, q_off=100, window=130),
    dict(B=1, H=1, d=128, Nq=300, chunk_rows=[128, 128, 128, 128], causal=True, q_off=2000, window=64,
         k_offs=[0, 1800, 1928, 2200]),                                    # first chunk out of every window
    dict(B=2, H=1, d=128, Nq=130, chunk_rows=[257], causal=True, q_off=60, window=1),   # each row sees one key
    dict(B=1, H=3, d=128, Nq=596, chunk_rows=[356], causal=True, q_off=107, window=1),  # P must be exactly 1: dV = dO
]


@pytest.mark.parametrize("spec", BF16_CASES, ids=lambda s: "-".join(f"{k}{v}" for k, v in s.items() if k != "d"))
def test_bf16_mfma_forward_backward(spec):
    case = workloads.make_case(dtype="bf16", seed=17, device=DEV, **spec)
    _, (O, lse, dQ, dKs, dVs) = run_case(case, "bf16")
    compare_all_heads(case, "bf16", O, lse, dQ, dKs, dVs)


# Block-sparse patterns (Sec. 2.6): one flag matrix per chunk, blocks of 64 .. 256 rows/keys; random flags
# (rows and whole chunks that see nothing included), a band around the diagonal, band + global blocks.
SPARSE_CASES = [
    dict(B=1, H=2, d=128, Nq=300, chunk_rows=[200, 64, 331], block=64, pattern="random"),
    dict(B=2, H=2, d=128, Nq=517, chunk_rows=[256, 1, 390], block=128, pattern="random", density=0.5),
    dict(B=1, H=3, d=128, Nq=700, chunk_rows=[512, 300], block=256, pattern="random", density=0.3),
    dict(B=1, H=2, d=128, Nq=640, chunk_rows=[640, 640], block=64, pattern="band", causal=True, q_off=640),
    dict(B=1, H=2, d=128, Nq=600, chunk_rows=[384, 421], block=128, pattern="band_global", causal=True, q_off=300),
    dict(B=1, H=1, d=128, Nq=520, chunk_rows=[300, 300, 300], block=64, pattern="random", density=0.6,
         causal=True, q_off=380, window=200),
    dict(B=1, H=2, d=128, Nq=200, chunk_rows=[256, 256], block=64, pattern="random", density=0.0),   # nothing visible
    # one flag matrix per (batch, head)
    dict(B=2, H=3, d=128, Nq=517, chunk_rows=[256, 390], block=64, pattern="random", density=0.5, per_head_flags=True),
    dict(B=1, H=4, d=128, Nq=512, chunk_rows=[300, 300], block=128, pattern="random", density=0.4, per_head_flags=True,
         kv_heads=2, causal=True, q_off=200),
    dict(B=1, H=4, d=64, Nq=300, chunk_rows=[200, 331], block=64, pattern="random", density=0.5, per_head_flags=True),
    dict(B=2, H=4, d=64, Nq=256, chunk_rows=[256, 130], block=64, pattern="random", density=0.4, per_head_flags=True,
         kv_heads=1, causal=True, q_off=130),
]


@pytest.mark.parametrize("spec", SPARSE_CASES, ids=lambda s: "-".join(f"{k}{v}" for k, v in s.items() if k != "d"))
def test_bf16_block_sparse_forward_backward(spec):
    case = workloads.make_case(dtype="bf16", seed=29, device=DEV, **spec)
    _, (O, lse, dQ, dKs, dVs) = run_case(case, "bf16")
    compare_all_heads(case, "bf16", O, lse, dQ, dKs, dVs)


@pytest.mark.parametrize("spec", [s for s in SPARSE_CASES if s["d"] == 128 and s["block"] == 64] + [
    # grouped heads: the lists of the 64-key workgroups run over the tiles of all heads of a group
    dict(B=1, H=4, kv_heads=2, d=128, Nq=256, chunk_rows=[256, 192], block=64, pattern="random", density=0.5),
    dict(B=2, H=6, kv_heads=2, d=128, Nq=448, chunk_rows=[300, 77], block=64, pattern="random", density=0.4,
         per_head_flags=True, causal=True, q_off=100, layout="seq"),
],
                         ids=lambda s: "-".join(f"{k}{v}" for k, v in s.items() if k != "d"))
def test_narrow_block_flags_with_the_kernels_chosen_per_call(spec, kernel_family):
    """Left to the per-call choice, 64-wide flags send the dK/dV half to the hand-scheduled kernel's
    shape with 64-key workgroups (the forced families above never take it)."""
    if kernel_family != 1:
        pytest.skip("one run is enough: the test sets the family itself")
    B.burst_set_kernel_family(0)
    case = workloads.make_case(dtype="bf16", seed=31, device=DEV, **spec)
    _, (O, lse, dQ, dKs, dVs) = run_case(case, "bf16")
    compare_all_heads(case, "bf16", O, lse, dQ, dKs, dVs)


def test_narrow_block_flags_accumulate_into_dk_dv(kernel_family):
    """accumulate_dkv = 1 in the 64-key shape of the dK/dV kernel: a second call on the same block
    pair doubles the first call's result exactly (fp32: x + x)."""
    if kernel_family != 1:
        pytest.skip("one run is enough: the test sets the family itself")
    B.burst_set_kernel_family(0)
    spec = dict(B=1, H=4, kv_heads=2, d=128, Nq=320, chunk_rows=[200], block=64, pattern="random", density=0.6)
    case = workloads.make_case(dtype="bf16", seed=33, device=DEV, **spec)
    walk, (O, lse, dQ, dKs, dVs) = run_case(case, "bf16")
    p = walk.params(200, case["k_offs"][0], case["masks"][0], case["K"][0])
    dK2, dV2 = dKs[0].clone(), dVs[0].clone()
    B.burst_local_bwd_dkv(case["Q"], case["K"][0], case["V"][0], case["dO"], walk.lse, walk.D, dK2, dV2, p, True)
    torch.cuda.synchronize()
    assert torch.equal(dK2, 2 * dKs[0]) and torch.equal(dV2, 2 * dVs[0])


@pytest.mark.parametrize("dtype,spec", [
    ("f32", dict(B=1, H=2, d=32, Nq=150, chunk_rows=[100, 90], block=64, pattern="random", density=0.5)),
    ("f32", dict(B=2, H=4, d=32, Nq=150, chunk_rows=[100, 90], block=64, pattern="random", density=0.5,
                 per_head_flags=True, kv_heads=2)),
    ("bf16", dict(B=1, H=2, d=64, Nq=130, chunk_rows=[200], block=64, pattern="band_global", causal=True, q_off=70)),
])
def test_generic_kernels_block_sparse(dtype, spec):
    case = workloads.make_case(dtype=dtype, seed=37, device=DEV, **spec)
    _, (O, lse, dQ, dKs, dVs) = run_case(case, dtype)
    compare_all_heads(case, dtype, O, lse, dQ, dKs, dVs)


# Tensors that are not contiguous [B, H, rows, d]: sequence-major and packed-projection views.
STRIDED_CASES = [
    ("bf16", dict(B=2, H=3, d=128, Nq=517, chunk_rows=[256, 1, 390], layout="seq")),
    ("bf16", dict(B=1, H=2, d=128, Nq=300, chunk_rows=[256, 192], causal=True, q_off=148, layout="packed")),
    ("bf16", dict(B=1, H=2, d=128, Nq=520, chunk_rows=[300, 300, 300], causal=True, q_off=380, window=200, layout="seq")),
    ("bf16", dict(B=2, H=4, d=128, Nq=512, chunk_rows=[300, 300], block=128, pattern="random", density=0.4,
                  per_head_flags=True, kv_heads=2, causal=True, q_off=200, layout="seq")),
    ("bf16", dict(B=1, H=6, d=128, Nq=256, chunk_rows=[200, 130], kv_heads=2, layout="packed")),
    ("bf16", dict(B=1, H=6, d=128, Nq=250, chunk_rows=[200, 130], kv_heads=3, layout="seq")),   # dK/dV: generic kernel
    ("bf16", dict(B=2, H=3, d=64, Nq=300, chunk_rows=[200, 64, 331], causal=True, q_off=250, layout="seq")),
    ("bf16", dict(B=1, H=4, d=64, Nq=256, chunk_rows=[256, 130], block=64, pattern="random", density=0.5,
                  kv_heads=2, layout="packed")),
    ("f32", dict(B=2, H=2, d=32, Nq=150, chunk_rows=[100, 90], causal=True, q_off=60, layout="seq")),
    ("f32", dict(B=1, H=4, d=128, Nq=70, chunk_rows=[50, 41], kv_heads=2, layout="packed")),
    ("bf16", dict(B=1, H=2, d=32, Nq=100, chunk_rows=[77], layout="seq")),                      # generic bf16
]


@pytest.mark.parametrize("dtype,spec", STRIDED_CASES,
                         ids=lambda v: v if isinstance(v, str) else "-".join(f"{k}{x}" for k, x in v.items()))
def test_strided_tensors(dtype, spec):
    case = workloads.make_case(dtype=dtype, seed=43, device=DEV, **spec)
    assert not case["Q"].is_contiguous() and not case["K"][0].is_contiguous()
    walk, (O, lse, dQ, dKs, dVs) = run_case(case, dtype)
    assert O.stride() == case["Q"].stride()                    # O is written where Q's layout says
    compare_all_heads(case, dtype, O, lse, dQ, dKs, dVs)
    # the same values in contiguous tensors give bitwise the same results
    same = workloads.make_case(dtype=dtype, seed=43, device=DEV, **{**spec, "layout": "head"})
    _, (O2, lse2, dQ2, dKs2, dVs2) = run_case(same, dtype)
    assert torch.equal(O, O2) and torch.equal(lse, lse2) and torch.equal(dQ, dQ2)
    assert all(torch.equal(a, b) for a, b in zip(dKs + dVs, dKs2 + dVs2))


def test_rows_too_far_apart_for_the_mfma_kernels_take_the_generic_ones():
    """The MFMA kernels reach a head's rows through 32-bit byte offsets; a call whose rows lie 4 MiB
    apart (64 rows + the prefetch margin > 4 GiB) must still be answered, by the generic kernels."""
    case = workloads.make_case(B=1, H=1, d=128, Nq=64, chunk_rows=[96], dtype="bf16", seed=47, device=DEV, causal=True,
                               q_off=40)
    pitch = 1 << 21                                                   # elements between rows
    def spread(x):
        big = torch.zeros((x.shape[2] - 1) * pitch + 128, dtype=x.dtype, device=DEV)
        view = big.as_strided(x.shape, (0, 0, pitch, 1))
        view.copy_(x)
        return view
    far = dict(case, Q=spread(case["Q"]), dO=spread(case["dO"]))
    p = B.params(1, 1, 64, 96, 128, "bf16", case["scale"], q_strides=B.strides_of(far["Q"]))
    assert tuple(p.q_strides) == (128, 128, pitch)
    _, (O, lse, dQ, dKs, dVs) = run_case(far, "bf16")
    compare_all_heads(case, "bf16", O, lse, dQ, dKs, dVs)


def test_unaligned_strides_are_rejected_on_the_device_path():
    case = workloads.make_case(B=1, H=2, d=128, Nq=64, chunk_rows=[64], dtype="bf16", seed=53, device=DEV)
    walk = RingWalk(case["Q"], case["scale"])
    walk.init()
    p = B.params(1, 2, 64, 64, 128, "bf16", case["scale"], kv_strides=(64 * 2 * 128, 64 * 128, 132))
    with pytest.raises(ValueError):                                   # the binding compares tensor and block
        B.burst_local_fwd(case["Q"], case["K"][0], case["V"][0], walk.O_acc, walk.m, walk.l, p)
    odd = torch.zeros((1, 2, 64, 132), dtype=torch.bfloat16, device=DEV)[..., :128]
    p = B.params(1, 2, 64, 64, 128, "bf16", case["scale"], kv_strides=B.strides_of(odd))
    with pytest.raises(B.BurstError):                                 # the library checks the block
        B.burst_local_fwd(case["Q"], odd, odd, walk.O_acc, walk.m, walk.l, p)


# bf16, d = 64: MFMA kernels of their own (32 rows or keys per wavefront, 64- and 32-key tiles).
D64_CASES = [
    dict(B=1, H=2, d=64, Nq=32, chunk_rows=[32]),
    dict(B=1, H=3, d=64, Nq=300, chunk_rows=[200, 64, 331]),
    dict(B=2, H=2, d=64, Nq=517, chunk_rows=[256, 1, 390]),
    dict(B=1, H=9, d=64, Nq=128, chunk_rows=[512]),
    dict(B=1, H=2, d=64, Nq=300, chunk_rows=[256, 192], causal=True, q_off=148),
    dict(B=1, H=2, d=64, Nq=384, chunk_rows=[128, 128, 128], causal=True, q_off=0),
    dict(B=1, H=1, d=64, Nq=100, chunk_rows=[64, 64], causal=True, q_off=-30),          # rows that see nothing
    dict(B=1, H=2, d=64, Nq=600, chunk_rows=[256, 200, 344], causal=True, q_off=200, window=40),
    dict(B=1, H=1, d=64, Nq=520, chunk_rows=[300, 300, 300], causal=False, q_off=100, window=130),
    dict(B=1, H=1, d=64, Nq=300, chunk_rows=[128, 128, 128, 128], causal=True, q_off=2000, window=64,
         k_offs=[0, 1800, 1928, 2200]),
    dict(B=1, H=3, d=64, Nq=596, chunk_rows=[356], causal=True, q_off=107, window=1),
    dict(B=1, H=6, kv_heads=2, d=64, Nq=300, chunk_rows=[260, 90], causal=True, q_off=100),   # grouped heads
    dict(B=1, H=4, d=64, Nq=2048, chunk_rows=[2048]),                                   # many tiles, several workgroups
    # block flags: lists of visible tiles
    dict(B=1, H=2, d=64, Nq=300, chunk_rows=[200, 64, 331], block=64, pattern="random"),
    dict(B=1, H=2, d=64, Nq=700, chunk_rows=[512, 300], block=128, pattern="random", density=0.3),
    dict(B=1, H=2, d=64, Nq=640, chunk_rows=[640, 640], block=64, pattern="band", causal=True, q_off=640),
    dict(B=1, H=1, d=64, Nq=520, chunk_rows=[300, 300, 300], block=64, pattern="random", density=0.6,
         causal=True, q_off=380, window=200),
    dict(B=1, H=4, kv_heads=2, d=64, Nq=256, chunk_rows=[256, 192], block=64, pattern="random", density=0.5),
    dict(B=1, H=2, d=64, Nq=200, chunk_rows=[256], block=64, pattern="random", density=0.0),       # nothing visible
]


@pytest.mark.parametrize("spec", D64_CASES, ids=lambda s: "-".join(f"{k}{v}" for k, v in s.items()))
def test_bf16_d64_forward_backward(spec):
    case = workloads.make_case(dtype="bf16", seed=19, device=DEV, **spec)
    _, (O, lse, dQ, dKs, dVs) = run_case(case, "bf16")
    compare_all_heads(case, "bf16", O, lse, dQ, dKs, dVs)


# Grouped-query attention (not in the paper): K, V, dK, dV with fewer heads than Q; dK, dV sum over the group.
GQA_CASES = [
    ("bf16", dict(B=1, H=4, kv_heads=2, d=128, Nq=256, chunk_rows=[200, 130])),               # dK/dV MFMA kernel: Nq % 64 == 0
    ("bf16", dict(B=2, H=8, kv_heads=2, d=128, Nq=320, chunk_rows=[256, 100], causal=True, q_off=120)),
    ("bf16", dict(B=1, H=6, kv_heads=1, d=128, Nq=384, chunk_rows=[300], causal=True, q_off=100, window=150)),
    ("bf16", dict(B=1, H=4, kv_heads=2, d=128, Nq=300, chunk_rows=[260])),                    # ragged Nq: generic dK/dV kernel
    ("bf16", dict(B=1, H=4, kv_heads=2, d=128, Nq=256, chunk_rows=[256, 192], block=64, pattern="random", density=0.5)),
    ("f32", dict(B=1, H=4, kv_heads=2, d=32, Nq=90, chunk_rows=[70, 40], causal=True, q_off=30)),
    # eight query heads per key/value head, several workgroups per head, a list of 256 query tiles per key block
    ("bf16", dict(B=1, H=16, kv_heads=2, d=128, Nq=2048, chunk_rows=[1024, 1024], causal=True, q_off=1024)),
]


@pytest.mark.parametrize("dtype,spec", GQA_CASES, ids=lambda v: v if isinstance(v, str) else "-".join(f"{k}{x}" for k, x in v.items()))
def test_grouped_query_heads(dtype, spec):
    case = workloads.make_case(dtype=dtype, seed=53, device=DEV, **spec)
    _, (O, lse, dQ, dKs, dVs) = run_case(case, dtype)
    assert dKs[0].shape[1] == spec["kv_heads"]
    compare_all_heads(case, dtype, O, lse, dQ, dKs, dVs)


def test_config0_tiny_fp32_complete():
    w = workloads.WORKLOADS[0]
    inp = workloads.make_inputs(w, DEV)
    case = dict(inp, k_offs=[w.k_off(j) for j in range(w.G)], q_off=w.q_off, causal=w.causal, scale=w.scale)
    _, (O, lse, dQ, dKs, dVs) = run_case(case, "f32")
    compare_all_heads(case, "f32", O, lse, dQ, dKs, dVs)


GENERIC_CASES = [
    ("f32", dict(B=1, H=2, d=40, Nq=70, chunk_rows=[33, 50], causal=True, q_off=20)),
    ("f32", dict(B=2, H=1, d=128, Nq=65, chunk_rows=[129])),
    ("f32", dict(B=1, H=1, d=7, Nq=5, chunk_rows=[3, 1])),
    ("bf16", dict(B=1, H=2, d=64, Nq=100, chunk_rows=[70, 90], causal=True, q_off=60)),
    ("bf16", dict(B=1, H=1, d=96, Nq=33, chunk_rows=[64])),
    ("f32", dict(B=1, H=2, d=64, Nq=90, chunk_rows=[50, 70], causal=True, q_off=30, window=17)),
    ("bf16", dict(B=1, H=1, d=64, Nq=80, chunk_rows=[100], causal=False, q_off=10, window=25)),
]


@pytest.mark.parametrize("dtype,spec", GENERIC_CASES)
def test_generic_kernels(dtype, spec):
    case = workloads.make_case(dtype=dtype, seed=23, device=DEV, **spec)
    _, (O, lse, dQ, dKs, dVs) = run_case(case, dtype)
    compare_all_heads(case, dtype, O, lse, dQ, dKs, dVs)


def test_g1_is_plain_attention():
    """One device: no global merge is needed and the path is plain tiled attention (Sec. 2.4)."""
    case = workloads.make_case(B=1, H=2, d=128, Nq=320, chunk_rows=[448], dtype="bf16", seed=5, device=DEV)
    _, (O, lse, dQ, dKs, dVs) = run_case(case, "bf16")
    compare_all_heads(case, "bf16", O, lse, dQ, dKs, dVs)


# ------------------------------------------------------------------ the HBM-bound steps
@pytest.mark.parametrize("d,dtype", [(128, "bf16"), (128, "f32"), (64, "f32"), (20, "f32"), (7, "bf16")])
def test_state_init_finalize_merge_prepare(d, dtype):
    g = torch.Generator(device=DEV).manual_seed(3)
    Bt, H, Nq = 2, 3, 77
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    p = B.params(Bt, H, Nq, 0, d, tdt, 0.5)
    O_acc = torch.full((Bt, H, Nq, d), 7.0, device=DEV)
    m = torch.full((Bt, H, Nq), 3.0, device=DEV)
    l = torch.full((Bt, H, Nq), 3.0, device=DEV)
    B.burst_state_init(O_acc, m, l, p)
    assert torch.all(O_acc == 0) and torch.all(l == 0) and torch.all(torch.isneginf(m))

    def rand_state():
        mm = torch.randn((Bt, H, Nq), generator=g, device=DEV) * 5
        ll = torch.rand((Bt, H, Nq), generator=g, device=DEV) * 10 + 1.0
        O = torch.randn((Bt, H, Nq, d), generator=g, device=DEV) * ll[..., None]   # O_acc / l ~ N(0,1)
        dead = torch.rand((Bt, H, Nq), generator=g, device=DEV) < 0.2       # rows that saw nothing
        O[dead] = 0
        mm[dead] = float("-inf")
        ll[dead] = 0
        return O, mm, ll

    Oa, ma, la = rand_state()
    Ob, mb, lb = rand_state()
    # finalize
    O_out = torch.empty((Bt, H, Nq, d), device=DEV, dtype=tdt)
    lse = torch.empty((Bt, H, Nq), device=DEV)
    B.burst_finalize(Oa, ma, la, O_out, lse, p)
    for b in range(Bt):
        for h in range(H):
            O_ref, lse_ref = orc.gao_finalize(f64(Oa[b, h]), f64(ma[b, h]), f64(la[b, h]))
            check("finalize O", f64(O_out[b, h]), O_ref, dtype)
            check("finalize lse", f64(lse[b, h]), lse_ref, dtype, "lse")
    # merge (in place on a); compared through the observable quantities
    refs = [[orc.gao_merge(f64(Oa[b, h]), f64(ma[b, h]), f64(la[b, h]), f64(Ob[b, h]), f64(mb[b, h]), f64(lb[b, h]))
             for h in range(H)] for b in range(Bt)]
    B.burst_merge_state(Oa, ma, la, Ob, mb, lb, p)
    for b in range(Bt):
        for h in range(H):
            O_ref, m_ref, l_ref = refs[b][h]
            check("merge m", f64(ma[b, h]), m_ref, "f32", "lse")
            check("merge l", f64(la[b, h]), l_ref, "f32")
            check("merge O", f64(Oa[b, h]), O_ref, "f32")
    # D = rowsum(dO o O)
    Ot = torch.randn((Bt, H, Nq, d), generator=g, device=DEV).to(tdt)
    dOt = torch.randn((Bt, H, Nq, d), generator=g, device=DEV).to(tdt)
    D = torch.empty((Bt, H, Nq), device=DEV)
    B.burst_bwd_prepare(Ot, dOt, D, p)
    for b in range(Bt):
        for h in range(H):
            check("D", f64(D[b, h]), orc.gao_bwd_prepare(f64(Ot[b, h]), f64(dOt[b, h])), "f32")


# ------------------------------------------------------------------ properties of the state machine
def test_empty_and_fully_masked_chunks_leave_the_state_bit_for_bit():
    case = workloads.make_case(B=1, H=2, d=128, Nq=200, chunk_rows=[192, 100], dtype="bf16", seed=9, device=DEV,
                               causal=True, q_off=100)
    walk = RingWalk(case["Q"], case["scale"], True, case["q_off"])
    walk.init()
    walk.step(case["K"][0], case["V"][0], 0)
    snap = [t.clone() for t in (walk.O_acc, walk.m, walk.l)]
    empty = torch.empty((1, 2, 0, 128), device=DEV, dtype=torch.bfloat16)
    walk.step(empty, empty, 50)                                  # Nc = 0
    walk.step(case["K"][1], case["V"][1], 10_000)                # every key lies after every query
    torch.cuda.synchronize()
    for a, b in zip(snap, (walk.O_acc, walk.m, walk.l)):
        assert torch.equal(a, b)
    # and into a fresh state: it stays fresh
    walk.init()
    walk.step(case["K"][1], case["V"][1], 10_000)
    torch.cuda.synchronize()
    assert torch.all(walk.O_acc == 0) and torch.all(walk.l == 0) and torch.all(torch.isneginf(walk.m))
    O, lse = walk.finalize()
    torch.cuda.synchronize()
    assert torch.all(O == 0) and torch.all(torch.isneginf(lse))


def test_chunk_order_and_split_merge():
    case = workloads.make_case(B=1, H=2, d=128, Nq=300, chunk_rows=[128, 200, 64, 150], dtype="bf16", seed=31, device=DEV)
    w0, (O0, lse0, *_r) = run_case(case, "bf16", backward=False)
    O0, lse0 = O0.clone(), lse0.clone()
    for order in ([3, 2, 1, 0], [2, 3, 0, 1]):
        _, (O1, lse1, *_r) = run_case(case, "bf16", backward=False, order=order)
        compare_all_heads(case, "bf16", O1, lse1)
        assert float((lse1 - lse0).abs().max()) < 1e-5
    # two half walks from fresh states, merged, equal the straight walk
    wa = RingWalk(case["Q"], case["scale"])
    wb = RingWalk(case["Q"], case["scale"])
    wa.init(); wb.init()
    for j in (0, 1):
        wa.step(case["K"][j], case["V"][j], case["k_offs"][j])
    for j in (2, 3):
        wb.step(case["K"][j], case["V"][j], case["k_offs"][j])
    B.burst_merge_state(wa.O_acc, wa.m, wa.l, wb.O_acc, wb.m, wb.l, wa.params(0, 0))
    O2, lse2 = wa.finalize()
    torch.cuda.synchronize()
    compare_all_heads(case, "bf16", O2, lse2)
    assert float((lse2 - lse0).abs().max()) < 1e-5


@pytest.mark.parametrize("d", [128, 64])
def test_checkpoint_resume_and_determinism_are_bitwise(d):
    case = workloads.make_case(B=1, H=3, d=d, Nq=260, chunk_rows=[100, 130, 90], dtype="bf16", seed=41, device=DEV,
                               causal=True, q_off=60)
    _, (O0, lse0, dQ0, dKs0, dVs0) = run_case(case, "bf16")
    keep = [t.clone() for t in (O0, lse0, dQ0, *dKs0, *dVs0)]
    # same call sequence again: every output bit-identical (no atomics anywhere)
    _, (O1, lse1, dQ1, dKs1, dVs1) = run_case(case, "bf16")
    for a, b in zip(keep, (O1, lse1, dQ1, *dKs1, *dVs1)):
        assert torch.equal(a, b)
    # stop after chunk 0, move the state through host memory into new buffers, continue
    w1 = RingWalk(case["Q"], case["scale"], True, case["q_off"])
    w1.init()
    w1.step(case["K"][0], case["V"][0], case["k_offs"][0])
    saved = [t.cpu() for t in (w1.O_acc, w1.m, w1.l)]
    w2 = RingWalk(case["Q"], case["scale"], True, case["q_off"])
    for dst, src in zip((w2.O_acc, w2.m, w2.l), saved):
        dst.copy_(src)
    for j in (1, 2):
        w2.step(case["K"][j], case["V"][j], case["k_offs"][j])
    O2, lse2 = w2.finalize()
    torch.cuda.synchronize()
    assert torch.equal(O2, keep[0]) and torch.equal(lse2, keep[1])


@pytest.mark.parametrize("source", ["hbm", "pinned_host"])
def test_double_buffered_walk_is_bitwise_the_plain_walk(source):
    """Paper Sec. 2.5 / Alg. 3: fetching chunk j+1 into the alternate buffer on a second stream while
    chunk j computes must not change a single bit of the results (forward and backward)."""
    case = workloads.make_case(B=1, H=4, d=128, Nq=384, chunk_rows=[256, 192, 256, 128, 256], dtype="bf16", seed=43,
                               device=DEV, causal=True, q_off=700)
    plain = RingWalk(case["Q"], case["scale"], True, case["q_off"])
    O0, lse0 = plain.forward(case["K"], case["V"], case["k_offs"])
    dQ0, dKs0, dVs0 = plain.backward(case["K"], case["V"], case["k_offs"], case["dO"])
    torch.cuda.synchronize()
    if source == "pinned_host":
        src_K = [k.cpu().pin_memory() for k in case["K"]]
        src_V = [v.cpu().pin_memory() for v in case["V"]]
    else:
        src_K = [k.clone() for k in case["K"]]
        src_V = [v.clone() for v in case["V"]]
    for rep in range(2):                                  # second pass reuses the receive buffers
        db = DoubleBufferedWalk(case["Q"], case["scale"], True, case["q_off"]) if rep == 0 else db
        O1, lse1 = db.forward(src_K, src_V, case["k_offs"])
        dQ1, dKs1, dVs1 = db.backward(src_K, src_V, case["k_offs"], case["dO"])
        torch.cuda.synchronize()
        assert torch.equal(O1, O0) and torch.equal(lse1, lse0) and torch.equal(dQ1, dQ0)
        for a, b in zip(dKs1 + dVs1, dKs0 + dVs0):
            assert torch.equal(a, b)
        # and the double-buffered results themselves against the oracle, every head, all five outputs
        compare_all_heads(case, "bf16", O1, lse1, dQ1, dKs1, dVs1)


def test_backward_without_D_on_two_streams_at_once():
    """burst_local_bwd with D = NULL keeps one library-owned D buffer per (device, stream): two
    walks with different inputs and sizes, enqueued alternately on two streams with no event
    between them, must each give the gradients of the walk with D given, bit for bit (a buffer
    shared by the two streams would be overwritten by the other walk's D); the second, larger
    round also makes both buffers grow while the first round's kernels may still be running."""
    streams = [torch.cuda.Stream(device=DEV), torch.cuda.Stream(device=DEV)]
    for rnd, sizes in enumerate((((2, 200, [150, 170]), (3, 330, [260])), ((2, 900, [512, 300]), (4, 650, [700])))):
        cases, walks, refs = [], [], []
        for i, (H, Nq, rows) in enumerate(sizes):
            case = workloads.make_case(B=1, H=H, d=128, Nq=Nq, chunk_rows=rows, dtype="bf16", seed=70 + 2 * rnd + i,
                                       device=DEV, causal=bool(i), q_off=100 * i)
            walk, (O, lse, dQ, dKs, dVs) = run_case(case, "bf16", use_D=True)
            cases.append(case)
            walks.append(walk)
            refs.append((dQ.clone(), [t.clone() for t in dKs], [t.clone() for t in dVs]))
        torch.cuda.synchronize()
        outs = []
        for i, case in enumerate(cases):
            dQ = torch.zeros_like(refs[i][0])
            outs.append((dQ, [torch.empty_like(t) for t in refs[i][1]], [torch.empty_like(t) for t in refs[i][2]]))
        n_chunks = max(len(c["K"]) for c in cases)
        for j in range(n_chunks):                       # alternate the two streams chunk by chunk
            for i, case in enumerate(cases):
                if j >= len(case["K"]):
                    continue
                with torch.cuda.stream(streams[i]):
                    w = walks[i]
                    B.burst_local_bwd(case["Q"], case["K"][j], case["V"][j], w.O, case["dO"], w.lse, None,
                                      outs[i][0], outs[i][1][j], outs[i][2][j],
                                      w.params(case["K"][j].shape[2], case["k_offs"][j], None, case["K"][j]),
                                      accumulate_dq=True, accumulate_dkv=False)
        torch.cuda.synchronize()
        for (dQ, dKs, dVs), (rQ, rKs, rVs) in zip(outs, refs):
            assert torch.equal(dQ, rQ)
            for a, b in zip(dKs + dVs, rKs + rVs):
                assert torch.equal(a, b)


def test_backward_without_D_and_accumulate_flags():
    case = workloads.make_case(B=1, H=2, d=128, Nq=200, chunk_rows=[150, 170], dtype="bf16", seed=51, device=DEV)
    walk, (O, lse, dQ, dKs, dVs) = run_case(case, "bf16", use_D=True)
    dQ, dKs, dVs = dQ.clone(), [t.clone() for t in dKs], [t.clone() for t in dVs]
    dQ2, dKs2, dVs2 = walk.backward(case["K"], case["V"], case["k_offs"], case["dO"], use_D=False)
    torch.cuda.synchronize()
    assert torch.equal(dQ, dQ2)
    for a, b in zip(dKs + dVs, dKs2 + dVs2):
        assert torch.equal(a, b)
    # accumulate_dq = 0 overwrites whatever the buffer held; accumulate_dkv = 1 adds to it
    junk = torch.full_like(dQ, 123.0)
    p = walk.params(150, 0)
    B.burst_local_bwd(case["Q"], case["K"][0], case["V"][0], walk.O, case["dO"], walk.lse, walk.D,
                      junk, dKs2[0], dVs2[0], p, accumulate_dq=False, accumulate_dkv=True)
    torch.cuda.synchronize()
    only0 = torch.zeros_like(dQ)
    dk_tmp, dv_tmp = torch.empty_like(dKs[0]), torch.empty_like(dVs[0])
    B.burst_local_bwd(case["Q"], case["K"][0], case["V"][0], walk.O, case["dO"], walk.lse, walk.D,
                      only0, dk_tmp, dv_tmp, p, accumulate_dq=True, accumulate_dkv=False)
    torch.cuda.synchronize()
    assert torch.equal(junk, only0)
    assert torch.allclose(dKs2[0], 2 * dKs[0], rtol=1e-6, atol=1e-7)
    assert torch.allclose(dVs2[0], 2 * dVs[0], rtol=1e-6, atol=1e-7)


def test_key_side_pinned_orientation():
    """Alg. 2 as printed: K_i, V_i pinned, query slices (Q_j, dO_j, D_j, lse_j) visit; dK_i, dV_i accumulate."""
    spec = dict(B=1, H=2, d=128, dtype="bf16", seed=61, device=DEV)
    full = workloads.make_case(Nq=384, chunk_rows=[200], **spec)
    walk, (O, lse, dQ, dKs, dVs) = run_case(full, "bf16")
    dK = torch.zeros_like(dKs[0]); dV = torch.zeros_like(dVs[0])
    dQ_parts = []
    for s0, s1 in ((0, 128), (128, 384)):
        sl = lambda t: t[:, :, s0:s1].contiguous()
        Qj, dOj, Oj, lsej, Dj = sl(full["Q"]), sl(full["dO"]), sl(walk.O), sl(walk.lse), sl(walk.D)
        dQj = torch.zeros((1, 2, s1 - s0, 128), device=DEV)
        p = B.params(1, 2, s1 - s0, 200, 128, torch.bfloat16, full["scale"], False, s0, 0)
        B.burst_local_bwd(Qj, full["K"][0], full["V"][0], Oj, dOj, lsej, Dj, dQj, dK, dV, p,
                          accumulate_dq=True, accumulate_dkv=True)
        dQ_parts.append(dQj)
    torch.cuda.synchronize()
    assert torch.equal(torch.cat(dQ_parts, dim=2), dQ)
    assert torch.allclose(dK, dKs[0], rtol=1e-5, atol=1e-6) and torch.allclose(dV, dVs[0], rtol=1e-5, atol=1e-6)
    compare_all_heads(full, "bf16", O, lse, torch.cat(dQ_parts, dim=2), [dK], [dV])


def test_error_codes_on_device_buffers():
    x = torch.zeros(4096, device=DEV)
    p = B.params(1, 1, 16, 16, 128, torch.bfloat16, 0.5)
    with pytest.raises(B.BurstError) as e:
        B.burst_state_init(x[1:], x, x, p)                       # 4-byte offset: misaligned
    assert e.value.code == -2
    with pytest.raises(B.BurstError) as e:
        B.burst_local_fwd(None, x, x, x, x, x, p)
    assert e.value.code == -1
    bad = B.params(1, 1, 16, 16, 129, torch.bfloat16, 0.5)
    with pytest.raises(B.BurstError) as e:
        B.burst_state_init(x, x, x, bad)
    assert e.value.code == -3
    assert torch.all(x == 0)                                     # nothing was written


GUARD_CASES = {
    "d128": dict(B=1, H=3, d=128, Nq=333, chunk_rows=[257, 95], causal=True, q_off=40, window=200),
    "d128-flags-grouped": dict(B=1, H=6, kv_heads=3, d=128, Nq=320, chunk_rows=[257, 95], causal=True, q_off=40,
                               block=64, pattern="random", density=0.6),
    "d64": dict(B=1, H=3, d=64, Nq=333, chunk_rows=[257, 95], causal=True, q_off=40, window=200),
    "d64-flags-grouped": dict(B=1, H=6, kv_heads=2, d=64, Nq=301, chunk_rows=[200, 130], block=128, pattern="random",
                              density=0.5),
    "generic-f32": dict(B=1, H=2, d=48, Nq=77, chunk_rows=[65, 31], causal=True, q_off=20, dtype="f32"),
}


@pytest.mark.parametrize("name", list(GUARD_CASES))
def test_no_kernel_writes_outside_its_buffers(name):
    """Every output buffer (and the workspace of the stored-score step) sits between guard bands filled
    with a pattern; after the whole path has run on ragged shapes (tails in rows, keys and heads) the
    bands must be untouched, and so must the read-only inputs."""
    spec = dict(GUARD_CASES[name])
    dtype = spec.pop("dtype", "bf16")
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    case = workloads.make_case(dtype=dtype, seed=47, device=DEV, **spec)
    G = 4096                                    # guard elements on each side
    def guarded(shape, dt, fill=None):
        n = int(np.prod(shape))
        pat = 12345.0 if dt != torch.bfloat16 else 77.0
        flat = torch.full((n + 2 * G,), pat, device=DEV, dtype=dt)
        view = flat[G:G + n].view(*shape)
        if fill is not None:
            view.fill_(fill)
        return flat, view, pat
    Bt, H, Nq, d = case["Q"].shape
    bufs = {}
    for nm, shape, dt in (("O_acc", (Bt, H, Nq, d), torch.float32), ("m", (Bt, H, Nq), torch.float32),
                          ("l", (Bt, H, Nq), torch.float32), ("O", (Bt, H, Nq, d), tdt),
                          ("lse", (Bt, H, Nq), torch.float32), ("D", (Bt, H, Nq), torch.float32),
                          ("dQ", (Bt, H, Nq, d), torch.float32),
                          ("O_acc2", (Bt, H, Nq, d), torch.float32), ("m2", (Bt, H, Nq), torch.float32),
                          ("l2", (Bt, H, Nq), torch.float32)):
        bufs[nm] = guarded(shape, dt, 0.0 if nm == "dQ" else None)
    dK = [guarded(tuple(k.shape), torch.float32) for k in case["K"]]
    dV = [guarded(tuple(k.shape), torch.float32) for k in case["K"]]
    inputs_before = [t.clone() for t in (case["Q"], case["dO"], *case["K"], *case["V"])]
    masks = case.get("masks", [None] * len(case["K"]))
    prm = lambda Nc, ko, mask=None: B.params(Bt, H, Nq, Nc, d, tdt, case["scale"], case["causal"], case["q_off"], ko,
                                             case["window"], mask, case.get("block", 0), case.get("kv_heads", 0))
    v = {k: t[1] for k, t in bufs.items()}
    B.burst_state_init(v["O_acc"], v["m"], v["l"], prm(0, 0))
    for K, V, ko, mk in zip(case["K"], case["V"], case["k_offs"], masks):
        B.burst_local_fwd(case["Q"], K, V, v["O_acc"], v["m"], v["l"], prm(K.shape[2], ko, mk))
    B.burst_finalize(v["O_acc"], v["m"], v["l"], v["O"], v["lse"], prm(0, 0))
    B.burst_bwd_prepare(v["O"], case["dO"], v["D"], prm(0, 0))
    for j, (K, V, ko, mk) in enumerate(zip(case["K"], case["V"], case["k_offs"], masks)):
        B.burst_local_bwd(case["Q"], K, V, v["O"], case["dO"], v["lse"], v["D"], v["dQ"], dK[j][1], dV[j][1],
                          prm(K.shape[2], ko, mk), accumulate_dq=True, accumulate_dkv=False)
    # the chunk step that stores S and P, with a workspace of exactly the size it asks for
    B.burst_state_init(v["O_acc2"], v["m2"], v["l2"], prm(0, 0))
    spaces = []
    for K, V, ko, mk in zip(case["K"], case["V"], case["k_offs"], masks):
        need = B.burst_materialized_workspace_bytes(prm(K.shape[2], ko, mk))
        flat = torch.full((need + 2 * G,), 201, device=DEV, dtype=torch.uint8)
        spaces.append((flat, need))
        B.burst_local_fwd_materialized(case["Q"], K, V, v["O_acc2"], v["m2"], v["l2"], flat[G:G + need], prm(K.shape[2], ko, mk))
    torch.cuda.synchronize()
    for nm, (flat, view, pat) in list(bufs.items()) + [(f"dK{j}", t) for j, t in enumerate(dK)] + \
            [(f"dV{j}", t) for j, t in enumerate(dV)]:
        n = view.numel()
        assert bool((flat[:G] == pat).all()) and bool((flat[G + n:] == pat).all()), f"guard band of {nm} was written"
    for flat, need in spaces:
        assert bool((flat[:G] == 201).all()) and bool((flat[G + need:] == 201).all()), "guard band of the workspace was written"
    for before, now in zip(inputs_before, (case["Q"], case["dO"], *case["K"], *case["V"])):
        assert torch.equal(before, now)
    # and the results are the right ones (the two forward paths agree with the oracle independently)
    compare_all_heads(case, dtype, v["O"], v["lse"], v["dQ"], [t[1] for t in dK], [t[1] for t in dV])
    O2, lse2 = torch.empty_like(v["O"]), torch.empty_like(v["lse"])
    B.burst_finalize(v["O_acc2"], v["m2"], v["l2"], O2, lse2, prm(0, 0))
    torch.cuda.synchronize()
    compare_all_heads(case, dtype, O2, lse2)


@pytest.mark.parametrize("rank", [0, 2, 3])
def test_zigzag_rank_against_the_oracle(rank):
    """Load-balanced causal assignment: a rank owns stripes r and 2G-1-r of the sequence; its two
    query spans walk all 2G key/value stripes (most of them fully visible or skipped whole)."""
    N, G, H, d = 1536, 4, 2, 128
    n = N // (2 * G)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(900 + rank)
    mk = lambda rows: torch.randn((1, H, rows, d), generator=gen, device=DEV).to(torch.bfloat16)
    Ks, Vs = [mk(n) for _ in range(2 * G)], [mk(n) for _ in range(2 * G)]
    k_offs = [i * n for i in range(2 * G)]
    spans = workloads.zigzag_spans(N, G, rank)
    Qs, dOs = [mk(rows) for _, rows in spans], [mk(rows) for _, rows in spans]
    walk = SpanWalk(Qs, [first for first, _ in spans], 1.0 / np.sqrt(d), causal=True)
    outs = walk.forward(Ks, Vs, k_offs)
    dQs, dKs, dVs = walk.backward(Ks, Vs, k_offs, dOs)
    torch.cuda.synchronize()
    q_pos = np.concatenate([first + np.arange(rows) for first, rows in spans])
    for h in range(H):
        K = np.concatenate([f64(k[0, h]) for k in Ks])
        V = np.concatenate([f64(v[0, h]) for v in Vs])
        Q = np.concatenate([f64(q[0, h]) for q in Qs])
        dO = np.concatenate([f64(g[0, h]) for g in dOs])
        O_ref, lse_ref = orc.full_forward(Q, K, V, 1.0 / np.sqrt(d), True, q_pos, np.arange(N))
        dQ_ref, dK_ref, dV_ref = orc.full_backward(Q, K, V, dO, 1.0 / np.sqrt(d), True, q_pos, np.arange(N))
        check(f"O[h{h}]", np.concatenate([f64(o[0, h]) for o, _ in outs]), O_ref, "bf16")
        check(f"lse[h{h}]", np.concatenate([f64(l[0, h]) for _, l in outs]), lse_ref, "bf16", "lse")
        check(f"dQ[h{h}]", np.concatenate([f64(x[0, h]) for x in dQs]), dQ_ref, "bf16")
        check(f"dK[h{h}]", np.concatenate([f64(x[0, h]) for x in dKs]), dK_ref, "bf16")
        check(f"dV[h{h}]", np.concatenate([f64(x[0, h]) for x in dVs]), dV_ref, "bf16")


def test_autograd_wrapper_with_block_flags():
    from paper_2403_09347_amd.autograd import burst_attention
    case = workloads.make_case(B=1, H=2, d=128, Nq=300, chunk_rows=[256, 200], dtype="bf16", seed=61, device=DEV,
                               block=64, pattern="random", density=0.5, causal=True, q_off=200)
    q = case["Q"].clone().requires_grad_(True)
    ks = [k.clone().requires_grad_(True) for k in case["K"]]
    vs = [v.clone().requires_grad_(True) for v in case["V"]]
    O, lse = burst_attention(q, ks, vs, causal=True, q_off=200, block_masks=case["masks"], block=64)
    (O.float() * case["dO"].float()).sum().backward()
    torch.cuda.synchronize()
    compare_all_heads(case, "bf16", O.detach(), lse, q.grad.float(), [k.grad.float() for k in ks], [v.grad.float() for v in vs])


@pytest.mark.parametrize("layout", ["head", "seq"])
def test_autograd_wrapper_against_the_oracle(layout):
    """The differentiable torch call (chunk walk forward, Alg. 2 walk backward) on a causal, grouped-head
    case: outputs and the gradients autograd hands back, against the fp64 oracle.  "seq": the inputs
    are transposed views of [B, rows, H, d] leaves, read in place."""
    from paper_2403_09347_amd.autograd import burst_attention
    case = workloads.make_case(B=1, H=4, kv_heads=2, d=128, Nq=320, chunk_rows=[256, 100], dtype="bf16", seed=59,
                               device=DEV, causal=True, q_off=120, layout=layout)
    leaf = lambda t: t.detach().clone(memory_format=torch.preserve_format).requires_grad_(True)
    q = leaf(case["Q"])
    ks = [leaf(k) for k in case["K"]]
    vs = [leaf(v) for v in case["V"]]
    assert q.stride() == case["Q"].stride()
    O, lse = burst_attention(q, ks, vs, causal=True, q_off=120)
    (O.float() * case["dO"].float()).sum().backward()
    torch.cuda.synchronize()
    assert q.grad.dtype == torch.bfloat16 and ks[0].grad.shape == case["K"][0].shape
    compare_all_heads(case, "bf16", O.detach(), lse, q.grad.float(), [k.grad.float() for k in ks], [v.grad.float() for v in vs])


def test_c_abi_called_with_raw_pointers():
    """The boundary without the binding's helpers: the shared library loaded with ctypes, a parameter
    block laid out by hand, raw device addresses, the default stream; result against the oracle."""
    import ctypes
    import struct
    lib = ctypes.CDLL(B.LIB_PATH)
    Bt, H, Nq, Nc, d = 1, 2, 96, 160, 128
    case = workloads.make_case(B=Bt, H=H, d=d, Nq=Nq, chunk_rows=[Nc], dtype="bf16", seed=83, device=DEV, causal=True,
                               q_off=64)
    # burst_params: 7 x int32, float, 3 x int64, pointer, 2 x int32, 7 x int64 (mask stride, 2 x 3 strides)
    blob = struct.pack("<7if3qQ2i7q", Bt, H, Nq, Nc, d, 0, 1, case["scale"], 64, 0, 0, 0, 0, 0, *([0] * 7))
    assert len(blob) == 128
    params = ctypes.create_string_buffer(blob)
    O_acc = torch.empty((Bt, H, Nq, d), device=DEV, dtype=torch.float32)
    m = torch.empty((Bt, H, Nq), device=DEV, dtype=torch.float32)
    l = torch.empty_like(m)
    O = torch.empty((Bt, H, Nq, d), device=DEV, dtype=torch.bfloat16)
    lse = torch.empty_like(m)
    ptr = lambda t: ctypes.c_void_p(t.data_ptr())
    for fn in (lib.burst_state_init, lib.burst_local_fwd, lib.burst_finalize):
        fn.restype = ctypes.c_int
    torch.cuda.synchronize()                       # the calls below go to the default stream (NULL)
    assert lib.burst_state_init(ptr(O_acc), ptr(m), ptr(l), params, None) == 0
    assert lib.burst_local_fwd(ptr(case["Q"]), ptr(case["K"][0]), ptr(case["V"][0]), ptr(O_acc), ptr(m), ptr(l),
                               params, None) == 0
    assert lib.burst_finalize(ptr(O_acc), ptr(m), ptr(l), ptr(O), ptr(lse), params, None) == 0
    torch.cuda.synchronize()
    compare_all_heads(case, "bf16", O, lse)


@pytest.mark.parametrize("source", ["hbm", "pinned_host"])
def test_whole_ring_emulated_with_the_paper_orientation_backward(source):
    """Four devices' worth of a causal sequence on one GPU.  Forward: every device walks all chunks
    (Alg. 1).  Backward as the paper prints it (Alg. 2, double buffer of Alg. 4): every device keeps
    its K_i, V_i; the payloads (Q_j, dO_j, D_j, lse_j, dQ_j) of all devices pass through two receive
    buffers, each dQ_j collecting one contribution per device.  Everything against the oracle's
    gradient of attention over the whole sequence."""
    G, n, H, d = 4, 192, 2, 128
    case = workloads.make_case(B=1, H=H, d=d, Nq=G * n, chunk_rows=[n] * G, dtype="bf16", seed=89, device=DEV,
                               causal=True, q_off=0)
    sl = lambda t, i: t[:, :, i * n:(i + 1) * n].contiguous()
    payloads, O_parts, lse_parts = [], [], []
    for i in range(G):                                           # forward on "device" i
        walk = RingWalk(sl(case["Q"], i), case["scale"], True, i * n)
        O_i, lse_i = walk.forward(case["K"], case["V"], case["k_offs"], order=[(i + s) % G for s in range(G)])
        walk.prepare(sl(case["dO"], i))
        O_parts.append(O_i); lse_parts.append(lse_i)
        pay = {"Q": walk.Q, "dO": sl(case["dO"], i), "D": walk.D.clone(), "lse": lse_i.clone(),
               "dQ": torch.zeros((1, H, n, d), device=DEV, dtype=torch.float32), "q_off": i * n}
        if source == "pinned_host":
            pay = {k: (v.cpu().pin_memory() if torch.is_tensor(v) else v) for k, v in pay.items()}
        payloads.append(pay)
    torch.cuda.synchronize()
    dKs, dVs = [], []
    for i in range(G):                                           # backward on "device" i: payloads arrive in ring order
        dev_i = KeyPinnedBackward(case["K"][i], case["V"][i], case["scale"], True, i * n)
        dK_i, dV_i = dev_i.backward([payloads[(i + s) % G] for s in range(G)])
        torch.cuda.synchronize()
        dKs.append(dK_i); dVs.append(dV_i)
    dQ = torch.cat([p["dQ"].to(DEV) for p in payloads], dim=2)
    compare_all_heads(case, "bf16", torch.cat(O_parts, dim=2), torch.cat(lse_parts, dim=2), dQ, dKs, dVs)


@pytest.mark.parametrize("dtype,spec", [
    ("f32", dict(B=1, H=1, d=64, Nq=256, chunk_rows=[256] * 4)),                                     # the tiny fp32 configuration
    ("bf16", dict(B=1, H=3, d=128, Nq=300, chunk_rows=[200, 64, 331], causal=True, q_off=295)),
    ("bf16", dict(B=1, H=4, d=64, Nq=256, chunk_rows=[256, 130], block=64, pattern="random", density=0.5, kv_heads=2)),
])
def test_step_recorded_as_a_graph_replays_bitwise(dtype, spec):
    """A whole step recorded as one HIP graph: three replays, each on new input values copied into
    the recorded tensors, with eager work and synchronisations of its own between them, every
    replay bitwise equal to the eager step on the same values; the last one also against the oracle."""
    from paper_2403_09347_amd.harness import GraphedStep
    case = workloads.make_case(dtype=dtype, seed=101, device=DEV, **spec)
    args = (case["scale"], case["causal"], case["q_off"], case.get("window", 0), case.get("block", 0), case.get("kv_heads", 0))
    walk = RingWalk(case["Q"].clone(), *args)
    Ks, Vs, dO = [k.clone() for k in case["K"]], [v.clone() for v in case["V"]], case["dO"].clone()
    step = GraphedStep(walk, Ks, Vs, case["k_offs"], dO, masks=case.get("masks"))
    for rep in range(3):
        fresh = workloads.make_case(dtype=dtype, seed=200 + rep, device=DEV, **spec) if rep < 2 else case
        if "masks" in case:                                            # the recording holds the block flags
            fresh = dict(fresh, masks=case["masks"], flags=case["flags"])
        walk.Q.copy_(fresh["Q"]); dO.copy_(fresh["dO"])
        for dst, src in zip(Ks + Vs, fresh["K"] + fresh["V"]):
            dst.copy_(src)
        O, lse, dQ, dKs, dVs = step.replay()
        torch.cuda.synchronize()
        got = [t.clone() for t in (O, lse, dQ, *dKs, *dVs)]
        _, (O2, lse2, dQ2, dKs2, dVs2) = run_case(fresh, dtype)           # eager work between the replays
        for a, b in zip(got, (O2, lse2, dQ2, *dKs2, *dVs2)):
            assert torch.equal(a, b)
    compare_all_heads(case, dtype, got[0], got[1], got[2], got[3:3 + len(Ks)], got[3 + len(Ks):])
