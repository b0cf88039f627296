"""ctypes binding of libburst.so: same names as the C ABI, argument marshalling only.

Every step of the path runs inside the library's HIP kernels; nothing here computes.
PyTorch tensors are used as device buffers; kernels are enqueued on torch's current
stream.  There is no fallback: if the library is missing, loading raises.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libburst.so")

BURST_BF16, BURST_F32 = 0, 1

EXPORTS = [
    "burst_state_init", "burst_local_fwd", "burst_finalize", "burst_merge_state",
    "burst_bwd_prepare", "burst_local_bwd", "burst_local_bwd_dq", "burst_local_bwd_dkv", "burst_event_create", "burst_event_record",
    "burst_event_elapsed_ms", "burst_event_destroy", "burst_strerror", "burst_version",
    "burst_materialized_workspace_bytes", "burst_local_fwd_materialized", "burst_workspace_bytes",
    "burst_materialized_bwd_workspace_bytes", "burst_local_bwd_materialized", "burst_set_kernel_family",
    "burst_kernel_family_for", "burst_local_bwd_static", "burst_probe_mfma", "burst_probe_atomic_dq",
]


class BurstParams(ctypes.Structure):
    _fields_ = [
        ("B", ctypes.c_int32), ("H", ctypes.c_int32), ("Nq", ctypes.c_int32), ("Nc", ctypes.c_int32),
        ("d", ctypes.c_int32), ("dtype", ctypes.c_int32), ("causal", ctypes.c_int32),
        ("scale", ctypes.c_float), ("q_off", ctypes.c_int64), ("k_off", ctypes.c_int64),
        ("window", ctypes.c_int64), ("block_mask", ctypes.c_void_p), ("block", ctypes.c_int32),
        ("kv_heads", ctypes.c_int32), ("block_mask_stride", ctypes.c_int64),
        ("q_strides", ctypes.c_int64 * 3), ("kv_strides", ctypes.c_int64 * 3),
    ]


class BurstError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        super().__init__(f"{where}: {strerror(code)} (status {code})")


_lib = None


def load():
    """Loads the shared library (once).  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} not found: build it first (python -c 'import __graft_entry__ as g; g.build()')")
    lib = ctypes.CDLL(LIB_PATH)
    vp, fp, pp = ctypes.c_void_p, ctypes.c_void_p, ctypes.POINTER(BurstParams)
    lib.burst_state_init.argtypes = [fp, fp, fp, pp, vp]
    lib.burst_local_fwd.argtypes = [vp, vp, vp, fp, fp, fp, pp, vp]
    lib.burst_finalize.argtypes = [fp, fp, fp, vp, fp, pp, vp]
    lib.burst_materialized_workspace_bytes.argtypes = [pp]
    lib.burst_materialized_workspace_bytes.restype = ctypes.c_size_t
    lib.burst_materialized_bwd_workspace_bytes.argtypes = [pp]
    lib.burst_materialized_bwd_workspace_bytes.restype = ctypes.c_size_t
    lib.burst_workspace_bytes.argtypes = [pp]
    lib.burst_workspace_bytes.restype = ctypes.c_size_t
    lib.burst_local_fwd_materialized.argtypes = [vp, vp, vp, fp, fp, fp, vp, ctypes.c_size_t, pp, vp]
    lib.burst_local_fwd_materialized.restype = ctypes.c_int
    lib.burst_local_bwd_materialized.argtypes = [vp, vp, vp, vp, fp, fp, fp, fp, fp, ctypes.c_int, ctypes.c_int,
                                                 vp, ctypes.c_size_t, pp, vp]
    lib.burst_local_bwd_materialized.restype = ctypes.c_int
    lib.burst_merge_state.argtypes = [fp, fp, fp, fp, fp, fp, pp, vp]
    lib.burst_bwd_prepare.argtypes = [vp, vp, fp, pp, vp]
    lib.burst_local_bwd.argtypes = [vp, vp, vp, vp, vp, fp, fp, fp, fp, fp, ctypes.c_int, ctypes.c_int, pp, vp]
    lib.burst_local_bwd_static.argtypes = [vp, vp, vp, vp, vp, fp, fp, fp, fp, ctypes.c_int, ctypes.c_int, pp, vp]
    lib.burst_local_bwd_static.restype = ctypes.c_int
    lib.burst_local_bwd_dq.argtypes = [vp, vp, vp, vp, fp, fp, fp, ctypes.c_int, pp, vp]
    lib.burst_local_bwd_dkv.argtypes = [vp, vp, vp, vp, fp, fp, fp, fp, ctypes.c_int, pp, vp]
    for name in ("burst_local_bwd_dq", "burst_local_bwd_dkv", "burst_state_init", "burst_local_fwd", "burst_finalize", "burst_merge_state",
                 "burst_bwd_prepare", "burst_local_bwd", "burst_event_record", "burst_version"):
        getattr(lib, name).restype = ctypes.c_int
    lib.burst_event_create.argtypes = []
    lib.burst_event_create.restype = vp
    lib.burst_event_record.argtypes = [vp, vp]
    lib.burst_event_elapsed_ms.argtypes = [vp, vp, ctypes.POINTER(ctypes.c_float)]
    lib.burst_event_elapsed_ms.restype = ctypes.c_int
    lib.burst_event_destroy.argtypes = [vp]
    lib.burst_event_destroy.restype = None
    lib.burst_strerror.argtypes = [ctypes.c_int]
    lib.burst_strerror.restype = ctypes.c_char_p
    _lib = lib
    return lib


def strerror(code):
    return load().burst_strerror(int(code)).decode()


def version():
    return load().burst_version()


def strides_of(t):
    """(batch, head, row) element strides of a [B, H, rows, d] tensor whose last dimension is
    contiguous, for params(); None if the tensor is contiguous.  Dimensions of size 1 (whose
    stride addresses nothing) are given the row length."""
    if t.dim() != 4 or (t.shape[3] > 1 and t.stride(3) != 1):
        raise ValueError("a [B, H, rows, d] tensor with a contiguous last dimension expected")
    if t.is_contiguous():
        return None
    return tuple(int(t.stride(i)) if t.shape[i] > 1 else int(t.shape[3]) for i in range(3))


def params(B, H, Nq, Nc, d, dtype, scale, causal=False, q_off=0, k_off=0, window=0, block_mask=None, block=0,
           kv_heads=0, q_strides=None, kv_strides=None):
    """block_mask: a contiguous uint8 device tensor [ceil(Nq/block), ceil(Nc/block)] shared by all
    heads, or [B, H, ceil(Nq/block), ceil(Nc/block)] with one matrix per (batch, query head) (or
    None); the caller keeps it alive and unchanged until the kernels that use these parameters
    have run.  q_strides / kv_strides: (batch, head, row) element strides of Q, dO, O and of
    K, V (see strides_of); None = contiguous."""
    code = {torch.bfloat16: BURST_BF16, torch.float32: BURST_F32, "bf16": BURST_BF16, "f32": BURST_F32}.get(dtype, dtype)
    ptr, stride = None, 0
    if block_mask is not None:
        if block_mask.dtype != torch.uint8 or not block_mask.is_cuda or not block_mask.is_contiguous():
            raise ValueError("block_mask: contiguous uint8 device tensor expected")
        if block <= 0:
            raise ValueError("block_mask needs block > 0")
        one = (-(-Nq // block), -(-Nc // block))
        if tuple(block_mask.shape) == (B, H) + one:
            stride = one[0] * one[1]
        elif tuple(block_mask.shape) != one:
            raise ValueError("block_mask: shape must be [ceil(Nq/block), ceil(Nc/block)], alone or after [B, H]")
        ptr = block_mask.data_ptr()
    return BurstParams(B, H, Nq, Nc, d, code, 1 if causal else 0, scale, q_off, k_off, window, ptr,
                       block if block_mask is not None else 0, kv_heads, stride,
                       (ctypes.c_int64 * 3)(*(q_strides or (0, 0, 0))), (ctypes.c_int64 * 3)(*(kv_strides or (0, 0, 0))))


def _ptr(t):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("device tensor expected")
    if not t.is_contiguous():
        raise ValueError("contiguous tensor expected")
    return ctypes.c_void_p(t.data_ptr())


def _strided(t, want):
    """Pointer of a storage-type tensor that must lie in memory as the parameter block says."""
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("device tensor expected")
    want = tuple(want)
    if want == (0, 0, 0):
        if not t.is_contiguous():
            raise ValueError("contiguous tensor expected (or give its strides to params())")
    else:
        if t.dim() != 4 or (t.shape[3] > 1 and t.stride(3) != 1):
            raise ValueError("a [B, H, rows, d] tensor with a contiguous last dimension expected")
        if any(t.shape[i] > 1 and t.stride(i) != want[i] for i in range(3)):
            raise ValueError(f"tensor strides {tuple(t.stride())} differ from the parameter block's {want}")
    return ctypes.c_void_p(t.data_ptr())


def _q(t, p):
    return _strided(t, p.q_strides)


def _kv(t, p):
    return _strided(t, p.kv_strides)


def _f32(t):
    if t is not None and t.dtype != torch.float32:
        raise ValueError("float32 tensor expected")
    return _ptr(t)


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(code, where):
    if code != 0:
        raise BurstError(code, where)


def burst_state_init(O_acc, m, l, p):
    _check(load().burst_state_init(_f32(O_acc), _f32(m), _f32(l), ctypes.byref(p), _stream()), "burst_state_init")


def burst_local_fwd(Q, K_chunk, V_chunk, O_acc, m, l, p):
    _check(load().burst_local_fwd(_q(Q, p), _kv(K_chunk, p), _kv(V_chunk, p), _f32(O_acc), _f32(m), _f32(l),
                                  ctypes.byref(p), _stream()), "burst_local_fwd")


def burst_set_kernel_family(family):
    """0 = automatic, 1 = hand-scheduled d = 128 kernels only, 2 = plainly written ones (see burst.h)."""
    lib = load()
    lib.burst_set_kernel_family.argtypes = [ctypes.c_int]
    lib.burst_set_kernel_family.restype = ctypes.c_int
    _check(lib.burst_set_kernel_family(int(family)), "burst_set_kernel_family")


def burst_kernel_family_for(p):
    lib = load()
    lib.burst_kernel_family_for.argtypes = [ctypes.POINTER(BurstParams)]
    lib.burst_kernel_family_for.restype = ctypes.c_int
    return int(lib.burst_kernel_family_for(ctypes.byref(p)))


def burst_probe_mfma(a_from_lds, wavefronts_per_simd, operands, sink, iters):
    """operands: >= 64 KiB of bf16 on the device; sink: >= 256 * 512 float32 (see burst.h)."""
    lib = load()
    lib.burst_probe_mfma.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int,
                                     ctypes.c_void_p]
    lib.burst_probe_mfma.restype = ctypes.c_int
    if operands.numel() * operands.element_size() < 65536 or sink.numel() < 256 * 512:
        raise ValueError("burst_probe_mfma: operands >= 64 KiB and sink >= 131072 floats expected")
    _check(lib.burst_probe_mfma(int(a_from_lds), int(wavefronts_per_simd), _ptr(operands), _f32(sink), int(iters),
                                _stream()), "burst_probe_mfma")


def burst_probe_atomic_dq(dQ, heads, Nq, key_blocks, mode):
    """mode: 1 = fp32 atomic adds, 0 = plain stores, 2 = plain load-add-store (see burst.h)."""
    lib = load()
    lib.burst_probe_atomic_dq.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                          ctypes.c_void_p]
    lib.burst_probe_atomic_dq.restype = ctypes.c_int
    if dQ.numel() < heads * Nq * 128:
        raise ValueError("burst_probe_atomic_dq: dQ too small")
    _check(lib.burst_probe_atomic_dq(_f32(dQ), int(heads), int(Nq), int(key_blocks), int(mode), _stream()),
           "burst_probe_atomic_dq")


def burst_workspace_bytes(p):
    return int(load().burst_workspace_bytes(ctypes.byref(p)))


def burst_materialized_workspace_bytes(p):
    return int(load().burst_materialized_workspace_bytes(ctypes.byref(p)))


def burst_local_fwd_materialized(Q, K_chunk, V_chunk, O_acc, m, l, workspace, p):
    """workspace: a contiguous uint8 device tensor (see burst_materialized_workspace_bytes)."""
    _check(load().burst_local_fwd_materialized(_q(Q, p), _kv(K_chunk, p), _kv(V_chunk, p), _f32(O_acc), _f32(m), _f32(l),
                                               _ptr(workspace), ctypes.c_size_t(workspace.numel() * workspace.element_size()),
                                               ctypes.byref(p), _stream()), "burst_local_fwd_materialized")


def burst_materialized_bwd_workspace_bytes(p):
    return int(load().burst_materialized_bwd_workspace_bytes(ctypes.byref(p)))


def burst_local_bwd_materialized(Q, K_chunk, V_chunk, dO, lse, D, dQ, dK_chunk, dV_chunk, workspace, p,
                                 accumulate_dq=True, accumulate_dkv=False):
    """workspace: a contiguous uint8 device tensor (see burst_materialized_bwd_workspace_bytes)."""
    _check(load().burst_local_bwd_materialized(_q(Q, p), _kv(K_chunk, p), _kv(V_chunk, p), _q(dO, p), _f32(lse), _f32(D),
                                               _f32(dQ), _f32(dK_chunk), _f32(dV_chunk),
                                               1 if accumulate_dq else 0, 1 if accumulate_dkv else 0,
                                               _ptr(workspace), ctypes.c_size_t(workspace.numel() * workspace.element_size()),
                                               ctypes.byref(p), _stream()), "burst_local_bwd_materialized")


def burst_finalize(O_acc, m, l, O_out, lse, p):
    _check(load().burst_finalize(_f32(O_acc), _f32(m), _f32(l), _q(O_out, p), _f32(lse),
                                 ctypes.byref(p), _stream()), "burst_finalize")


def burst_merge_state(O_a, m_a, l_a, O_b, m_b, l_b, p):
    _check(load().burst_merge_state(_f32(O_a), _f32(m_a), _f32(l_a), _f32(O_b), _f32(m_b), _f32(l_b),
                                    ctypes.byref(p), _stream()), "burst_merge_state")


def burst_bwd_prepare(O, dO, D, p):
    _check(load().burst_bwd_prepare(_q(O, p), _q(dO, p), _f32(D), ctypes.byref(p), _stream()), "burst_bwd_prepare")


def burst_local_bwd(Q, K_chunk, V_chunk, O, dO, lse, D, dQ, dK_chunk, dV_chunk, p,
                    accumulate_dq=True, accumulate_dkv=False):
    _check(load().burst_local_bwd(_q(Q, p), _kv(K_chunk, p), _kv(V_chunk, p), _q(O, p), _q(dO, p), _f32(lse), _f32(D),
                                  _f32(dQ), _f32(dK_chunk), _f32(dV_chunk),
                                  1 if accumulate_dq else 0, 1 if accumulate_dkv else 0,
                                  ctypes.byref(p), _stream()), "burst_local_bwd")


BURST_STATIC_MAX_ROWS = 2 * 1024 * 1024


def burst_local_bwd_static(Q, K_chunk, V_chunk, O, dO, lse, dQ, dK_chunk, dV_chunk, p,
                           accumulate_dq=True, accumulate_dkv=False):
    """burst_local_bwd with D computed into the library's static device scratch: allocates nothing."""
    _check(load().burst_local_bwd_static(_q(Q, p), _kv(K_chunk, p), _kv(V_chunk, p), _q(O, p), _q(dO, p), _f32(lse),
                                         _f32(dQ), _f32(dK_chunk), _f32(dV_chunk),
                                         1 if accumulate_dq else 0, 1 if accumulate_dkv else 0,
                                         ctypes.byref(p), _stream()), "burst_local_bwd_static")


def burst_local_bwd_dq(Q, K_chunk, V_chunk, dO, lse, D, dQ, p, accumulate_dq=True):
    _check(load().burst_local_bwd_dq(_q(Q, p), _kv(K_chunk, p), _kv(V_chunk, p), _q(dO, p), _f32(lse), _f32(D),
                                     _f32(dQ), 1 if accumulate_dq else 0, ctypes.byref(p), _stream()),
           "burst_local_bwd_dq")


def burst_local_bwd_dkv(Q, K_chunk, V_chunk, dO, lse, D, dK_chunk, dV_chunk, p, accumulate_dkv=False):
    _check(load().burst_local_bwd_dkv(_q(Q, p), _kv(K_chunk, p), _kv(V_chunk, p), _q(dO, p), _f32(lse), _f32(D),
                                      _f32(dK_chunk), _f32(dV_chunk), 1 if accumulate_dkv else 0,
                                      ctypes.byref(p), _stream()), "burst_local_bwd_dkv")


class Event:
    """HIP event recorded on the stream the kernels are launched on."""

    def __init__(self):
        self.h = load().burst_event_create()
        if not self.h:
            raise RuntimeError("burst_event_create failed")

    def record(self):
        _check(load().burst_event_record(self.h, _stream()), "burst_event_record")

    def elapsed_ms_until(self, stop):
        ms = ctypes.c_float(0.0)
        _check(load().burst_event_elapsed_ms(self.h, stop.h, ctypes.byref(ms)), "burst_event_elapsed_ms")
        return ms.value

    def __del__(self):
        try:
            if self.h:
                load().burst_event_destroy(self.h)
                self.h = None
        except Exception:
            pass
