"""The C-ABI library loads and exports every symbol that include/burst.h declares."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "burst.h")
LIB = os.path.join(ROOT, "paper_2403_09347_amd", "libburst.so")


def declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(burst_[a-z_0-9]+)\s*\(", text)))


def test_header_declares_the_boundary():
    names = declared_symbols()
    for required in ("burst_state_init", "burst_local_fwd", "burst_finalize", "burst_merge_state",
                     "burst_bwd_prepare", "burst_local_bwd", "burst_strerror", "burst_version"):
        assert required in names


def test_library_exports_every_declared_symbol():
    if not os.path.exists(LIB):
        pytest.fail("libburst.so is not built: run __graft_entry__.build() first")
    lib = ctypes.CDLL(LIB)
    for name in declared_symbols():
        assert hasattr(lib, name), name
    lib.burst_version.restype = ctypes.c_int
    assert lib.burst_version() >= 100
    lib.burst_strerror.restype = ctypes.c_char_p
    lib.burst_strerror.argtypes = [ctypes.c_int]
    assert lib.burst_strerror(0) == b"ok"
    assert b"NULL" in lib.burst_strerror(-1)


def test_binding_lists_the_same_exports():
    from paper_2403_09347_amd import binding
    assert sorted(binding.EXPORTS) == declared_symbols()
    p = binding.params(1, 2, 3, 4, 128, "bf16", 0.5, True, 7, 9)
    assert (p.B, p.H, p.Nq, p.Nc, p.d, p.dtype, p.causal, p.q_off, p.k_off) == (1, 2, 3, 4, 128, 0, 1, 7, 9)
    assert ctypes.sizeof(p) == 128
    assert (p.block_mask, p.block, p.kv_heads, p.block_mask_stride) == (None, 0, 0, 0)


def test_argument_validation_without_gpu():
    """Bad parameter blocks are rejected before any device call."""
    from paper_2403_09347_amd import binding
    lib = binding.load()
    null = ctypes.c_void_p(0)
    bad = binding.params(1, 1, 16, 16, 128, 7, 0.5)            # unknown dtype
    assert lib.burst_state_init(null, null, null, ctypes.byref(bad), null) == -4
    bad = binding.params(1, 1, 16, 16, 300, "bf16", 0.5)       # d too large
    assert lib.burst_state_init(null, null, null, ctypes.byref(bad), null) == -3
    bad = binding.params(1, 1, 16, 16, 128, "bf16", -1.0)      # scale must be > 0
    assert lib.burst_local_fwd(null, null, null, null, null, null, ctypes.byref(bad), null) == -3
    bad = binding.params(1, 1, 16, 16, 128, "bf16", 0.5, window=-3)   # window must be >= 0
    assert lib.burst_local_fwd(null, null, null, null, null, null, ctypes.byref(bad), null) == -3
    bad = binding.params(1, 1, 16, 16, 128, "bf16", 0.5)
    bad.block_mask, bad.block = 4096, 48                        # block edge must be a multiple of 64
    assert lib.burst_local_fwd(null, null, null, null, null, null, ctypes.byref(bad), null) == -3
    bad = binding.params(1, 2, 128, 128, 128, "bf16", 0.5)
    bad.block_mask, bad.block, bad.block_mask_stride = 4096, 64, 3   # per-head matrices (2 x 2 bytes) would overlap
    assert lib.burst_local_fwd(null, null, null, null, null, null, ctypes.byref(bad), null) == -3
    bad = binding.params(1, 2, 16, 16, 128, "bf16", 0.5, q_strides=(4096, 128, 64))    # row stride below d
    assert lib.burst_local_fwd(null, null, null, null, null, null, ctypes.byref(bad), null) == -3
    bad = binding.params(1, 2, 16, 16, 128, "bf16", 0.5, kv_strides=(4096, 132, 256))  # head stride not 16-byte aligned
    assert lib.burst_local_fwd(null, null, null, null, null, null, ctypes.byref(bad), null) == -3
    bad = binding.params(1, 6, 16, 16, 128, "bf16", 0.5, kv_heads=4)   # H must be a multiple of kv_heads
    assert lib.burst_local_fwd(null, null, null, null, null, null, ctypes.byref(bad), null) == -3
    ok = binding.params(1, 1, 16, 16, 128, "bf16", 0.5)
    assert lib.burst_state_init(null, null, null, ctypes.byref(ok), null) == -1      # NULL pointer
    assert lib.burst_state_init(null, null, null, None, null) == -1                  # NULL params
    mis = ctypes.c_void_p(8)
    assert lib.burst_state_init(mis, mis, mis, ctypes.byref(ok), null) == -2         # misaligned
    empty = binding.params(1, 1, 0, 16, 128, "bf16", 0.5)      # nothing to do: ok without pointers
    assert lib.burst_state_init(null, null, null, ctypes.byref(empty), null) == 0


def test_materialized_workspace_size_without_gpu():
    """S (fp32) + P (input type) with the key count rounded up to 8, each region rounded up to
    256 bytes, plus two per-row vectors; 0 for an invalid parameter block."""
    from paper_2403_09347_amd import binding
    p = binding.params(1, 2, 5, 9, 8, "bf16", 0.5)             # 10 rows x 16 padded keys
    assert binding.burst_materialized_workspace_bytes(p) == 768 + 512 + 2 * 256
    p = binding.params(2, 2, 5, 16, 8, "f32", 0.5)             # 20 rows x 16 keys
    assert binding.burst_materialized_workspace_bytes(p) == 1280 + 1280 + 2 * 256
    bad = binding.params(1, 1, 16, 16, 300, "bf16", 0.5)
    assert binding.burst_materialized_workspace_bytes(bad) == 0
    assert binding.burst_workspace_bytes(binding.params(2, 3, 100, 40, 128, "bf16", 0.5)) == 2 * 3 * 100 * 4
    assert binding.burst_workspace_bytes(bad) == 0
    lib = binding.load()
    null = ctypes.c_void_p(0)
    assert lib.burst_local_fwd_materialized(null, null, null, null, null, null, null, 0, ctypes.byref(bad), null) == -3
