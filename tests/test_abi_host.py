"""Host-side checks of the C-ABI library that need no GPU: it loads, exports
every symbol the header declares, and rejects bad arguments before touching
the device."""
import ctypes
import os
import re

import pytest

import paper_2411_08446_amd as lsh

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "lshmoe.h")


@pytest.fixture(scope="module")
def lib():
    from paper_2411_08446_amd import build
    if not os.path.exists(lsh.LIB_PATH) or not os.path.exists(build.PEAKS_LIB_PATH):
        build.build(verbose=False)
    return lsh.load_library()


def _declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lshmoe_[a-z_0-9]+)\s*\(", text)))


def test_header_symbols_are_exported(lib):
    names = _declared_symbols()
    assert {"lshmoe_hash", "lshmoe_compress", "lshmoe_decompress", "lshmoe_decompress_combine", "lshmoe_workspace_bytes",
            "lshmoe_backward_workspace_bytes", "lshmoe_decompress_backward", "lshmoe_compress_backward", "lshmoe_hash_gate",
            "lshmoe_status_string", "lshmoe_last_error", "lshmoe_abi_version", "lshmoe_compress_static", "lshmoe_decompress_combine_backward", "lshmoe_hash_sphere"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def test_probe_library_loads_and_exports(lib):
    # the measured-peak probes of bench.py --peaks live in a library of their own, built by the same build step
    from paper_2411_08446_amd import build
    assert os.path.exists(build.PEAKS_LIB_PATH)
    probes = ctypes.CDLL(build.PEAKS_LIB_PATH)
    for n in ("peaks_read", "peaks_copy", "peaks_mfma_bf16"):
        assert hasattr(probes, n), n
    probes.peaks_read.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p]
    assert probes.peaks_read(None, 16, None, 1, None) != 0          # rejected before any GPU call


def test_status_strings(lib):
    assert lib.lshmoe_status_string(0) == b"LSHMOE_OK"
    assert lib.lshmoe_status_string(4) == b"LSHMOE_ERR_WORKSPACE"
    assert lib.lshmoe_status_string(99) == b"LSHMOE_ERR_UNKNOWN"


def test_workspace_bytes_and_shape_errors(lib):
    n = lsh.lshmoe_workspace_bytes(65536, 1024, 2, 64, 4, 64, lsh.LSHMOE_BF16)
    N = 131072
    # two (key, index) buffers and a count table, plus the centroid step's window sums (2 rows of d binary32 per 128 positions)
    assert n >= 2 * N * 8 + 2 * N * 4 + (N // 64) * 1024 * 4 and n < 64 * N + (N // 64) * 1024 * 4
    assert lib.lshmoe_last_error() == b""
    for args, code in [
        ((0, 1024, 2, 64, 4, 64, 1), lsh.LSHMOE_ERR_SHAPE),
        ((16, 1024, 3, 2, 4, 64, 1), lsh.LSHMOE_ERR_SHAPE),          # k > E
        ((16, 1024, 1, 2, 0, 64, 1), lsh.LSHMOE_ERR_SHAPE),
        ((16, 1023, 1, 2, 4, 64, 1), lsh.LSHMOE_ERR_UNSUPPORTED),    # row not a multiple of 16 bytes
        ((16, 1022, 1, 2, 4, 64, 0), lsh.LSHMOE_ERR_UNSUPPORTED),
        ((16, 1024, 1, 2, 9, 64, 1), lsh.LSHMOE_ERR_UNSUPPORTED),    # (2r)^L = 2^63
        ((16, 1024, 1, 2, 4, 1, 1), lsh.LSHMOE_ERR_UNSUPPORTED),     # r < 2
        ((16, 1024, 1, 70000, 8, 64, 1), lsh.LSHMOE_ERR_UNSUPPORTED),  # 17 expert bits + 56 bucket bits
        ((2 ** 30, 8, 1, 2, 2, 4, 1), lsh.LSHMOE_ERR_UNSUPPORTED),
        ((16, 1024, 1, 2, 4, 64, 7), lsh.LSHMOE_ERR_UNSUPPORTED),    # unknown dtype
    ]:
        with pytest.raises(lsh.LshmoeError) as ei:
            lsh.lshmoe_workspace_bytes(*args)
        assert ei.value.status == code, (args, str(ei.value))
        assert lib.lshmoe_last_error() != b""
    out = ctypes.c_size_t(0)
    assert lib.lshmoe_workspace_bytes(16, 1024, 1, 2, 4, 64, 1, None) == lsh.LSHMOE_ERR_NULL
    assert lib.lshmoe_workspace_bytes(16, 8, 1, 2, 8, 64, 1, ctypes.byref(out)) == lsh.LSHMOE_OK   # 2^56 buckets fit


def test_entry_points_reject_bad_arguments_without_a_gpu(lib):
    p = 0x1000  # never dereferenced: every check below fails before any GPU call
    assert lib.lshmoe_hash(None, p, 16, 64, 2, 8, 1, p, None) == lsh.LSHMOE_ERR_NULL
    assert lib.lshmoe_hash(p, p, 16, 64, 2, 8, 1, None, None) == lsh.LSHMOE_ERR_NULL
    assert lib.lshmoe_hash(p, p, -1, 64, 2, 8, 1, p, None) == lsh.LSHMOE_ERR_SHAPE
    assert lib.lshmoe_hash(p, p, 16, 64, 2, 0, 1, p, None) == lsh.LSHMOE_ERR_SHAPE
    assert lib.lshmoe_hash(p, p, 16, 60, 2, 8, 1, p, None) == lsh.LSHMOE_ERR_UNSUPPORTED
    assert lib.lshmoe_hash(p, p, 16, 1024, 2, 512, 1, p, None) == lsh.LSHMOE_ERR_UNSUPPORTED   # r > 256
    assert b"256" in lib.lshmoe_last_error()
    assert lib.lshmoe_hash_sphere(p, p, None, 16, 64, 8, 1, p, None) == lsh.LSHMOE_ERR_NULL
    assert lib.lshmoe_hash_sphere(p, p, p, 16, 64, 0, 1, p, None) == lsh.LSHMOE_ERR_SHAPE
    assert lib.lshmoe_hash_sphere(p, p, p, 16, 64, 64, 1, p, None) == lsh.LSHMOE_ERR_UNSUPPORTED   # more than 63 bits
    assert lib.lshmoe_hash_sphere(p, p, p, 16, 60, 8, 1, p, None) == lsh.LSHMOE_ERR_UNSUPPORTED    # row not whole pieces
    ptrs = [p] * 7
    assert lib.lshmoe_compress(p, p, p, 16, 64, 1, 4, 2, 8, 1, *ptrs, None, 0, None) == lsh.LSHMOE_ERR_WORKSPACE
    assert lib.lshmoe_compress(p, p, p, 16, 64, 1, 4, 2, 8, 1, *ptrs, 0x1010, 1 << 30, None) == lsh.LSHMOE_ERR_WORKSPACE
    assert b"aligned" in lib.lshmoe_last_error()
    assert lib.lshmoe_compress(p, p, p, 16, 64, 1, 4, 2, 8, 1, *ptrs, 0x1000, 64, None) == lsh.LSHMOE_ERR_WORKSPACE
    assert lib.lshmoe_compress(p, None, p, 16, 64, 1, 4, 2, 8, 1, *ptrs, 0x1000, 1 << 30, None) == lsh.LSHMOE_ERR_NULL
    assert lib.lshmoe_compress(p, p, p, 16, 64, 5, 4, 2, 8, 1, *ptrs, 0x1000, 1 << 30, None) == lsh.LSHMOE_ERR_SHAPE
    assert lib.lshmoe_decompress(p, p, p, None, None, None, None, 16, 64, 1, 1, 0, p, None) == lsh.LSHMOE_ERR_NULL
    assert lib.lshmoe_decompress(p, p, p, p, None, None, None, 16, 64, 0, 1, 0, p, None) == lsh.LSHMOE_ERR_SHAPE
    assert lib.lshmoe_decompress(p, p, p, p, None, None, None, 16, 64, 1, 1, 2, p, None) == lsh.LSHMOE_ERR_UNSUPPORTED
    assert lib.lshmoe_decompress(p, p, p, p, None, None, None, 16, 63, 1, 0, 0, p, None) == lsh.LSHMOE_ERR_UNSUPPORTED
    assert lib.lshmoe_decompress(p, p, p, p, None, p, None, 16, 64, 1, 1, 0, p, None) == lsh.LSHMOE_ERR_NULL   # perm alone
    assert lib.lshmoe_decompress_combine(p, p, p, p, None, None, 16, 64, 2, 1, 0, p, None) == lsh.LSHMOE_ERR_NULL
    assert lib.lshmoe_decompress_combine(p, p, p, p, None, p, 16, 64, 2, 1, 4, p, None) == lsh.LSHMOE_ERR_UNSUPPORTED
    assert lib.lshmoe_decompress_combine(p, p, p, p, None, p, 0, 64, 2, 1, 0, p, None) == lsh.LSHMOE_ERR_SHAPE
    # hash + gate
    assert lib.lshmoe_hash_gate(p, p, None, 16, 256, 2, 8, 4, 1, p, p, None) == lsh.LSHMOE_ERR_NULL
    assert lib.lshmoe_hash_gate(p, p, p, 16, 256, 2, 8, 0, 1, p, p, None) == lsh.LSHMOE_ERR_SHAPE
    assert lib.lshmoe_hash_gate(p, p, p, 16, 256, 2, 8, 129, 1, p, p, None) == lsh.LSHMOE_ERR_UNSUPPORTED   # E > 128
    assert lib.lshmoe_hash_gate(p, p, p, 16, 256, 2, 12, 4, 1, p, p, None) == lsh.LSHMOE_ERR_UNSUPPORTED    # r % 8
    assert lib.lshmoe_hash_gate(p, p, p, 16, 264, 2, 8, 4, 1, p, p, None) == lsh.LSHMOE_ERR_UNSUPPORTED     # 528-byte rows
    # backward
    need = lsh.lshmoe_backward_workspace_bytes(16, 64, 2, lsh.LSHMOE_BF16)
    assert 0 < need <= lsh.lshmoe_workspace_bytes(16, 64, 2, 4, 2, 8, lsh.LSHMOE_BF16)   # a compress workspace is enough
    assert lib.lshmoe_decompress_backward(p, p, p, p, None, 16, 64, 2, 1, p, 0x1000, 1 << 20, None) == lsh.LSHMOE_ERR_NULL
    assert lib.lshmoe_decompress_backward(p, p, p, p, p, 16, 64, 2, 1, p, None, 0, None) == lsh.LSHMOE_ERR_WORKSPACE
    assert lib.lshmoe_decompress_backward(p, p, p, p, p, 16, 64, 2, 1, p, 0x1000, need - 1, None) == lsh.LSHMOE_ERR_WORKSPACE
    assert lib.lshmoe_decompress_backward(p, p, p, p, p, 16, 60, 2, 1, p, 0x1000, 1 << 20, None) == lsh.LSHMOE_ERR_UNSUPPORTED
    assert lib.lshmoe_decompress_backward(p, p, p, p, p, 16, 64, 0, 1, p, 0x1000, 1 << 20, None) == lsh.LSHMOE_ERR_SHAPE
    assert lib.lshmoe_compress_backward(None, p, None, p, p, 16, 64, 2, 1, 0, p, None) == lsh.LSHMOE_ERR_NULL
    assert lib.lshmoe_compress_backward(p, p, p, p, None, 16, 64, 2, 1, 0, p, None) == lsh.LSHMOE_ERR_NULL
    assert lib.lshmoe_compress_backward(p, p, p, p, p, 16, 64, 2, 1, 8, p, None) == lsh.LSHMOE_ERR_UNSUPPORTED
    assert lib.lshmoe_compress_backward(p, p, p, p, p, -3, 64, 2, 1, 0, p, None) == lsh.LSHMOE_ERR_SHAPE


def test_binding_refuses_host_tensors():
    import torch
    x = torch.zeros(4, 8)
    with pytest.raises(ValueError):
        lsh.lshmoe_hash(x, torch.zeros(1, 2, 8), torch.zeros(4, dtype=torch.int64))
