"""ctypes binding of ``liblshmoe.so``: same names as the C ABI, argument
marshalling only.  Tensors are torch CUDA(ROCm) tensors used purely as device
memory; every step of the path runs in the library's HIP kernels.  There is no
fallback: a missing library raises."""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "lib", "liblshmoe.so")

LSHMOE_OK = 0
LSHMOE_ERR_NULL = 1
LSHMOE_ERR_SHAPE = 2
LSHMOE_ERR_UNSUPPORTED = 3
LSHMOE_ERR_WORKSPACE = 4
LSHMOE_ERR_HIP = 5
LSHMOE_F32 = 0
LSHMOE_BF16 = 1
LSHMOE_FLAG_NO_RESIDUAL = 1
ABI_VERSION = 6   # of include/lshmoe.h as this binding declares it


class LshmoeError(RuntimeError):
    def __init__(self, status: int, name: str, detail: str):
        super().__init__("%s: %s" % (name, detail))
        self.status = status


_lib = None


def load_library(path: str = LIB_PATH) -> ctypes.CDLL:
    """Load the shared library (once) and declare the prototypes."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(path):
        raise ImportError(
            "%s is missing: build it with `python -m paper_2411_08446_amd.build` "
            "(there is no non-HIP fallback)" % path)
    lib = ctypes.CDLL(path)
    vp, i32, i64, u32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_uint32
    lib.lshmoe_status_string.restype = ctypes.c_char_p
    lib.lshmoe_status_string.argtypes = [ctypes.c_int]
    lib.lshmoe_last_error.restype = ctypes.c_char_p
    lib.lshmoe_last_error.argtypes = []
    lib.lshmoe_abi_version.restype = ctypes.c_int
    lib.lshmoe_abi_version.argtypes = []
    if lib.lshmoe_abi_version() != ABI_VERSION:
        raise ImportError("%s has ABI version %d, this binding expects %d: rebuild it with "
                          "`python -m paper_2411_08446_amd.build`" % (path, lib.lshmoe_abi_version(), ABI_VERSION))
    lib.lshmoe_workspace_bytes.restype = ctypes.c_int
    lib.lshmoe_workspace_bytes.argtypes = [i64, i32, i32, i32, i32, i32, ctypes.c_int, ctypes.POINTER(ctypes.c_size_t)]
    lib.lshmoe_hash.restype = ctypes.c_int
    lib.lshmoe_hash.argtypes = [vp, vp, i64, i32, i32, i32, ctypes.c_int, vp, vp]
    lib.lshmoe_hash_sphere.restype = ctypes.c_int
    lib.lshmoe_hash_sphere.argtypes = [vp, vp, vp, i64, i32, i32, ctypes.c_int, vp, vp]
    lib.lshmoe_hash_gate.restype = ctypes.c_int
    lib.lshmoe_hash_gate.argtypes = [vp, vp, vp, i64, i32, i32, i32, i32, ctypes.c_int, vp, vp, vp]
    lib.lshmoe_compress.restype = ctypes.c_int
    lib.lshmoe_compress.argtypes = [vp, vp, vp, i64, i32, i32, i32, i32, i32, ctypes.c_int,
                                    vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.lshmoe_compress_static.restype = ctypes.c_int
    lib.lshmoe_compress_static.argtypes = [vp, vp, vp, i64, i32, i32, i32, i32, i32, ctypes.c_int,
                                           vp, vp, vp, vp, vp, vp, vp, vp]
    lib.lshmoe_decompress.restype = ctypes.c_int
    lib.lshmoe_decompress.argtypes = [vp, vp, vp, vp, vp, vp, vp, i64, i32, i32, ctypes.c_int, u32, vp, vp]
    lib.lshmoe_decompress_combine.restype = ctypes.c_int
    lib.lshmoe_decompress_combine.argtypes = [vp, vp, vp, vp, vp, vp, i64, i32, i32, ctypes.c_int, u32, vp, vp]
    lib.lshmoe_decompress_combine_backward.restype = ctypes.c_int
    lib.lshmoe_decompress_combine_backward.argtypes = [vp, vp, vp, vp, vp, vp, vp, i64, i32, i32, ctypes.c_int, u32, vp, vp, vp]
    lib.lshmoe_backward_workspace_bytes.restype = ctypes.c_int
    lib.lshmoe_backward_workspace_bytes.argtypes = [i64, i32, i32, ctypes.c_int, ctypes.POINTER(ctypes.c_size_t)]
    lib.lshmoe_decompress_backward.restype = ctypes.c_int
    lib.lshmoe_decompress_backward.argtypes = [vp, vp, vp, vp, vp, i64, i32, i32, ctypes.c_int, vp, vp, ctypes.c_size_t, vp]
    lib.lshmoe_compress_backward.restype = ctypes.c_int
    lib.lshmoe_compress_backward.argtypes = [vp, vp, vp, vp, vp, i64, i32, i32, ctypes.c_int, u32, vp, vp]
    _lib = lib
    return lib


def _check(status: int) -> None:
    if status != LSHMOE_OK:
        lib = load_library()
        raise LshmoeError(status, lib.lshmoe_status_string(status).decode(), lib.lshmoe_last_error().decode())


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return LSHMOE_F32
    if t.dtype == torch.bfloat16:
        return LSHMOE_BF16
    raise TypeError("tokens must be float32 or bfloat16, got %s" % t.dtype)


def _ptr(t, dtype=None) -> int:
    if t is None:
        return 0
    if not t.is_cuda:
        raise ValueError("the library takes device pointers; got a %s tensor" % t.device)
    if not t.is_contiguous():
        raise ValueError("tensors must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise TypeError("expected %s, got %s" % (dtype, t.dtype))
    return t.data_ptr()


def _stream(stream) -> int:
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream


def lshmoe_workspace_bytes(T: int, d: int, k: int, E: int, L: int, r: int, dtype_code: int) -> int:
    out = ctypes.c_size_t(0)
    _check(load_library().lshmoe_workspace_bytes(T, d, k, E, L, r, dtype_code, ctypes.byref(out)))
    return int(out.value)


def lshmoe_hash(tokens: torch.Tensor, rot: torch.Tensor, bucket: torch.Tensor, stream=None) -> None:
    """tokens [T, d], rot [L, r, d] (same dtype) -> bucket [T] (int64 tensor holding uint64 ids)."""
    T, d = tokens.shape
    L, r, d2 = rot.shape
    if d2 != d or rot.dtype != tokens.dtype or bucket.numel() != T:
        raise ValueError("shape/dtype mismatch between tokens, rot and bucket")
    _check(load_library().lshmoe_hash(_ptr(tokens), _ptr(rot), T, d, L, r, _dtype_code(tokens),
                                      _ptr(bucket, torch.int64), _stream(stream)))


def lshmoe_hash_sphere(tokens: torch.Tensor, pivots: torch.Tensor, radius_sq: torch.Tensor, bucket: torch.Tensor,
                       stream=None) -> None:
    """tokens [T, d], pivots [B, d] (same dtype), radius_sq [B] (float32) -> bucket [T]: one bit per sphere."""
    T, d = tokens.shape
    B, d2 = pivots.shape
    if d2 != d or pivots.dtype != tokens.dtype or radius_sq.numel() != B or bucket.numel() != T:
        raise ValueError("shape/dtype mismatch between tokens, pivots, radius_sq and bucket")
    _check(load_library().lshmoe_hash_sphere(_ptr(tokens), _ptr(pivots), _ptr(radius_sq, torch.float32), T, d, B,
                                             _dtype_code(tokens), _ptr(bucket, torch.int64), _stream(stream)))


def lshmoe_hash_gate(tokens: torch.Tensor, rot: torch.Tensor, gate_w: torch.Tensor, bucket: torch.Tensor,
                     logits: torch.Tensor, stream=None) -> None:
    """As lshmoe_hash, and logits [T, E] (float32) = tokens @ gate_w.T from the same pass over the tokens."""
    T, d = tokens.shape
    L, r, d2 = rot.shape
    E = gate_w.shape[0]
    if d2 != d or gate_w.shape[1] != d or rot.dtype != tokens.dtype or gate_w.dtype != tokens.dtype \
            or bucket.numel() != T or logits.shape != (T, E):
        raise ValueError("shape/dtype mismatch between tokens, rot, gate_w, bucket and logits")
    _check(load_library().lshmoe_hash_gate(_ptr(tokens), _ptr(rot), _ptr(gate_w), T, d, L, r, E, _dtype_code(tokens),
                                           _ptr(bucket, torch.int64), _ptr(logits, torch.float32), _stream(stream)))


@dataclass
class CompressOutputs:
    """Caller-owned device buffers of lshmoe_compress, sized for S == N."""
    centroids: torch.Tensor       # [N, d]
    seg_offsets: torch.Tensor     # [N + 1] int32
    seg_expert: torch.Tensor      # [N] int32
    expert_offsets: torch.Tensor  # [E + 1] int32
    perm: torch.Tensor            # [N] int32
    seg_of: torch.Tensor          # [N] int32
    num_segments: torch.Tensor    # [1] int32
    workspace: torch.Tensor       # uint8

    @staticmethod
    def allocate(T: int, d: int, k: int, E: int, L: int, r: int, dtype: torch.dtype, device="cuda") -> "CompressOutputs":
        N = T * k
        code = LSHMOE_F32 if dtype == torch.float32 else LSHMOE_BF16
        i32 = dict(dtype=torch.int32, device=device)
        ws = lshmoe_workspace_bytes(T, d, k, E, L, r, code)
        return CompressOutputs(
            centroids=torch.empty((N, d), dtype=dtype, device=device),
            seg_offsets=torch.empty(N + 1, **i32), seg_expert=torch.empty(N, **i32),
            expert_offsets=torch.empty(E + 1, **i32), perm=torch.empty(N, **i32), seg_of=torch.empty(N, **i32),
            num_segments=torch.empty(1, **i32),
            workspace=torch.empty(ws + 256, dtype=torch.uint8, device=device))


def _aligned_ws(ws: torch.Tensor):
    base = ws.data_ptr()
    pad = (-base) % 256
    return base + pad, ws.numel() - pad


def lshmoe_compress(tokens: torch.Tensor, expert: torch.Tensor, bucket: torch.Tensor, E: int, L: int, r: int,
                    out: CompressOutputs, stream=None) -> None:
    T, d = tokens.shape
    k = expert.shape[1]
    if expert.shape[0] != T or bucket.numel() != T:
        raise ValueError("expert must be [T, k] and bucket [T]")
    N = T * k
    if (out.centroids.shape != (N, d) or out.centroids.dtype != tokens.dtype or out.seg_offsets.numel() != N + 1
            or out.seg_expert.numel() != N or out.expert_offsets.numel() != E + 1 or out.perm.numel() != N
            or out.seg_of.numel() != N or out.num_segments.numel() != 1):
        raise ValueError("output buffers do not match T, k, d, E")
    ws_ptr, ws_bytes = _aligned_ws(out.workspace)
    i32 = torch.int32
    _check(load_library().lshmoe_compress(
        _ptr(tokens), _ptr(expert, i32), _ptr(bucket, torch.int64), T, d, k, E, L, r, _dtype_code(tokens),
        _ptr(out.centroids), _ptr(out.seg_offsets, i32), _ptr(out.seg_expert, i32), _ptr(out.expert_offsets, i32),
        _ptr(out.perm, i32), _ptr(out.seg_of, i32), _ptr(out.num_segments, i32), ws_ptr, ws_bytes, _stream(stream)))


def lshmoe_compress_static(tokens: torch.Tensor, expert: torch.Tensor, bucket: torch.Tensor, E: int, L: int, r: int,
                           out: CompressOutputs, stream=None) -> None:
    """lshmoe_compress on the library's built-in scratch: out.workspace is not used and nothing is allocated."""
    T, d = tokens.shape
    k = expert.shape[1]
    if expert.shape[0] != T or bucket.numel() != T:
        raise ValueError("expert must be [T, k] and bucket [T]")
    N = T * k
    if (out.centroids.shape != (N, d) or out.centroids.dtype != tokens.dtype or out.seg_offsets.numel() != N + 1
            or out.seg_expert.numel() != N or out.expert_offsets.numel() != E + 1 or out.perm.numel() != N
            or out.seg_of.numel() != N or out.num_segments.numel() != 1):
        raise ValueError("output buffers do not match T, k, d, E")
    i32 = torch.int32
    _check(load_library().lshmoe_compress_static(
        _ptr(tokens), _ptr(expert, i32), _ptr(bucket, torch.int64), T, d, k, E, L, r, _dtype_code(tokens),
        _ptr(out.centroids), _ptr(out.seg_offsets, i32), _ptr(out.seg_expert, i32), _ptr(out.expert_offsets, i32),
        _ptr(out.perm, i32), _ptr(out.seg_of, i32), _ptr(out.num_segments, i32), _stream(stream)))


def lshmoe_decompress(tokens: torch.Tensor, centroids: torch.Tensor, expert_out: torch.Tensor, seg_of: torch.Tensor,
                      seg_offsets, k: int, out: torch.Tensor, flags: int = 0, stream=None, perm=None,
                      num_segments=None) -> None:
    T, d = tokens.shape
    if out.numel() != T * k * d or out.dtype != tokens.dtype or seg_of.numel() != T * k:
        raise ValueError("out must hold [T, k, d] elements of the token dtype and seg_of N entries")
    if centroids.dtype != tokens.dtype or expert_out.dtype != tokens.dtype:
        raise TypeError("centroids and expert_out must have the token dtype")
    if perm is not None and perm.numel() != T * k:
        raise ValueError("perm must have T*k entries")
    _check(load_library().lshmoe_decompress(
        _ptr(tokens), _ptr(centroids), _ptr(expert_out), _ptr(seg_of, torch.int32),
        _ptr(seg_offsets, torch.int32), _ptr(perm, torch.int32), _ptr(num_segments, torch.int32),
        T, d, k, _dtype_code(tokens), flags, _ptr(out), _stream(stream)))


def lshmoe_decompress_combine(tokens: torch.Tensor, centroids: torch.Tensor, expert_out: torch.Tensor,
                              seg_of: torch.Tensor, seg_offsets, gate_weight: torch.Tensor, out: torch.Tensor,
                              flags: int = 0, stream=None) -> None:
    """out [T, d] = sum_j gate_weight[t, j] * restored row of assignment (t, j)."""
    T, d = tokens.shape
    k = gate_weight.shape[1]
    if gate_weight.shape[0] != T or seg_of.numel() != T * k or out.shape != (T, d) or out.dtype != tokens.dtype:
        raise ValueError("gate_weight must be [T, k], seg_of N entries and out [T, d] of the token dtype")
    if centroids.dtype != tokens.dtype or expert_out.dtype != tokens.dtype:
        raise TypeError("centroids and expert_out must have the token dtype")
    _check(load_library().lshmoe_decompress_combine(
        _ptr(tokens), _ptr(centroids), _ptr(expert_out), _ptr(seg_of, torch.int32),
        _ptr(seg_offsets, torch.int32), _ptr(gate_weight, torch.float32), T, d, k, _dtype_code(tokens), flags,
        _ptr(out), _stream(stream)))


def lshmoe_decompress_combine_backward(tokens: torch.Tensor, centroids: torch.Tensor, expert_out: torch.Tensor,
                                       seg_of: torch.Tensor, seg_offsets, gate_weight: torch.Tensor,
                                       grad_out: torch.Tensor, grad_gate_weight: torch.Tensor, grad_rows: torch.Tensor,
                                       flags: int = 0, stream=None) -> None:
    """grad_out [T, d] -> grad_gate_weight [T, k] (binary32) and grad_rows [T, k, d] = w[t, j] * grad_out[t]."""
    T, d = tokens.shape
    k = gate_weight.shape[1]
    if (gate_weight.shape[0] != T or seg_of.numel() != T * k or grad_out.shape != (T, d) or grad_out.dtype != tokens.dtype
            or grad_gate_weight.shape != (T, k) or grad_rows.numel() != T * k * d or grad_rows.dtype != tokens.dtype):
        raise ValueError("gate_weight and grad_gate_weight must be [T, k], grad_out [T, d] and grad_rows [T, k, d]")
    if centroids.dtype != tokens.dtype or expert_out.dtype != tokens.dtype:
        raise TypeError("centroids and expert_out must have the token dtype")
    _check(load_library().lshmoe_decompress_combine_backward(
        _ptr(tokens), _ptr(centroids), _ptr(expert_out), _ptr(seg_of, torch.int32), _ptr(seg_offsets, torch.int32),
        _ptr(gate_weight, torch.float32), _ptr(grad_out), T, d, k, _dtype_code(tokens), flags,
        _ptr(grad_gate_weight, torch.float32), _ptr(grad_rows), _stream(stream)))


def lshmoe_backward_workspace_bytes(T: int, d: int, k: int, dtype_code: int) -> int:
    out = ctypes.c_size_t(0)
    _check(load_library().lshmoe_backward_workspace_bytes(T, d, k, dtype_code, ctypes.byref(out)))
    return int(out.value)


def lshmoe_decompress_backward(grad_out: torch.Tensor, perm: torch.Tensor, seg_offsets: torch.Tensor,
                               seg_of: torch.Tensor, num_segments: torch.Tensor, grad_expert_out: torch.Tensor,
                               workspace: torch.Tensor, stream=None) -> None:
    """grad_out [T, k, d] -> grad_expert_out [N, d] (rows 0..S-1): per-cluster sums of the output gradient."""
    T, k, d = grad_out.shape
    N = T * k
    if perm.numel() != N or seg_of.numel() != N or seg_offsets.numel() < 2 or grad_expert_out.shape != (N, d) \
            or grad_expert_out.dtype != grad_out.dtype:
        raise ValueError("perm and seg_of must have N entries and grad_expert_out be [N, d] of the gradient dtype")
    ws_ptr, ws_bytes = _aligned_ws(workspace)
    i32 = torch.int32
    _check(load_library().lshmoe_decompress_backward(
        _ptr(grad_out), _ptr(perm, i32), _ptr(seg_offsets, i32), _ptr(seg_of, i32), _ptr(num_segments, i32),
        T, d, k, _dtype_code(grad_out), _ptr(grad_expert_out), ws_ptr, ws_bytes, _stream(stream)))


def lshmoe_compress_backward(grad_out, grad_centroids: torch.Tensor, grad_expert_out, seg_of: torch.Tensor,
                             seg_offsets: torch.Tensor, k: int, grad_tokens: torch.Tensor, flags: int = 0,
                             stream=None) -> None:
    """grad_tokens [T, d] = sum_j grad_out[a] + (grad_centroids[s] - grad_expert_out[s]) / n_s."""
    T, d = grad_tokens.shape
    if seg_of.numel() != T * k or grad_centroids.dtype != grad_tokens.dtype:
        raise ValueError("seg_of must have T*k entries and the gradients the dtype of grad_tokens")
    for g in (grad_out, grad_expert_out):
        if g is not None and g.dtype != grad_tokens.dtype:
            raise TypeError("gradients must share one dtype")
    _check(load_library().lshmoe_compress_backward(
        _ptr(grad_out), _ptr(grad_centroids), _ptr(grad_expert_out), _ptr(seg_of, torch.int32),
        _ptr(seg_offsets, torch.int32), T, d, k, _dtype_code(grad_tokens), flags, _ptr(grad_tokens), _stream(stream)))
