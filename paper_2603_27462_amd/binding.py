"""ctypes binding for librsr.so: same names as include/rsr.h, marshalling only.

Tensors are PyTorch CUDA(ROCm) tensors used purely as device memory; streams
are ``torch.cuda.Stream`` objects (or None for torch's current stream).
"""
from __future__ import annotations

import ctypes
import os
import warnings
from typing import Optional

import numpy as np

from . import build as _build

RSR_BINARY, RSR_TERNARY_2PASS, RSR_TERNARY_FUSED, RSR_DENSE_TERNARY_P2 = 0, 1, 2, 3
RSR_F32, RSR_BF16 = 0, 1

# every symbol include/rsr.h declares
exported_symbols = [
    "rsr_preprocess", "rsr_matvec", "rsr_matvec_ex", "rsr_destroy", "rsr_last_error",
    "rsr_error_string", "rsr_get_perm", "rsr_get_offsets", "rsr_get_packed",
    "rsr_preprocess_transposed", "rsr_serialized_size", "rsr_serialize", "rsr_deserialize",
    "rsr_num_blocks", "rsr_block_height", "rsr_num_patterns", "rsr_num_passes",
    "rsr_algorithmic_bytes",
    "rsr_kernel_name", "rsr_preprocess_into", "rsr_launch_shape", "rsr_probe_empty", "rsr_probe_read",
    "rsr_preprocess_stacked", "rsr_matvec_stacked", "rsr_num_layers",
]


class RsrError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__("%s failed: %s (code %d)" % (where, rsr_error_string(code), code))


_lib = None


def load_library(path: Optional[str] = None) -> ctypes.CDLL:
    """Load librsr.so (building it first only if no built library exists)."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    path = path or _build.LIB_PATH
    if not os.path.exists(path):
        _build.build_library()
    elif path == _build.LIB_PATH:
        newer = _build.sources_newer_than_library()
        if newer:
            warnings.warn("librsr.so is older than %s: it does not contain the current sources; "
                          "rebuild with paper_2603_27462_amd.build.build_library()" % ", ".join(newer))
    # PyTorch ships its own HIP runtime; it has to be in the process first so that
    # librsr binds to the same one the tensors were allocated with.
    import torch  # noqa: F401
    lib = ctypes.CDLL(path)
    i64, vp, ci, cf = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int, ctypes.c_float
    lib.rsr_preprocess.restype = vp
    lib.rsr_preprocess.argtypes = [vp, i64, i64, ci, ci]
    lib.rsr_matvec.restype = ci
    lib.rsr_matvec.argtypes = [vp, vp, vp, vp]
    lib.rsr_matvec_ex.restype = ci
    lib.rsr_matvec_ex.argtypes = [vp, vp, ci, cf, vp, ci, i64, i64, vp]
    lib.rsr_destroy.restype = None
    lib.rsr_destroy.argtypes = [vp]
    lib.rsr_last_error.restype = ci
    lib.rsr_last_error.argtypes = []
    lib.rsr_error_string.restype = ctypes.c_char_p
    lib.rsr_error_string.argtypes = [ci]
    for name in ("rsr_get_perm", "rsr_get_offsets"):
        getattr(lib, name).restype = ci
        getattr(lib, name).argtypes = [vp, ci, vp]
    lib.rsr_get_packed.restype = ci
    lib.rsr_get_packed.argtypes = [vp, vp]
    for name in ("rsr_num_blocks", "rsr_num_patterns"):
        getattr(lib, name).restype = i64
        getattr(lib, name).argtypes = [vp]
    lib.rsr_num_passes.restype = ci
    lib.rsr_num_passes.argtypes = [vp]
    lib.rsr_preprocess_transposed.restype = vp
    lib.rsr_preprocess_transposed.argtypes = [vp, i64, i64, ci, ci]
    lib.rsr_preprocess_into.restype = ci
    lib.rsr_preprocess_into.argtypes = [vp, vp]
    lib.rsr_launch_shape.restype = ci
    lib.rsr_launch_shape.argtypes = [vp, ci, vp, vp, vp]
    lib.rsr_probe_empty.restype = ci
    lib.rsr_probe_empty.argtypes = [ci, ci, ci, vp]
    lib.rsr_probe_read.restype = ci
    lib.rsr_probe_read.argtypes = [vp, i64, ci, ci, vp, vp]
    lib.rsr_preprocess_stacked.restype = vp
    lib.rsr_preprocess_stacked.argtypes = [vp, vp, ci, i64, ci, ci]
    lib.rsr_matvec_stacked.restype = ci
    lib.rsr_matvec_stacked.argtypes = [vp, vp, ci, vp, vp, vp]
    lib.rsr_num_layers.restype = ci
    lib.rsr_num_layers.argtypes = [vp]
    lib.rsr_serialized_size.restype = i64
    lib.rsr_serialized_size.argtypes = [vp]
    lib.rsr_serialize.restype = ci
    lib.rsr_serialize.argtypes = [vp, vp, i64]
    lib.rsr_deserialize.restype = vp
    lib.rsr_deserialize.argtypes = [vp, i64]
    lib.rsr_block_height.restype = ci
    lib.rsr_block_height.argtypes = [vp]
    lib.rsr_algorithmic_bytes.restype = i64
    lib.rsr_algorithmic_bytes.argtypes = [vp, ci, ci]
    lib.rsr_kernel_name.restype = ctypes.c_char_p
    lib.rsr_kernel_name.argtypes = [vp, ci]
    _lib = lib
    return lib


class Handle:
    """Owns an rsr_handle_t; freed by rsr_destroy() or garbage collection."""

    def __init__(self, ptr: int, rows: int, cols: int, k: int, kind: int):
        self.ptr, self.rows, self.cols, self.k, self.kind = ptr, rows, cols, k, kind

    def __del__(self):
        try:
            rsr_destroy(self)
        except Exception:
            pass


def _stream_ptr(stream) -> int:
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return int(s.cuda_stream)


def rsr_last_error() -> int:
    return int(load_library().rsr_last_error())


def rsr_error_string(code: int) -> str:
    return load_library().rsr_error_string(int(code)).decode()


def rsr_preprocess(M, k: int, kind: int) -> Handle:
    """M: int8 CUDA tensor [rows][cols], row-major."""
    import torch
    if not (isinstance(M, torch.Tensor) and M.is_cuda and M.dtype == torch.int8 and M.dim() == 2):
        raise TypeError("M must be a 2-D int8 CUDA tensor")
    M = M.contiguous()
    rows, cols = M.shape
    with torch.cuda.device(M.device):
        torch.cuda.current_stream().synchronize()   # M was produced on torch's stream
        ptr = load_library().rsr_preprocess(M.data_ptr(), rows, cols, int(k), int(kind))
    if not ptr:
        raise RsrError(rsr_last_error(), "rsr_preprocess")
    return Handle(ptr, rows, cols, int(load_library().rsr_block_height(ptr)), int(kind))


def rsr_preprocess_transposed(M, k: int, kind: int) -> Handle:
    """Handle of M^T (M: int8 CUDA tensor [rows][cols]): multiplies vectors of length rows."""
    import torch
    if not (isinstance(M, torch.Tensor) and M.is_cuda and M.dtype == torch.int8 and M.dim() == 2):
        raise TypeError("M must be a 2-D int8 CUDA tensor")
    M = M.contiguous()
    rows, cols = M.shape
    with torch.cuda.device(M.device):
        torch.cuda.current_stream().synchronize()
        ptr = load_library().rsr_preprocess_transposed(M.data_ptr(), rows, cols, int(k), int(kind))
    if not ptr:
        raise RsrError(rsr_last_error(), "rsr_preprocess_transposed")
    return Handle(ptr, cols, rows, int(load_library().rsr_block_height(ptr)), int(kind))


def rsr_preprocess_stacked(Ms, k: int, kind: int) -> Handle:
    """Ms: int8 CUDA tensors [rows_i][cols] that share cols (sibling layers with one input)."""
    import torch
    Ms = [M.contiguous() for M in Ms]
    if not Ms or any(not (M.is_cuda and M.dtype == torch.int8 and M.dim() == 2 and
                          M.shape[1] == Ms[0].shape[1]) for M in Ms):
        raise TypeError("Ms must be 2-D int8 CUDA tensors with the same number of columns")
    n, cols = len(Ms), Ms[0].shape[1]
    ptrs = (ctypes.c_void_p * n)(*[M.data_ptr() for M in Ms])
    rows = (ctypes.c_int64 * n)(*[M.shape[0] for M in Ms])
    with torch.cuda.device(Ms[0].device):
        torch.cuda.current_stream().synchronize()
        ptr = load_library().rsr_preprocess_stacked(ptrs, rows, n, cols, int(k), int(kind))
    if not ptr:
        raise RsrError(rsr_last_error(), "rsr_preprocess_stacked")
    h = Handle(ptr, sum(M.shape[0] for M in Ms), cols, int(load_library().rsr_block_height(ptr)), int(kind))
    h.layer_rows = [M.shape[0] for M in Ms]
    return h


def rsr_matvec_stacked(h: Handle, v, scales=None, outs=None, stream=None):
    """One launch for all layers of a stacked handle; returns the list of float32 outputs."""
    import torch
    n = len(h.layer_rows)
    if not (v.is_cuda and v.dim() == 1 and v.numel() == h.cols and v.is_contiguous()):
        raise TypeError("v must be a contiguous CUDA vector of length cols")
    if outs is None:
        outs = [torch.empty(r, dtype=torch.float32, device=v.device) for r in h.layer_rows]
    optr = (ctypes.c_void_p * n)(*[o.data_ptr() for o in outs])
    sc = (ctypes.c_float * n)(*[float(x) for x in scales]) if scales is not None else None
    rc = load_library().rsr_matvec_stacked(h.ptr, v.data_ptr(), _dtype_code(v), sc, optr, _stream_ptr(stream))
    if rc:
        raise RsrError(rc, "rsr_matvec_stacked")
    return outs


def rsr_preprocess_into(h: Handle, M) -> None:
    """Replace the matrix of h by M (same shape) without allocating device memory."""
    import torch
    if not (isinstance(M, torch.Tensor) and M.is_cuda and M.dtype == torch.int8 and
            tuple(M.shape) == (h.rows, h.cols) and M.is_contiguous()):
        raise TypeError("M must be a contiguous int8 CUDA tensor [rows][cols] of the handle's shape")
    with torch.cuda.device(M.device):
        torch.cuda.current_stream().synchronize()
        rc = load_library().rsr_preprocess_into(h.ptr, M.data_ptr())
    if rc:
        raise RsrError(rc, "rsr_preprocess_into")


def rsr_serialize(h: Handle) -> np.ndarray:
    """The handle as a uint8 array (host)."""
    lib = load_library()
    n = int(lib.rsr_serialized_size(h.ptr))
    if n < 0:
        raise RsrError(rsr_last_error(), "rsr_serialized_size")
    buf = np.empty(n, dtype=np.uint8)
    rc = lib.rsr_serialize(h.ptr, buf.ctypes.data, n)
    if rc:
        raise RsrError(rc, "rsr_serialize")
    return buf


def rsr_deserialize(buf) -> Handle:
    """A new handle on the current device from the bytes rsr_serialize returned."""
    buf = np.ascontiguousarray(np.frombuffer(buf, dtype=np.uint8) if not isinstance(buf, np.ndarray) else buf,
                               dtype=np.uint8)
    lib = load_library()
    ptr = lib.rsr_deserialize(buf.ctypes.data, buf.size)
    if not ptr:
        raise RsrError(rsr_last_error(), "rsr_deserialize")
    # geometry from the header: kind, k at int32 words 2 and 3; rows, cols at bytes 40 and 48
    words = buf[:64].view(np.int32)
    rows, cols = (int(x) for x in buf[40:56].view(np.int64))
    return Handle(ptr, rows, cols, int(lib.rsr_block_height(ptr)), int(words[2]))


def rsr_destroy(h: Handle) -> None:
    if h.ptr:
        load_library().rsr_destroy(h.ptr)
        h.ptr = 0


def _dtype_code(v) -> int:
    import torch
    if v.dtype == torch.float32:
        return RSR_F32
    if v.dtype == torch.bfloat16:
        return RSR_BF16
    raise TypeError("v must be float32 or bfloat16")


def rsr_matvec(h: Handle, v, out=None, stream=None):
    """out = M v for one float32 vector."""
    import torch
    if not (v.is_cuda and v.dtype == torch.float32 and v.is_contiguous() and v.numel() == h.cols):
        raise TypeError("v must be a contiguous float32 CUDA tensor of length cols")
    if out is None:
        out = torch.empty(h.rows, dtype=torch.float32, device=v.device)
    rc = load_library().rsr_matvec(h.ptr, v.data_ptr(), out.data_ptr(), _stream_ptr(stream))
    if rc:
        raise RsrError(rc, "rsr_matvec")
    return out


def rsr_matvec_ex(h: Handle, v, scale: float = 1.0, out=None, stream=None):
    """v: [cols] or [batch][cols], float32 or bfloat16; returns float32 [rows] or [batch][rows]."""
    import torch
    if not v.is_cuda or v.dim() not in (1, 2) or v.shape[-1] != h.cols or v.stride(-1) != 1:
        raise TypeError("v must be a CUDA tensor [cols] or [batch][cols] with unit inner stride")
    batch = 1 if v.dim() == 1 else v.shape[0]
    ldv = h.cols if v.dim() == 1 else v.stride(0)
    if out is None:
        shape = (h.rows,) if v.dim() == 1 else (batch, h.rows)
        out = torch.empty(shape, dtype=torch.float32, device=v.device)
    ldo = h.rows if out.dim() == 1 else out.stride(0)
    rc = load_library().rsr_matvec_ex(h.ptr, v.data_ptr(), _dtype_code(v), float(scale),
                                      out.data_ptr(), batch, ldv, ldo, _stream_ptr(stream))
    if rc:
        raise RsrError(rc, "rsr_matvec_ex")
    return out


def rsr_num_blocks(h: Handle) -> int:
    return int(load_library().rsr_num_blocks(h.ptr))


def rsr_num_patterns(h: Handle) -> int:
    return int(load_library().rsr_num_patterns(h.ptr))


def rsr_block_height(h: Handle) -> int:
    return int(load_library().rsr_block_height(h.ptr))


def rsr_num_passes(h: Handle) -> int:
    return int(load_library().rsr_num_passes(h.ptr))


def rsr_get_perm(h: Handle, pass_: int = 0) -> np.ndarray:
    pi = np.empty((rsr_num_blocks(h), h.cols), dtype=np.uint32)
    rc = load_library().rsr_get_perm(h.ptr, pass_, pi.ctypes.data)
    if rc:
        raise RsrError(rc, "rsr_get_perm")
    return pi


def rsr_get_offsets(h: Handle, pass_: int = 0) -> np.ndarray:
    off = np.empty((rsr_num_blocks(h), rsr_num_patterns(h) + 1), dtype=np.uint32)
    rc = load_library().rsr_get_offsets(h.ptr, pass_, off.ctypes.data)
    if rc:
        raise RsrError(rc, "rsr_get_offsets")
    return off


def rsr_get_packed(h: Handle) -> np.ndarray:
    packed = np.empty((h.rows, (h.cols + 3) // 4), dtype=np.uint8)
    rc = load_library().rsr_get_packed(h.ptr, packed.ctypes.data)
    if rc:
        raise RsrError(rc, "rsr_get_packed")
    return packed


def rsr_algorithmic_bytes(h: Handle, v_dtype: int = RSR_F32, batch: int = 1) -> int:
    n = int(load_library().rsr_algorithmic_bytes(h.ptr, v_dtype, batch))
    if n < 0:
        raise RsrError(rsr_last_error(), "rsr_algorithmic_bytes")
    return n


def rsr_launch_shape(h: Handle, v_dtype: int = RSR_F32):
    """(workgroups per vector, threads per workgroup, LDS bytes per workgroup) of the multiply kernel."""
    wg, th, lds = ctypes.c_int(), ctypes.c_int(), ctypes.c_int()
    rc = load_library().rsr_launch_shape(h.ptr, v_dtype, ctypes.byref(wg), ctypes.byref(th), ctypes.byref(lds))
    if rc:
        raise RsrError(rc, "rsr_launch_shape")
    return wg.value, th.value, lds.value


def rsr_probe_empty(workgroups: int, threads: int, lds_bytes: int, stream=None) -> None:
    rc = load_library().rsr_probe_empty(int(workgroups), int(threads), int(lds_bytes), _stream_ptr(stream))
    if rc:
        raise RsrError(rc, "rsr_probe_empty")


def rsr_probe_read(src, nbytes: int, workgroups: int, threads: int, stream=None) -> None:
    """src: a CUDA tensor of at least nbytes bytes, read once and discarded."""
    if src.numel() * src.element_size() < nbytes:
        raise ValueError("src is smaller than nbytes")
    rc = load_library().rsr_probe_read(src.data_ptr(), int(nbytes), int(workgroups), int(threads), None,
                                       _stream_ptr(stream))
    if rc:
        raise RsrError(rc, "rsr_probe_read")


def rsr_kernel_name(h: Handle, v_dtype: int = RSR_F32) -> str:
    s = load_library().rsr_kernel_name(h.ptr, v_dtype)
    if s is None:
        raise RsrError(rsr_last_error(), "rsr_kernel_name")
    return s.decode()
