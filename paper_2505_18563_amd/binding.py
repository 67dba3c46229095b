"""ctypes binding of libpactrain.so: same names as the C ABI, torch tensors for device memory.

Argument marshalling only.  Every step of the path runs in the library's kernels.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence, Tuple

import torch  # first: the library binds to the HIP runtime torch has already loaded

from . import build as _build

PAC_F32 = 0
PAC_BF16 = 1
PAC_MAX_WORKERS = 64

_STATUS_NAMES = {0: "PAC_OK", -1: "PAC_ERR_ARG", -2: "PAC_ERR_ALIGN", -3: "PAC_ERR_RANGE",
                 -4: "PAC_ERR_COUNT", -5: "PAC_ERR_HIP", -6: "PAC_ERR_NOMEM"}

_lib = None


class PacError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"{_STATUS_NAMES.get(status, status)}: {text}")
        self.status = status


def library_path() -> str:
    return _build.LIB


def load_library() -> ctypes.CDLL:
    """Load libpactrain.so; compile it first only if no built library exists."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_build.LIB):
        _build.build(force=True)
    lib = ctypes.CDLL(_build.LIB)
    u64, u32, i32, vp, dbl = ctypes.c_uint64, ctypes.c_uint32, ctypes.c_int32, ctypes.c_void_p, ctypes.c_double
    lib.pac_create.restype = i32
    lib.pac_create.argtypes = [ctypes.POINTER(vp), ctypes.c_int, u64, u32]
    lib.pac_destroy.restype = i32
    lib.pac_destroy.argtypes = [vp]
    lib.pac_last_error.restype = ctypes.c_char_p
    lib.pac_last_error.argtypes = [vp]
    lib.pac_keep_count.restype = u64
    lib.pac_keep_count.argtypes = [u64, dbl]
    lib.pac_mask_words.restype = u64
    lib.pac_mask_words.argtypes = [u64]
    lib.pac_build_mask.restype = i32
    lib.pac_build_mask.argtypes = [vp, vp, u64, ctypes.POINTER(u64), u32, ctypes.POINTER(dbl), vp, vp,
                                   ctypes.POINTER(u64), vp]
    lib.pac_compress.restype = i32
    lib.pac_compress.argtypes = [vp, vp, i32, u64, vp, vp, vp, u64, vp]
    lib.pac_reduce_local.restype = i32
    lib.pac_reduce_local.argtypes = [vp, ctypes.POINTER(vp), u32, i32, u64, vp, vp]
    lib.pac_decompress.restype = i32
    lib.pac_decompress.argtypes = [vp, vp, i32, u64, vp, vp, vp, u64, vp]
    lib.pac_debug_set_candidate_capacity.restype = i32
    lib.pac_debug_set_candidate_capacity.argtypes = [vp, u64]
    _lib = lib
    return lib


def _check(ctx, status: int) -> None:
    if status != 0:
        raise PacError(status, pac_last_error(ctx))


def _stream_ptr(stream: Optional[torch.cuda.Stream]) -> int:
    s = stream if stream is not None else torch.cuda.current_stream()
    return int(s.cuda_stream)


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return PAC_F32
    if t.dtype == torch.bfloat16:
        return PAC_BF16
    raise TypeError(f"gradient payload must be float32 or bfloat16, got {t.dtype}")


def _dev_ptr(t: Optional[torch.Tensor]) -> int:
    if t is None:
        return 0
    if not t.is_cuda:
        raise ValueError("device tensor expected")
    if not t.is_contiguous():
        raise ValueError("contiguous tensor expected")
    return int(t.data_ptr())


# ------------------------------------------------------------------ functions named as in the ABI
def pac_keep_count(n: int, sparsity: float) -> int:
    return int(load_library().pac_keep_count(int(n), float(sparsity)))


def pac_mask_words(n: int) -> int:
    return int(load_library().pac_mask_words(int(n)))


def pac_last_error(ctx) -> str:
    return load_library().pac_last_error(ctx).decode()


def pac_create(device: int, max_elems: int, max_segments: int = 1):
    lib = load_library()
    out = ctypes.c_void_p()
    st = lib.pac_create(ctypes.byref(out), int(device), int(max_elems), int(max_segments))
    if st != 0:
        raise PacError(st, pac_last_error(None))
    return out


def pac_destroy(ctx) -> None:
    load_library().pac_destroy(ctx)


def pac_debug_set_candidate_capacity(ctx, capacity: int) -> None:
    _check(ctx, load_library().pac_debug_set_candidate_capacity(ctx, int(capacity)))


def pac_build_mask(ctx, weights: torch.Tensor, seg_offsets: Sequence[int], sparsity: Sequence[float],
                   mask: torch.Tensor, prefix: torch.Tensor, stream=None) -> int:
    """weights fp32 [n]; mask int64 [ceil(n/64)] (bit patterns of uint64); prefix int32 [ceil(n/64)].
    Returns nnz = sum of the scopes' keep counts."""
    if weights.dtype != torch.float32:
        raise TypeError("weights must be float32")
    if mask.dtype != torch.int64 or prefix.dtype != torch.int32:
        raise TypeError("mask must be int64 and prefix int32")
    n = weights.numel()
    words = (n + 63) // 64
    if mask.numel() < words or prefix.numel() < words:
        raise ValueError("mask/prefix too short")
    nseg = len(seg_offsets) - 1
    off = (ctypes.c_uint64 * (nseg + 1))(*[int(x) for x in seg_offsets])
    sp = (ctypes.c_double * nseg)(*[float(x) for x in sparsity])
    nnz = ctypes.c_uint64(0)
    st = load_library().pac_build_mask(ctx, _dev_ptr(weights) if n else 0, n, off, nseg, sp,
                                       _dev_ptr(mask) if n else 0, _dev_ptr(prefix) if n else 0,
                                       ctypes.byref(nnz), _stream_ptr(stream))
    _check(ctx, st)
    return int(nnz.value)


def pac_compress(ctx, grad: torch.Tensor, mask: torch.Tensor, prefix: torch.Tensor, compact: torch.Tensor,
                 nnz: int, stream=None) -> None:
    dt = _dtype_code(grad)
    if compact.dtype != grad.dtype:
        raise TypeError("compact buffer must have the gradient's dtype")
    if compact.numel() < nnz:
        raise ValueError("compact buffer too short")
    st = load_library().pac_compress(ctx, _dev_ptr(grad), dt, grad.numel(), _dev_ptr(mask), _dev_ptr(prefix),
                                     _dev_ptr(compact), int(nnz), _stream_ptr(stream))
    _check(ctx, st)


def pac_reduce_local(ctx, bufs: Sequence[torch.Tensor], out: torch.Tensor, nnz: int, stream=None) -> None:
    dt = _dtype_code(out)
    W = len(bufs)
    for b in bufs:
        if b.dtype != out.dtype:
            raise TypeError("all buffers must share one dtype")
        if b.numel() < nnz:
            raise ValueError("compact buffer too short")
    if out.numel() < nnz:
        raise ValueError("output buffer too short")
    ptrs = (ctypes.c_void_p * max(W, 1))(*[_dev_ptr(b) for b in bufs])
    st = load_library().pac_reduce_local(ctx, ptrs, W, dt, int(nnz), _dev_ptr(out), _stream_ptr(stream))
    _check(ctx, st)


def pac_decompress(ctx, compact: torch.Tensor, mask: torch.Tensor, prefix: torch.Tensor, dense: torch.Tensor,
                   nnz: int, stream=None) -> None:
    dt = _dtype_code(dense)
    if compact.dtype != dense.dtype:
        raise TypeError("compact buffer must have the output's dtype")
    if compact.numel() < nnz:
        raise ValueError("compact buffer too short")
    st = load_library().pac_decompress(ctx, _dev_ptr(compact), dt, int(nnz), _dev_ptr(mask), _dev_ptr(prefix),
                                       _dev_ptr(dense), dense.numel(), _stream_ptr(stream))
    _check(ctx, st)


# ------------------------------------------------------------------------------ convenience
class PacContext:
    """Owns one pac_ctx and allocates outputs with torch; the arithmetic stays in the library."""

    def __init__(self, max_elems: int, max_segments: int = 1, device: Optional[int] = None):
        self.device = torch.cuda.current_device() if device is None else int(device)
        self.max_elems = int(max_elems)
        self.handle = pac_create(self.device, max_elems, max_segments)

    def close(self) -> None:
        if self.handle is not None:
            pac_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    def _dev(self):
        return torch.device("cuda", self.device)

    def build_mask(self, weights: torch.Tensor, seg_offsets=None, sparsity=0.0, mask=None, prefix=None,
                   stream=None) -> Tuple[torch.Tensor, torch.Tensor, int]:
        n = weights.numel()
        if seg_offsets is None:
            seg_offsets = [0, n]
        nseg = len(seg_offsets) - 1
        if isinstance(sparsity, (int, float)):
            sparsity = [float(sparsity)] * nseg
        words = (n + 63) // 64
        if mask is None:
            mask = torch.empty(words, dtype=torch.int64, device=self._dev())
        if prefix is None:
            prefix = torch.empty(words, dtype=torch.int32, device=self._dev())
        nnz = pac_build_mask(self.handle, weights, seg_offsets, sparsity, mask, prefix, stream)
        return mask, prefix, nnz

    def compress(self, grad, mask, prefix, nnz, out=None, stream=None) -> torch.Tensor:
        if out is None:
            out = torch.empty(nnz, dtype=grad.dtype, device=self._dev())
        pac_compress(self.handle, grad, mask, prefix, out, nnz, stream)
        return out

    def reduce_local(self, bufs: List[torch.Tensor], nnz: Optional[int] = None, out=None, stream=None) -> torch.Tensor:
        if nnz is None:
            nnz = bufs[0].numel()
        if out is None:
            out = torch.empty(nnz, dtype=bufs[0].dtype, device=self._dev())
        pac_reduce_local(self.handle, bufs, out, nnz, stream)
        return out

    def decompress(self, compact, mask, prefix, n, nnz: Optional[int] = None, out=None, stream=None) -> torch.Tensor:
        if nnz is None:
            nnz = compact.numel()
        if out is None:
            out = torch.empty(n, dtype=compact.dtype, device=self._dev())
        pac_decompress(self.handle, compact, mask, prefix, out, nnz, stream)
        return out
