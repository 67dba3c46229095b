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
PAC_TABLE_SLOTS = 4

# bits of the device status word (pac_device_status)
PAC_DEV_SCAN_STALLED = 0x01
PAC_DEV_COUNT_MISMATCH = 0x02
PAC_DEV_META_MISMATCH = 0x04
PAC_DEV_RETRY_TAKEN = 0x100
PAC_DEV_SLOW_PATH = 0x200
PAC_DEV_ERROR_MASK = 0xFF

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
    lib.pac_step_fused.restype = i32
    lib.pac_step_fused.argtypes = [vp, ctypes.POINTER(vp), u32, i32, u64, vp, vp, vp, u64, vp]
    lib.pac_debug_set_candidate_capacity.restype = i32
    lib.pac_debug_set_candidate_capacity.argtypes = [vp, u64]
    lib.pac_debug_set_scan_spin_limit.restype = i32
    lib.pac_debug_set_scan_spin_limit.argtypes = [vp, u32]
    lib.pac_device_status.restype = i32
    lib.pac_device_status.argtypes = [vp, vp, ctypes.POINTER(u32), ctypes.c_int, vp]
    lib.pac_mask_from_nonzero.restype = i32
    lib.pac_mask_from_nonzero.argtypes = [vp, vp, i32, u64, vp, vp, vp, vp]
    lib.pac_mask_from_nonzero_noalloc.restype = i32
    lib.pac_mask_from_nonzero_noalloc.argtypes = [vp, i32, u64, vp, vp, vp, vp, vp]
    lib.pac_mask_equal.restype = i32
    lib.pac_mask_equal.argtypes = [vp, vp, vp, u64, vp, vp]
    lib.pac_tracker_create.restype = i32
    lib.pac_tracker_create.argtypes = [vp, u64, u32, ctypes.POINTER(vp)]
    lib.pac_tracker_update.restype = i32
    lib.pac_tracker_update.argtypes = [vp, vp, u64, vp, vp]
    lib.pac_tracker_destroy.restype = i32
    lib.pac_tracker_destroy.argtypes = [vp]
    lib.pac_absmax.restype = i32
    lib.pac_absmax.argtypes = [vp, vp, i32, u64, ctypes.c_int, vp, vp]
    lib.pac_ternarize.restype = i32
    lib.pac_ternarize.argtypes = [vp, vp, i32, u64, vp, u64, u64, vp, vp]
    lib.pac_ternary_reduce_local.restype = i32
    lib.pac_ternary_reduce_local.argtypes = [vp, ctypes.POINTER(vp), u32, u64, vp, i32, vp, vp]
    lib.pac_decompress_update.restype = i32
    lib.pac_decompress_update.argtypes = [vp, vp, i32, u64, vp, vp, ctypes.c_float, vp, u64, vp]
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


def pac_debug_set_scan_spin_limit(ctx, polls: int) -> None:
    _check(ctx, load_library().pac_debug_set_scan_spin_limit(ctx, int(polls)))


def pac_device_status(ctx, flags_out: Optional[torch.Tensor] = None, to_host: bool = True, clear: bool = False,
                      stream=None) -> Optional[int]:
    """flags_out: device int32 [1] that receives the status word in stream order.  With to_host the call
    waits for the stream and returns the word; otherwise it returns None."""
    if flags_out is not None and (flags_out.dtype != torch.int32 or flags_out.numel() < 1):
        raise TypeError("flags_out must be an int32 tensor")
    host = ctypes.c_uint32(0)
    st = load_library().pac_device_status(ctx, _dev_ptr(flags_out), ctypes.byref(host) if to_host else None,
                                          1 if clear else 0, _stream_ptr(stream))
    _check(ctx, st)
    return int(host.value) if to_host else None


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


def pac_step_fused(ctx, grads: Sequence[torch.Tensor], mask: torch.Tensor, prefix: torch.Tensor, reduced: torch.Tensor,
                   nnz: int, stream=None) -> None:
    """Gather and sum the W dense gradients in one pass: reduced[:nnz] as pac_reduce_local over W pac_compress outputs."""
    dt = _dtype_code(reduced)
    W = len(grads)
    n = grads[0].numel() if W else 0
    for g in grads:
        if g.dtype != reduced.dtype:
            raise TypeError("all gradients and the reduced buffer must share one dtype")
        if g.numel() != n:
            raise ValueError("gradients must have equal lengths")
    if reduced.numel() < nnz:
        raise ValueError("reduced buffer too short")
    ptrs = (ctypes.c_void_p * max(W, 1))(*[_dev_ptr(g) for g in grads])
    st = load_library().pac_step_fused(ctx, ptrs, W, dt, n, _dev_ptr(mask), _dev_ptr(prefix), _dev_ptr(reduced),
                                       int(nnz), _stream_ptr(stream))
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


def pac_mask_from_nonzero(ctx, values: torch.Tensor, mask: torch.Tensor, prefix: torch.Tensor,
                          nnz_out: Optional[torch.Tensor] = None, stream=None) -> None:
    """values fp32 or bf16 [n]; nnz_out: device int64 [1] (the count stays on the device)."""
    dt = _dtype_code(values)
    n = values.numel()
    words = (n + 63) // 64
    if mask.dtype != torch.int64 or prefix.dtype != torch.int32:
        raise TypeError("mask must be int64 and prefix int32")
    if mask.numel() < words or prefix.numel() < words:
        raise ValueError("mask/prefix too short")
    if nnz_out is not None and (nnz_out.dtype != torch.int64 or nnz_out.numel() < 1):
        raise TypeError("nnz_out must be an int64 tensor")
    st = load_library().pac_mask_from_nonzero(ctx, _dev_ptr(values) if n else 0, dt, n, _dev_ptr(mask) if n else 0,
                                              _dev_ptr(prefix) if n else 0, _dev_ptr(nnz_out), _stream_ptr(stream))
    _check(ctx, st)


def pac_mask_from_nonzero_noalloc(values: torch.Tensor, mask: torch.Tensor, prefix: torch.Tensor,
                                  nnz_out: Optional[torch.Tensor] = None, flags_out: Optional[torch.Tensor] = None,
                                  stream=None) -> None:
    """pac_mask_from_nonzero without a context and without any allocation, on the current device.
    nnz_out: device int64 [1]; flags_out: device int32 [1]."""
    dt = _dtype_code(values)
    n = values.numel()
    words = (n + 63) // 64
    if mask.dtype != torch.int64 or prefix.dtype != torch.int32:
        raise TypeError("mask must be int64 and prefix int32")
    if mask.numel() < words or prefix.numel() < words:
        raise ValueError("mask/prefix too short")
    if nnz_out is not None and (nnz_out.dtype != torch.int64 or nnz_out.numel() < 1):
        raise TypeError("nnz_out must be an int64 tensor")
    if flags_out is not None and (flags_out.dtype != torch.int32 or flags_out.numel() < 1):
        raise TypeError("flags_out must be an int32 tensor")
    st = load_library().pac_mask_from_nonzero_noalloc(_dev_ptr(values) if n else 0, dt, n, _dev_ptr(mask) if n else 0,
                                                      _dev_ptr(prefix) if n else 0, _dev_ptr(nnz_out),
                                                      _dev_ptr(flags_out), _stream_ptr(stream))
    _check(None, st)


def pac_mask_equal(ctx, mask_a: torch.Tensor, mask_b: torch.Tensor, n: int, diff_out: torch.Tensor,
                   stream=None) -> None:
    """diff_out: device int64 [1], receives the number of differing positions below n."""
    words = (int(n) + 63) // 64
    if mask_a.dtype != torch.int64 or mask_b.dtype != torch.int64 or diff_out.dtype != torch.int64:
        raise TypeError("masks and diff_out must be int64")
    if mask_a.numel() < words or mask_b.numel() < words or diff_out.numel() < 1:
        raise ValueError("tensor too short")
    st = load_library().pac_mask_equal(ctx, _dev_ptr(mask_a) if n else 0, _dev_ptr(mask_b) if n else 0, int(n),
                                       _dev_ptr(diff_out), _stream_ptr(stream))
    _check(ctx, st)


def pac_tracker_create(ctx, max_elems: int, patience: int):
    out = ctypes.c_void_p()
    _check(ctx, load_library().pac_tracker_create(ctx, int(max_elems), int(patience), ctypes.byref(out)))
    return out


def pac_tracker_update(ctx, tracker, mask: torch.Tensor, n: int, state_out: Optional[torch.Tensor] = None,
                       stream=None) -> None:
    """state_out: device int32 [2], receives {unchanged comparisons, stable}."""
    if mask.dtype != torch.int64:
        raise TypeError("mask must be int64")
    if mask.numel() < (int(n) + 63) // 64:
        raise ValueError("mask too short")
    if state_out is not None and (state_out.dtype != torch.int32 or state_out.numel() < 2):
        raise TypeError("state_out must be an int32 tensor of 2 elements")
    st = load_library().pac_tracker_update(tracker, _dev_ptr(mask) if n else 0, int(n), _dev_ptr(state_out),
                                           _stream_ptr(stream))
    _check(ctx, st)


def pac_tracker_destroy(tracker) -> None:
    load_library().pac_tracker_destroy(tracker)


def pac_decompress_update(ctx, reduced: torch.Tensor, mask: torch.Tensor, prefix: torch.Tensor, alpha: float,
                          weights: torch.Tensor, nnz: int, stream=None) -> None:
    """weights fp32 [n], updated in place."""
    dt = _dtype_code(reduced)
    if weights.dtype != torch.float32:
        raise TypeError("weights must be float32")
    if reduced.numel() < nnz:
        raise ValueError("reduced buffer too short")
    st = load_library().pac_decompress_update(ctx, _dev_ptr(reduced), dt, int(nnz), _dev_ptr(mask), _dev_ptr(prefix),
                                              ctypes.c_float(alpha), _dev_ptr(weights), weights.numel(),
                                              _stream_ptr(stream))
    _check(ctx, st)


def pac_absmax(ctx, values: torch.Tensor, scale: torch.Tensor, accumulate: bool = False, count: Optional[int] = None,
               stream=None) -> None:
    """scale: device float32 [1]."""
    dt = _dtype_code(values)
    if scale.dtype != torch.float32 or scale.numel() < 1:
        raise TypeError("scale must be a float32 tensor")
    n = values.numel() if count is None else int(count)
    st = load_library().pac_absmax(ctx, _dev_ptr(values) if n else 0, dt, n, 1 if accumulate else 0, _dev_ptr(scale),
                                   _stream_ptr(stream))
    _check(ctx, st)


def pac_ternarize(ctx, values: torch.Tensor, scale: torch.Tensor, seed: int, stream_id: int, packed: torch.Tensor,
                  count: Optional[int] = None, stream=None) -> None:
    """packed: device uint8 [ceil(count/4)], 4-byte aligned."""
    dt = _dtype_code(values)
    n = values.numel() if count is None else int(count)
    if packed.dtype != torch.uint8 or packed.numel() < (n + 3) // 4:
        raise ValueError("packed must be uint8 with ceil(count/4) elements")
    if scale.dtype != torch.float32:
        raise TypeError("scale must be float32")
    st = load_library().pac_ternarize(ctx, _dev_ptr(values), dt, n, _dev_ptr(scale), int(seed) & (2**64 - 1),
                                      int(stream_id) & (2**64 - 1), _dev_ptr(packed), _stream_ptr(stream))
    _check(ctx, st)


def pac_ternary_reduce_local(ctx, packed: Sequence[torch.Tensor], scale: torch.Tensor, out: torch.Tensor, count: int,
                             stream=None) -> None:
    dt = _dtype_code(out)
    W = len(packed)
    for p in packed:
        if p.dtype != torch.uint8 or p.numel() < (count + 3) // 4:
            raise ValueError("packed buffers must be uint8 with ceil(count/4) elements")
    if out.numel() < count:
        raise ValueError("output buffer too short")
    ptrs = (ctypes.c_void_p * max(W, 1))(*[_dev_ptr(p) for p in packed])
    st = load_library().pac_ternary_reduce_local(ctx, ptrs, W, int(count), _dev_ptr(scale), dt, _dev_ptr(out),
                                                 _stream_ptr(stream))
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

    def device_status(self, clear: bool = False, stream=None) -> int:
        """The context's device status word (PAC_DEV_* bits); waits for the stream."""
        return pac_device_status(self.handle, None, True, clear, stream)

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

    def step_fused(self, grads: List[torch.Tensor], mask, prefix, nnz: int, out=None, stream=None) -> torch.Tensor:
        if out is None:
            out = torch.empty(nnz, dtype=grads[0].dtype, device=self._dev())
        pac_step_fused(self.handle, grads, mask, prefix, out, nnz, stream)
        return out

    def decompress(self, compact, mask, prefix, n, nnz: Optional[int] = None, out=None, stream=None) -> torch.Tensor:
        if nnz is None:
            nnz = compact.numel()
        if out is None:
            out = torch.empty(n, dtype=compact.dtype, device=self._dev())
        pac_decompress(self.handle, compact, mask, prefix, out, nnz, stream)
        return out

    def mask_from_nonzero(self, values, mask=None, prefix=None, nnz_out=None, stream=None):
        """Returns (mask, prefix, nnz_out); nnz_out is a device int64 tensor of one element."""
        words = (values.numel() + 63) // 64
        if mask is None:
            mask = torch.empty(words, dtype=torch.int64, device=self._dev())
        if prefix is None:
            prefix = torch.empty(words, dtype=torch.int32, device=self._dev())
        if nnz_out is None:
            nnz_out = torch.empty(1, dtype=torch.int64, device=self._dev())
        pac_mask_from_nonzero(self.handle, values, mask, prefix, nnz_out, stream)
        return mask, prefix, nnz_out

    def mask_equal(self, mask_a, mask_b, n, diff_out=None, stream=None) -> torch.Tensor:
        if diff_out is None:
            diff_out = torch.empty(1, dtype=torch.int64, device=self._dev())
        pac_mask_equal(self.handle, mask_a, mask_b, n, diff_out, stream)
        return diff_out

    def decompress_update(self, reduced, mask, prefix, alpha, weights, nnz: Optional[int] = None, stream=None):
        if nnz is None:
            nnz = reduced.numel()
        pac_decompress_update(self.handle, reduced, mask, prefix, alpha, weights, nnz, stream)
        return weights


class MaskTracker:
    """Owns one pac_tracker of a context."""

    def __init__(self, ctx: PacContext, max_elems: int, patience: int):
        self.ctx = ctx
        self.handle = pac_tracker_create(ctx.handle, max_elems, patience)

    def update(self, mask, n, state_out=None, stream=None) -> torch.Tensor:
        if state_out is None:
            state_out = torch.empty(2, dtype=torch.int32, device=self.ctx._dev())
        pac_tracker_update(self.ctx.handle, self.handle, mask, n, state_out, stream)
        return state_out

    def close(self) -> None:
        if self.handle is not None:
            pac_tracker_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
