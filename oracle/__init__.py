"""CPU oracle of the PacTrain compression path (test infrastructure only).

Thin ctypes wrapper around ``pac_oracle.cpp``: numpy arrays in, numpy arrays out.
Nothing here is used by the product; the GPU library shares no code with it.
Only tests, the smoke check and the benchmark's CPU-baseline leg import this package.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pac_oracle.cpp")
_SRC_MT = os.path.join(_HERE, "pac_oracle_mt.cpp")   # the all-core leg of the benchmark's CPU baseline
_LIB = os.path.join(_HERE, "libpac_oracle.so")

F32 = 0
BF16 = 1


def build(force: bool = False) -> str:
    """Compile the oracle with the host compiler (no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < max(os.path.getmtime(_SRC), os.path.getmtime(_SRC_MT)):
        cmd = ["g++", "-std=c++17", "-O2", "-fno-fast-math", "-ffp-contract=off", "-fPIC", "-shared", "-fopenmp",
               "-o", _LIB, _SRC, _SRC_MT]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        u64, u32, i32, vp = ctypes.c_uint64, ctypes.c_uint32, ctypes.c_int, ctypes.c_void_p
        lib.orc_keep_count.restype = u64
        lib.orc_keep_count.argtypes = [u64, ctypes.c_double]
        lib.orc_build_mask.restype = i32
        lib.orc_build_mask.argtypes = [vp, u64, vp, u32, vp, vp, vp, vp]
        lib.orc_compress.restype = u64
        lib.orc_compress.argtypes = [vp, i32, u64, vp, vp, u64]
        lib.orc_reduce.restype = None
        lib.orc_reduce.argtypes = [vp, u32, i32, u64, vp]
        lib.orc_decompress.restype = u64
        lib.orc_decompress.argtypes = [vp, i32, u64, vp, vp, u64]
        lib.orc_f32_to_bf16.restype = None
        lib.orc_f32_to_bf16.argtypes = [vp, vp, u64]
        lib.orc_mask_from_nonzero.restype = u64
        lib.orc_mask_from_nonzero.argtypes = [vp, i32, u64, vp, vp]
        lib.orc_mask_diff.restype = u64
        lib.orc_mask_diff.argtypes = [vp, vp, u64]
        lib.orc_philox4x32_10.restype = None
        lib.orc_philox4x32_10.argtypes = [vp, vp, vp]
        lib.orc_absmax.restype = ctypes.c_float
        lib.orc_absmax.argtypes = [vp, i32, u64, vp]
        lib.orc_ternarize.restype = None
        lib.orc_ternarize.argtypes = [vp, i32, u64, ctypes.c_float, u64, u64, vp]
        lib.orc_ternary_reduce.restype = None
        lib.orc_ternary_reduce.argtypes = [vp, u32, u64, ctypes.c_float, i32, vp]
        lib.orc_decompress_update.restype = u64
        lib.orc_decompress_update.argtypes = [vp, i32, u64, vp, ctypes.c_float, vp, u64]
        lib.orc_mt_threads.restype = i32
        lib.orc_mt_threads.argtypes = []
        lib.orc_build_mask_mt.restype = i32
        lib.orc_build_mask_mt.argtypes = [vp, u64, vp, u32, vp, vp, vp, vp]
        lib.orc_compress_mt.restype = None
        lib.orc_compress_mt.argtypes = [vp, i32, u64, vp, vp, vp]
        lib.orc_reduce_mt.restype = None
        lib.orc_reduce_mt.argtypes = [vp, u32, i32, u64, vp]
        lib.orc_decompress_mt.restype = None
        lib.orc_decompress_mt.argtypes = [vp, i32, vp, vp, vp, u64]
        _lib = lib
    return _lib


def _ptr(a: np.ndarray) -> int:
    return a.ctypes.data


def _elem_dtype(dtype: int):
    return np.float32 if dtype == F32 else np.uint16


def keep_count(n: int, sparsity: float) -> int:
    return int(_load().orc_keep_count(int(n), float(sparsity)))


def mask_words(n: int) -> int:
    return (int(n) + 63) // 64


def build_mask(weights: np.ndarray, seg_offsets=None, sparsity=0.0):
    """Return (mask uint64[ceil(n/64)], prefix uint32[ceil(n/64)], nnz)."""
    w = np.ascontiguousarray(weights, dtype=np.float32).reshape(-1)
    n = w.size
    if seg_offsets is None:
        seg_offsets = [0, n]
    off = np.ascontiguousarray(seg_offsets, dtype=np.uint64)
    nseg = off.size - 1
    sp = np.ascontiguousarray(np.broadcast_to(np.asarray(sparsity, dtype=np.float64), (nseg,)))
    words = mask_words(n)
    mask = np.zeros(max(words, 1), dtype=np.uint64)[:words]
    prefix = np.zeros(max(words, 1), dtype=np.uint32)[:words]
    nnz = ctypes.c_uint64(0)
    rc = _load().orc_build_mask(_ptr(w), n, _ptr(off), nseg, _ptr(sp), _ptr(mask), _ptr(prefix),
                                ctypes.addressof(nnz))
    if rc != 0:
        raise ValueError("orc_build_mask: bad arguments")
    return mask, prefix, int(nnz.value)


def compress(grad: np.ndarray, mask: np.ndarray, nnz: int, dtype: int = F32) -> np.ndarray:
    g = np.ascontiguousarray(grad, dtype=_elem_dtype(dtype)).reshape(-1)
    out = np.empty(nnz, dtype=_elem_dtype(dtype))
    got = _load().orc_compress(_ptr(g), dtype, g.size, _ptr(np.ascontiguousarray(mask)), _ptr(out), nnz)
    if got != nnz:
        raise ValueError(f"mask holds {got} set bits, caller said {nnz}")
    return out


def reduce_local(bufs, dtype: int = F32) -> np.ndarray:
    arrs = [np.ascontiguousarray(b, dtype=_elem_dtype(dtype)).reshape(-1) for b in bufs]
    nnz = arrs[0].size
    assert all(a.size == nnz for a in arrs)
    ptrs = (ctypes.c_void_p * len(arrs))(*[_ptr(a) for a in arrs])
    out = np.empty(nnz, dtype=_elem_dtype(dtype))
    _load().orc_reduce(ctypes.addressof(ptrs), len(arrs), dtype, nnz, _ptr(out))
    return out


def decompress(compact: np.ndarray, mask: np.ndarray, n: int, dtype: int = F32) -> np.ndarray:
    c = np.ascontiguousarray(compact, dtype=_elem_dtype(dtype)).reshape(-1)
    out = np.empty(n, dtype=_elem_dtype(dtype))
    used = _load().orc_decompress(_ptr(c), dtype, c.size, _ptr(np.ascontiguousarray(mask)), _ptr(out), n)
    if used != c.size:
        raise ValueError(f"mask holds {used} set bits, compact buffer has {c.size}")
    return out


def f32_to_bf16(x: np.ndarray) -> np.ndarray:
    a = np.ascontiguousarray(x, dtype=np.float32).reshape(-1)
    out = np.empty(a.size, dtype=np.uint16)
    _load().orc_f32_to_bf16(_ptr(a), _ptr(out), a.size)
    return out


# ---- the all-core leg (pac_oracle_mt.cpp): same results, OpenMP threads over 64-element words ----

def mt_threads() -> int:
    """Threads the *_mt functions use: the cores the process may run on, capped by OMP_NUM_THREADS."""
    return int(_load().orc_mt_threads())


def build_mask_mt(weights: np.ndarray, seg_offsets=None, sparsity=0.0):
    w = np.ascontiguousarray(weights, dtype=np.float32).reshape(-1)
    n = w.size
    if seg_offsets is None:
        seg_offsets = [0, n]
    off = np.ascontiguousarray(seg_offsets, dtype=np.uint64)
    nseg = off.size - 1
    sp = np.ascontiguousarray(np.broadcast_to(np.asarray(sparsity, dtype=np.float64), (nseg,)))
    words = mask_words(n)
    mask = np.zeros(max(words, 1), dtype=np.uint64)[:words]
    prefix = np.zeros(max(words, 1), dtype=np.uint32)[:words]
    nnz = ctypes.c_uint64(0)
    rc = _load().orc_build_mask_mt(_ptr(w), n, _ptr(off), nseg, _ptr(sp), _ptr(mask), _ptr(prefix),
                                   ctypes.addressof(nnz))
    if rc != 0:
        raise ValueError("orc_build_mask_mt: bad arguments")
    return mask, prefix, int(nnz.value)


def compress_mt(grad: np.ndarray, mask: np.ndarray, prefix: np.ndarray, nnz: int, dtype: int = F32) -> np.ndarray:
    g = np.ascontiguousarray(grad, dtype=_elem_dtype(dtype)).reshape(-1)
    out = np.empty(nnz, dtype=_elem_dtype(dtype))
    _load().orc_compress_mt(_ptr(g), dtype, g.size, _ptr(np.ascontiguousarray(mask)),
                            _ptr(np.ascontiguousarray(prefix)), _ptr(out))
    return out


def reduce_local_mt(bufs, dtype: int = F32) -> np.ndarray:
    arrs = [np.ascontiguousarray(b, dtype=_elem_dtype(dtype)).reshape(-1) for b in bufs]
    nnz = arrs[0].size
    assert all(a.size == nnz for a in arrs)
    ptrs = (ctypes.c_void_p * len(arrs))(*[_ptr(a) for a in arrs])
    out = np.empty(nnz, dtype=_elem_dtype(dtype))
    _load().orc_reduce_mt(ctypes.addressof(ptrs), len(arrs), dtype, nnz, _ptr(out))
    return out


def decompress_mt(compact: np.ndarray, mask: np.ndarray, prefix: np.ndarray, n: int, dtype: int = F32) -> np.ndarray:
    c = np.ascontiguousarray(compact, dtype=_elem_dtype(dtype)).reshape(-1)
    out = np.empty(n, dtype=_elem_dtype(dtype))
    _load().orc_decompress_mt(_ptr(c), dtype, _ptr(np.ascontiguousarray(mask)), _ptr(np.ascontiguousarray(prefix)),
                              _ptr(out), n)
    return out


# ---- around the hot path: Mask Tracker (Sec. III-B) and the weight update (Eq. 1) -----------

def mask_from_nonzero(values: np.ndarray, dtype: int = F32):
    """Mask of the non-zero elements (Eq. 2's Weight != 0).  Returns (mask, prefix, nnz)."""
    v = np.ascontiguousarray(values, dtype=_elem_dtype(dtype)).reshape(-1)
    words = mask_words(v.size)
    mask = np.zeros(max(words, 1), dtype=np.uint64)[:words]
    prefix = np.zeros(max(words, 1), dtype=np.uint32)[:words]
    nnz = _load().orc_mask_from_nonzero(_ptr(v), dtype, v.size, _ptr(mask), _ptr(prefix))
    return mask, prefix, int(nnz)


def mask_diff(a: np.ndarray, b: np.ndarray, n: int) -> int:
    """Number of positions below n at which two bitmasks differ."""
    a = np.ascontiguousarray(a, dtype=np.uint64)
    b = np.ascontiguousarray(b, dtype=np.uint64)
    assert a.size >= mask_words(n) and b.size >= mask_words(n)
    return int(_load().orc_mask_diff(_ptr(a), _ptr(b), int(n)))


class MaskTracker:
    """The Mask Tracker's bookkeeping (Sec. III-B; Alg. 1, mask-update step and stability test):
    keep the previous iteration's mask, compare, and call the pattern stable once it has stayed
    unchanged for `patience` consecutive comparisons.  The paper asks for several unchanged iterations without
    a number: `patience` is the caller's.  The first mask ever seen, and a mask of another length,
    count as a change."""

    def __init__(self, patience: int):
        assert patience >= 1
        self.patience = int(patience)
        self.prev = None
        self.prev_n = None
        self.unchanged = 0

    def update(self, mask: np.ndarray, n: int):
        """Returns (unchanged_comparisons, stable)."""
        same = self.prev is not None and self.prev_n == n and mask_diff(self.prev, mask, n) == 0
        self.unchanged = self.unchanged + 1 if same else 0
        self.prev = np.array(mask, dtype=np.uint64, copy=True)
        self.prev_n = n
        return self.unchanged, self.unchanged >= self.patience


def decompress_update(compact: np.ndarray, mask: np.ndarray, weights: np.ndarray, alpha: float,
                      dtype: int = F32) -> np.ndarray:
    """x <- x - alpha * g on kept weights (g = next summed compact value), +0 on pruned ones.  Returns the new
    weights; the input array is left alone."""
    c = np.ascontiguousarray(compact, dtype=_elem_dtype(dtype)).reshape(-1)
    w = np.array(weights, dtype=np.float32, copy=True).reshape(-1)
    used = _load().orc_decompress_update(_ptr(c), dtype, c.size, _ptr(np.ascontiguousarray(mask)),
                                         ctypes.c_float(alpha), _ptr(w), w.size)
    if used != c.size:
        raise ValueError(f"mask holds {used} set bits, compact buffer has {c.size}")
    return w


# ---- ternary payload (Sec. III-D) -----------------------------------------------------------

def philox4x32_10(counter, key) -> np.ndarray:
    c = np.ascontiguousarray(counter, dtype=np.uint32)
    k = np.ascontiguousarray(key, dtype=np.uint32)
    out = np.empty(4, dtype=np.uint32)
    _load().orc_philox4x32_10(_ptr(c), _ptr(k), _ptr(out))
    return out


def absmax(values: np.ndarray, dtype: int = F32, start=None) -> float:
    v = np.ascontiguousarray(values, dtype=_elem_dtype(dtype)).reshape(-1)
    st = None if start is None else np.array([start], dtype=np.float32)
    return float(_load().orc_absmax(_ptr(v), dtype, v.size, None if st is None else _ptr(st)))


def ternarize(values: np.ndarray, scale: float, seed: int, stream: int, dtype: int = F32) -> np.ndarray:
    """Packed 2-bit codes (0 = 0, 1 = +1, 2 = -1), four elements per byte, element j at bits 2*(j%4)."""
    v = np.ascontiguousarray(values, dtype=_elem_dtype(dtype)).reshape(-1)
    out = np.empty((v.size + 3) // 4, dtype=np.uint8)
    _load().orc_ternarize(_ptr(v), dtype, v.size, ctypes.c_float(scale), int(seed), int(stream), _ptr(out))
    return out


def ternary_reduce(packed, count: int, scale: float, out_dtype: int = F32) -> np.ndarray:
    arrs = [np.ascontiguousarray(p, dtype=np.uint8).reshape(-1) for p in packed]
    assert all(a.size >= (count + 3) // 4 for a in arrs)
    ptrs = (ctypes.c_void_p * len(arrs))(*[_ptr(a) for a in arrs])
    out = np.empty(count, dtype=_elem_dtype(out_dtype))
    _load().orc_ternary_reduce(ctypes.addressof(ptrs), len(arrs), count, ctypes.c_float(scale), out_dtype, _ptr(out))
    return out
