"""numpy front-end of the plain-C oracle (``cnr_oracle.c``).

TEST INFRASTRUCTURE ONLY.  Argument marshalling and nothing else: every value comes out of the C
file next to this one, which states the passages of the paper it follows.  The shared object is
compiled with gcc on first use (``-O2 -ffp-contract=off``, no fast-math, so each fp32 operation
is rounded once, exactly as the C source spells it).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import threading

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "cnr_oracle.c")
_LIB = os.path.join(_HERE, "libcnr_oracle.so")
_CFLAGS = ["-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared", "-pthread"]

RANGE_MINMAX = 0
RANGE_GREEDY = 1
RANGE_SYMMETRIC = 2

_lock = threading.Lock()
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle's shared object (always when ``force``, else only when stale)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", *_CFLAGS, "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    with _lock:
        if _lib is not None:
            return _lib
        lib = ctypes.CDLL(build())
        u64, u32, i32, f32, f64, vp = (ctypes.c_uint64, ctypes.c_uint32, ctypes.c_int,
                                       ctypes.c_float, ctypes.c_double, ctypes.c_void_p)
        lib.cnro_bitmap_words.restype = u64
        lib.cnro_bitmap_words.argtypes = [u64]
        lib.cnro_clear.restype = None
        lib.cnro_clear.argtypes = [vp, u64]
        lib.cnro_mark_touched.restype = u64
        lib.cnro_mark_touched.argtypes = [vp, u64, vp, u64, i32]
        lib.cnro_compact_dirty.restype = u64
        lib.cnro_compact_dirty.argtypes = [vp, u64, vp, u64]
        lib.cnro_quantize_rows.restype = i32
        lib.cnro_quantize_rows.argtypes = [vp, u32, vp, u64, i32, i32, u32, f32,
                                           vp, vp, vp, vp, vp, i32]
        lib.cnro_greedy_iterations.restype = u32
        lib.cnro_greedy_iterations.argtypes = [u32, f32]
        lib.cnro_fq_sq_error.restype = f64
        lib.cnro_fq_sq_error.argtypes = [vp, u32, f32, f32, i32]
        lib.cnro_packed_row_bytes.restype = u64
        lib.cnro_packed_row_bytes.argtypes = [u32, i32]
        lib.cnro_pack.restype = i32
        lib.cnro_pack.argtypes = [vp, u64, u32, i32, vp]
        lib.cnro_unpack.restype = i32
        lib.cnro_unpack.argtypes = [vp, u64, u32, i32, vp]
        lib.cnro_dequantize.restype = None
        lib.cnro_dequantize.argtypes = [vp, vp, vp, u64, u32, vp]
        lib.cnro_restore_rows.restype = i32
        lib.cnro_restore_rows.argtypes = [vp, u64, u32, vp, u64, i32, vp, vp, vp, i32]
        lib.cnro_row_l2.restype = f64
        lib.cnro_row_l2.argtypes = [vp, vp, u64, u32, vp]
        lib.cnro_full_checkpoint_due.restype = i32
        lib.cnro_full_checkpoint_due.argtypes = [vp, u32]
        _lib = lib
        return lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


# ------------------------------------------------------------------------------- tracking

def bitmap_words(n_rows: int) -> int:
    return int(_load().cnro_bitmap_words(n_rows))


def new_bitmap(n_rows: int) -> np.ndarray:
    return np.zeros(bitmap_words(n_rows), dtype=np.uint32)


def clear(bitmap: np.ndarray, n_rows: int) -> None:
    assert bitmap.dtype == np.uint32 and bitmap.flags.c_contiguous
    assert bitmap.size >= bitmap_words(n_rows)
    _load().cnro_clear(_ptr(bitmap), n_rows)


def mark_touched(bitmap: np.ndarray, n_rows: int, indices: np.ndarray) -> int:
    """ORs the looked-up rows into ``bitmap`` in place; returns the number of skipped indices."""
    assert bitmap.dtype == np.uint32 and bitmap.flags.c_contiguous
    assert bitmap.size >= bitmap_words(n_rows)
    if indices.dtype == np.int64:
        is64 = 1
    elif indices.dtype == np.int32:
        is64 = 0
    else:
        raise TypeError("indices must be int32 or int64")
    idx = np.ascontiguousarray(indices).reshape(-1)
    return int(_load().cnro_mark_touched(_ptr(bitmap), n_rows, _ptr(idx), idx.size, is64))


def compact_dirty(bitmap: np.ndarray, n_rows: int, capacity: int | None = None):
    """Returns (row_ids[:min(count, capacity)], count)."""
    assert bitmap.dtype == np.uint32 and bitmap.flags.c_contiguous
    assert bitmap.size >= bitmap_words(n_rows)
    cap = n_rows if capacity is None else int(capacity)
    ids = np.empty(cap, dtype=np.uint32)
    n = int(_load().cnro_compact_dirty(_ptr(bitmap), n_rows, _ptr(ids), cap))
    return ids[:min(n, cap)].copy(), n


# ------------------------------------------------------------------------------- quantize

def greedy_iterations(num_bins: int, ratio: float) -> int:
    return int(_load().cnro_greedy_iterations(num_bins, ratio))


def fq_sq_error(x: np.ndarray, lo: float, hi: float, bits: int) -> float:
    x = _c(x, np.float32).reshape(-1)
    return float(_load().cnro_fq_sq_error(_ptr(x), x.size, np.float32(lo), np.float32(hi), bits))


def quantize_rows(table: np.ndarray, row_ids: np.ndarray | None, bits: int,
                  mode: int = RANGE_MINMAX, num_bins: int = 0, ratio: float = 1.0,
                  n_threads: int = 1, want_codes: bool = True) -> dict:
    """Quantizes rows ``row_ids`` (all rows when None) of the fp32 ``table`` [rows, dim].

    Returns a dict with ``scale``, ``bias``, ``row_min``, ``row_max`` (fp32 [n]) and ``codes``
    (uint8 [n, dim], one code per byte; omitted when ``want_codes`` is false).
    """
    assert table.dtype == np.float32 and table.ndim == 2 and table.flags.c_contiguous
    n_rows, dim = table.shape
    if row_ids is None:
        n, ids = n_rows, None
    else:
        ids = _c(row_ids, np.uint32).reshape(-1)
        n = ids.size
        if n and int(ids.max()) >= n_rows:
            raise IndexError("row id outside the table")
    out = {k: np.empty(n, dtype=np.float32) for k in ("scale", "bias", "row_min", "row_max")}
    codes = np.empty((n, dim), dtype=np.uint8) if want_codes else None
    rc = _load().cnro_quantize_rows(_ptr(table), dim, _ptr(ids), n, bits, mode, num_bins,
                                    np.float32(ratio), _ptr(out["scale"]), _ptr(out["bias"]),
                                    _ptr(out["row_min"]), _ptr(out["row_max"]), _ptr(codes),
                                    n_threads)
    if rc != 0:
        raise ValueError("cnro_quantize_rows rejected its arguments (rc=%d)" % rc)
    if want_codes:
        out["codes"] = codes
    return out


def packed_row_bytes(dim: int, bits: int) -> int:
    return int(_load().cnro_packed_row_bytes(dim, bits))


def pack(codes: np.ndarray, bits: int) -> np.ndarray:
    codes = _c(codes, np.uint8)
    assert codes.ndim == 2
    n, dim = codes.shape
    packed = np.empty((n, packed_row_bytes(dim, bits)), dtype=np.uint8)
    if _load().cnro_pack(_ptr(codes), n, dim, bits, _ptr(packed)) != 0:
        raise ValueError("cnro_pack rejected its arguments")
    return packed


def unpack(packed: np.ndarray, dim: int, bits: int) -> np.ndarray:
    packed = _c(packed, np.uint8)
    n = packed.size // max(1, packed_row_bytes(dim, bits))
    codes = np.empty((n, dim), dtype=np.uint8)
    if _load().cnro_unpack(_ptr(packed), n, dim, bits, _ptr(codes)) != 0:
        raise ValueError("cnro_unpack rejected its arguments")
    return codes


# ------------------------------------------------------------------------------- restore

def dequantize(codes: np.ndarray, scale: np.ndarray, bias: np.ndarray) -> np.ndarray:
    codes = _c(codes, np.uint8)
    n, dim = codes.shape
    scale, bias = _c(scale, np.float32), _c(bias, np.float32)
    assert scale.size == n and bias.size == n
    out = np.empty((n, dim), dtype=np.float32)
    _load().cnro_dequantize(_ptr(codes), _ptr(scale), _ptr(bias), n, dim, _ptr(out))
    return out


def restore_rows(table: np.ndarray, row_ids: np.ndarray | None, bits: int, packed: np.ndarray,
                 scale: np.ndarray, bias: np.ndarray, n_threads: int = 1) -> None:
    """De-quantizes the packed rows and writes them over rows ``row_ids`` of ``table`` in place."""
    assert table.dtype == np.float32 and table.ndim == 2 and table.flags.c_contiguous
    n_rows, dim = table.shape
    scale, bias = _c(scale, np.float32), _c(bias, np.float32)
    packed = _c(packed, np.uint8)
    ids = None if row_ids is None else _c(row_ids, np.uint32).reshape(-1)
    n = scale.size
    assert bias.size == n and (ids is None or ids.size == n)
    assert packed.size == n * packed_row_bytes(dim, bits)
    rc = _load().cnro_restore_rows(_ptr(table), n_rows, dim, _ptr(ids), n, bits, _ptr(packed),
                                   _ptr(scale), _ptr(bias), n_threads)
    if rc != 0:
        raise ValueError("cnro_restore_rows rejected its arguments (rc=%d)" % rc)


def row_l2(a: np.ndarray, b: np.ndarray):
    """Per-row l2 distance (fp64) and its mean."""
    a, b = _c(a, np.float32), _c(b, np.float32)
    assert a.shape == b.shape and a.ndim == 2
    err = np.empty(a.shape[0], dtype=np.float64)
    mean = float(_load().cnro_row_l2(_ptr(a), _ptr(b), a.shape[0], a.shape[1], _ptr(err)))
    return err, mean


# ------------------------------------------------------------------------------- policy

def full_checkpoint_due(sizes) -> bool:
    """Intermittent-incremental predictor: ``sizes`` = [S_1, ..., S_i] as fractions of a full one."""
    s = _c(np.asarray(sizes, dtype=np.float64), np.float64).reshape(-1)
    return bool(_load().cnro_full_checkpoint_due(_ptr(s), s.size))



def select_bits(expected_resumes: int, observed_resumes: int = 0) -> int:
    """Dynamic bit-width selection (Section 6.2.1): how often a job may resume from a checkpoint of
    each width before the accuracy loss passes the threshold, narrowest sufficient width first;
    8 bits once more resumes have happened than were expected."""
    resumes_tolerated = ((2, 1), (3, 3), (4, 20))
    if observed_resumes > expected_resumes:
        return 8
    for bits, tolerated in resumes_tolerated:
        if expected_resumes <= tolerated:
            return bits
    return 8
