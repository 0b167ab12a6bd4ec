"""ctypes binding of libcnr.so: argument marshalling only.

Every function has the name and the argument order of its C declaration in ``include/cnr.h``
(which documents meaning, layout and error behaviour) and takes ``torch`` tensors that live on
the context's GPU where the C side takes device pointers.  Nothing is computed here: checks are
limited to dtype / device / contiguity of the tensors handed over, and a non-zero status is
raised as :class:`CnrError`.  There is no fallback: without the compiled library, or without a
GPU, these calls fail.
"""
from __future__ import annotations

import ctypes
import os
import threading

import torch

from . import build as _build

CNR_OK = 0
CNR_E_INVALID, CNR_E_BITS, CNR_E_DIM, CNR_E_ALIGN = 1, 2, 3, 4
CNR_E_CAPACITY, CNR_E_INDEX_RANGE, CNR_E_ROW_ID, CNR_E_HIP, CNR_E_TOO_LARGE, CNR_E_HOST_MEMORY = 5, 6, 7, 8, 9, 10
CNR_HOST_SERIAL, CNR_HOST_OVERLAP, CNR_HOST_DIRECT = 0, 1, 2
CNR_NOALLOC_MAX_ROWS = 1 << 30
CNR_IDX_I32, CNR_IDX_I64 = 0, 1
CNR_RANGE_MINMAX, CNR_RANGE_GREEDY, CNR_RANGE_SYMMETRIC = 0, 1, 2
CNR_FLAG_CAPACITY, CNR_FLAG_ROW_ID = 1, 2
CNR_MAX_DIM = 4096
CNR_MAX_BATCH = 16

# Every symbol include/cnr.h declares.
EXPORTS = (
    "cnr_create", "cnr_destroy", "cnr_bitmap_words", "cnr_packed_row_bytes", "cnr_scratch_bytes",
    "cnr_mark_scratch_bytes",
    "cnr_greedy_iterations", "cnr_clear_bitmap", "cnr_mark_touched", "cnr_compact_dirty", "cnr_compact_dirty_noalloc",
    "cnr_quantize_rows", "cnr_pack", "cnr_restore_rows", "cnr_quant_error", "cnr_poll_errors", "cnr_status_str",
    "cnr_last_hip_error", "cnr_full_checkpoint_due", "cnr_policy_init", "cnr_policy_next", "cnr_select_bits",
    "cnr_clear_bitmap_batch", "cnr_mark_touched_batch", "cnr_compact_dirty_batch", "cnr_quantize_rows_batch",
    "cnr_restore_rows_batch",
    "cnr_host_writer_device_bytes", "cnr_host_writer_create", "cnr_host_writer_destroy", "cnr_encode_to_host",
    "cnr_host_writer_wait", "cnr_restore_from_host", "cnr_select_scratch_bytes", "cnr_select_greedy_params",
)


class CnrError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s: %s (status %d)" % (where, status_str(status), status))


CNR_POLICY_ONE_SHOT, CNR_POLICY_CONSECUTIVE, CNR_POLICY_INTERMITTENT = 0, 1, 2
CNR_POLICY_MAX_HISTORY = 256


class cnr_policy(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int), ("n_history", ctypes.c_uint32),
                ("history", ctypes.c_double * CNR_POLICY_MAX_HISTORY)]


class cnr_policy_decision(ctypes.Structure):
    _fields_ = [("take_full", ctypes.c_int), ("clear_bitmap", ctypes.c_int)]


class cnr_greedy_params(ctypes.Structure):
    _fields_ = [("num_bins", ctypes.c_uint32), ("ratio", ctypes.c_float)]


class cnr_table_job(ctypes.Structure):
    """One table's buffers for the ``*_batch`` calls (field for field the C struct)."""
    _fields_ = [("table", ctypes.c_void_p), ("n_rows", ctypes.c_uint64), ("bitmap", ctypes.c_void_p),
                ("indices", ctypes.c_void_p), ("n_indices", ctypes.c_uint64), ("mark_scratch", ctypes.c_void_p),
                ("row_ids", ctypes.c_void_p), ("capacity", ctypes.c_uint64), ("n_dirty_dev", ctypes.c_void_p),
                ("compact_scratch", ctypes.c_void_p), ("scale", ctypes.c_void_p), ("bias", ctypes.c_void_p),
                ("row_min", ctypes.c_void_p), ("row_max", ctypes.c_void_p), ("codes_u8", ctypes.c_void_p),
                ("packed", ctypes.c_void_p)]


_lock = threading.Lock()
_lib = None


def ensure_built() -> str:
    """Path of a libcnr.so that matches the sources in this tree: compiles it when there is none, or
    when the one there was built from other sources (a stale library would be tested silently)."""
    if _build.is_stale():
        _build.build_lib(force=True)
    return _build.LIB


def load() -> ctypes.CDLL:
    """Loads libcnr.so, compiling it first only when no up-to-date library is there."""
    global _lib
    with _lock:
        if _lib is not None:
            return _lib
        lib = ctypes.CDLL(ensure_built())
        vp, u64, u32, i32, f32 = (ctypes.c_void_p, ctypes.c_uint64, ctypes.c_uint32, ctypes.c_int,
                                  ctypes.c_float)
        sz = ctypes.c_size_t
        sig = {
            "cnr_create": (i32, [ctypes.POINTER(vp), i32]),
            "cnr_destroy": (i32, [vp]),
            "cnr_bitmap_words": (sz, [u64]),
            "cnr_packed_row_bytes": (sz, [u32, i32]),
            "cnr_scratch_bytes": (sz, [u64]),
            "cnr_mark_scratch_bytes": (sz, [u64]),
            "cnr_greedy_iterations": (u32, [u32, f32]),
            "cnr_clear_bitmap": (i32, [vp, vp, u64, vp]),
            "cnr_mark_touched": (i32, [vp, vp, u64, vp, u64, i32, vp, vp]),
            "cnr_compact_dirty": (i32, [vp, vp, u64, vp, u64, vp, vp, vp]),
            "cnr_compact_dirty_noalloc": (i32, [vp, vp, u64, vp, u64, vp, vp]),
            "cnr_quantize_rows": (i32, [vp, vp, u64, u32, vp, vp, u64, i32, i32,
                                        ctypes.POINTER(cnr_greedy_params), vp, vp, vp, vp, vp, vp, vp]),
            "cnr_pack": (i32, [vp, vp, vp, u64, u32, i32, vp, vp]),
            "cnr_restore_rows": (i32, [vp, vp, u64, u32, vp, vp, u64, i32, vp, vp, vp, vp]),
            "cnr_quant_error": (i32, [vp, vp, u64, u32, vp, vp, u64, i32, vp, vp, vp, vp, vp, vp]),
            "cnr_poll_errors": (i32, [vp, vp, ctypes.POINTER(u64), ctypes.POINTER(u32)]),
            "cnr_status_str": (ctypes.c_char_p, [i32]),
            "cnr_last_hip_error": (i32, [vp]),
            "cnr_full_checkpoint_due": (i32, [ctypes.POINTER(ctypes.c_double), u32]),
            "cnr_policy_init": (i32, [ctypes.POINTER(cnr_policy), i32]),
            "cnr_policy_next": (cnr_policy_decision, [ctypes.POINTER(cnr_policy), ctypes.c_double]),
            "cnr_select_bits": (i32, [u32, u32]),
            "cnr_clear_bitmap_batch": (i32, [vp, ctypes.POINTER(cnr_table_job), u32, vp]),
            "cnr_mark_touched_batch": (i32, [vp, ctypes.POINTER(cnr_table_job), u32, i32, vp]),
            "cnr_compact_dirty_batch": (i32, [vp, ctypes.POINTER(cnr_table_job), u32, vp]),
            "cnr_quantize_rows_batch": (i32, [vp, ctypes.POINTER(cnr_table_job), u32, u32, i32, i32,
                                              ctypes.POINTER(cnr_greedy_params), vp]),
            "cnr_restore_rows_batch": (i32, [vp, ctypes.POINTER(cnr_table_job), u32, u32, i32, vp]),
            "cnr_host_writer_device_bytes": (sz, [u32, i32, u64]),
            "cnr_host_writer_create": (i32, [vp, u32, i32, u64, ctypes.POINTER(vp)]),
            "cnr_host_writer_destroy": (i32, [vp]),
            "cnr_encode_to_host": (i32, [vp, vp, u64, vp, u64, i32, ctypes.POINTER(cnr_greedy_params),
                                         vp, vp, vp, vp, i32, vp]),
            "cnr_host_writer_wait": (i32, [vp, vp]),
            "cnr_restore_from_host": (i32, [vp, vp, u64, vp, vp, vp, vp, u64, i32, vp]),
            "cnr_select_scratch_bytes": (sz, [u64, u32, i32]),
            "cnr_select_greedy_params": (i32, [vp, vp, u64, u32, vp, u64, i32, ctypes.POINTER(u32), u32,
                                               ctypes.POINTER(f32), u32, ctypes.c_double, vp,
                                               ctypes.POINTER(cnr_greedy_params), ctypes.POINTER(ctypes.c_double), vp]),
        }
        for name, (res, args) in sig.items():
            fn = getattr(lib, name)
            fn.restype, fn.argtypes = res, args
        _lib = lib
        return lib


def status_str(status: int) -> str:
    return load().cnr_status_str(int(status)).decode()


def _check(status: int, where: str) -> None:
    if status != CNR_OK:
        raise CnrError(status, where)


def _dev(t, dtype, name: str):
    """Device pointer of a contiguous tensor of the given dtype (None passes through as NULL)."""
    if t is None:
        return None
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError("%s must be a tensor on the GPU" % name)
    if t.dtype != dtype:
        raise TypeError("%s must be %s, got %s" % (name, dtype, t.dtype))
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % name)
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    """hipStream_t of a torch stream (the current one when None) as void*."""
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


# uint32 / uint64 buffers are held in torch's int32 / int64 tensors (same bits).
U32, U64, F32, U8 = torch.int32, torch.int64, torch.float32, torch.uint8


# ---- context and sizes -----------------------------------------------------------------------

def cnr_create(device: int = 0) -> ctypes.c_void_p:
    ctx = ctypes.c_void_p()
    _check(load().cnr_create(ctypes.byref(ctx), int(device)), "cnr_create")
    return ctx


def cnr_destroy(ctx) -> None:
    _check(load().cnr_destroy(ctx), "cnr_destroy")


def cnr_bitmap_words(n_rows: int) -> int:
    return int(load().cnr_bitmap_words(n_rows))


def cnr_packed_row_bytes(dim: int, bits: int) -> int:
    return int(load().cnr_packed_row_bytes(dim, bits))


def cnr_scratch_bytes(n_rows: int) -> int:
    return int(load().cnr_scratch_bytes(n_rows))


def cnr_mark_scratch_bytes(n_rows: int) -> int:
    return int(load().cnr_mark_scratch_bytes(n_rows))


def cnr_greedy_iterations(num_bins: int, ratio: float) -> int:
    return int(load().cnr_greedy_iterations(num_bins, ratio))


# ---- the path ------------------------------------------------------------------------------------

def cnr_clear_bitmap(ctx, bitmap, n_rows: int, stream=None) -> None:
    _check(load().cnr_clear_bitmap(ctx, _dev(bitmap, U32, "bitmap"), n_rows, _stream(stream)),
           "cnr_clear_bitmap")


def cnr_mark_touched(ctx, bitmap, n_rows: int, indices, scratch=None, stream=None) -> None:
    if indices.dtype == torch.int64:
        kind = CNR_IDX_I64
    elif indices.dtype == torch.int32:
        kind = CNR_IDX_I32
    else:
        raise TypeError("indices must be int32 or int64")
    if scratch is not None and scratch.numel() * scratch.element_size() < cnr_mark_scratch_bytes(n_rows):
        raise ValueError("scratch smaller than cnr_mark_scratch_bytes(n_rows)")
    _check(load().cnr_mark_touched(ctx, _dev(bitmap, U32, "bitmap"), n_rows,
                                   _dev(indices, indices.dtype, "indices"), indices.numel(), kind,
                                   None if scratch is None else _dev(scratch, scratch.dtype, "scratch"),
                                   _stream(stream)), "cnr_mark_touched")


def cnr_compact_dirty(ctx, bitmap, n_rows: int, row_ids, capacity: int, n_dirty_dev, scratch,
                      stream=None) -> None:
    if scratch.numel() * scratch.element_size() < cnr_scratch_bytes(n_rows):
        raise ValueError("scratch smaller than cnr_scratch_bytes(n_rows)")
    if row_ids is not None and row_ids.numel() < capacity:
        raise ValueError("row_ids shorter than capacity")
    _check(load().cnr_compact_dirty(ctx, _dev(bitmap, U32, "bitmap"), n_rows,
                                    _dev(row_ids, U32, "row_ids"), capacity,
                                    _dev(n_dirty_dev, U64, "n_dirty_dev"),
                                    _dev(scratch, scratch.dtype, "scratch"), _stream(stream)),
           "cnr_compact_dirty")


def cnr_compact_dirty_noalloc(ctx, bitmap, n_rows: int, row_ids, capacity: int, n_dirty_dev, stream=None) -> None:
    if row_ids is not None and row_ids.numel() < capacity:
        raise ValueError("row_ids shorter than capacity")
    _check(load().cnr_compact_dirty_noalloc(ctx, _dev(bitmap, U32, "bitmap"), n_rows,
                                            _dev(row_ids, U32, "row_ids"), capacity,
                                            _dev(n_dirty_dev, U64, "n_dirty_dev"), _stream(stream)),
           "cnr_compact_dirty_noalloc")


def cnr_quantize_rows(ctx, table, n_rows: int, dim: int, row_ids, n_dev, n_max: int, bits: int,
                      mode: int, greedy, scale, bias, row_min=None, row_max=None, codes_u8=None,
                      packed=None, stream=None) -> None:
    """``greedy`` is None or a (num_bins, ratio) pair."""
    gp = None
    if greedy is not None:
        gp = ctypes.pointer(cnr_greedy_params(int(greedy[0]), float(greedy[1])))
    if table.numel() < n_rows * dim:
        raise ValueError("table smaller than n_rows * dim")
    for name, t, per_row in (("scale", scale, 1), ("bias", bias, 1), ("row_min", row_min, 1),
                             ("row_max", row_max, 1), ("codes_u8", codes_u8, dim),
                             ("packed", packed, cnr_packed_row_bytes(dim, bits))):
        if t is not None and t.numel() < n_max * per_row:
            raise ValueError("%s too small for n_max rows" % name)
    if row_ids is not None and row_ids.numel() < n_max:
        raise ValueError("row_ids shorter than n_max")
    _check(load().cnr_quantize_rows(ctx, _dev(table, F32, "table"), n_rows, dim,
                                    _dev(row_ids, U32, "row_ids"), _dev(n_dev, U64, "n_dev"), n_max,
                                    bits, mode, gp, _dev(scale, F32, "scale"), _dev(bias, F32, "bias"),
                                    _dev(row_min, F32, "row_min"), _dev(row_max, F32, "row_max"),
                                    _dev(codes_u8, U8, "codes_u8"), _dev(packed, U8, "packed"),
                                    _stream(stream)), "cnr_quantize_rows")


def cnr_pack(ctx, codes_u8, n_dev, n_max: int, dim: int, bits: int, packed, stream=None) -> None:
    if codes_u8.numel() < n_max * dim or packed.numel() < n_max * cnr_packed_row_bytes(dim, bits):
        raise ValueError("buffer too small for n_max rows")
    _check(load().cnr_pack(ctx, _dev(codes_u8, U8, "codes_u8"), _dev(n_dev, U64, "n_dev"), n_max, dim,
                           bits, _dev(packed, U8, "packed"), _stream(stream)), "cnr_pack")


def cnr_restore_rows(ctx, table, n_rows: int, dim: int, row_ids, n_dev, n_max: int, bits: int,
                     packed, scale, bias, stream=None) -> None:
    if table.numel() < n_rows * dim:
        raise ValueError("table smaller than n_rows * dim")
    if (packed.numel() < n_max * cnr_packed_row_bytes(dim, bits) or scale.numel() < n_max
            or bias.numel() < n_max or (row_ids is not None and row_ids.numel() < n_max)):
        raise ValueError("buffer too small for n_max rows")
    _check(load().cnr_restore_rows(ctx, _dev(table, F32, "table"), n_rows, dim,
                                   _dev(row_ids, U32, "row_ids"), _dev(n_dev, U64, "n_dev"), n_max,
                                   bits, _dev(packed, U8, "packed"), _dev(scale, F32, "scale"),
                                   _dev(bias, F32, "bias"), _stream(stream)), "cnr_restore_rows")


def cnr_quant_error(ctx, table, n_rows: int, dim: int, row_ids, n_dev, n_max: int, bits: int, packed,
                    scale, bias, err, mean_out=None, stream=None) -> None:
    if (packed.numel() < n_max * cnr_packed_row_bytes(dim, bits) or scale.numel() < n_max
            or bias.numel() < n_max or err.numel() < n_max or (row_ids is not None and row_ids.numel() < n_max)):
        raise ValueError("buffer too small for n_max rows")
    _check(load().cnr_quant_error(ctx, _dev(table, F32, "table"), n_rows, dim, _dev(row_ids, U32, "row_ids"),
                                  _dev(n_dev, U64, "n_dev"), n_max, bits, _dev(packed, U8, "packed"),
                                  _dev(scale, F32, "scale"), _dev(bias, F32, "bias"),
                                  _dev(err, torch.float64, "err"), _dev(mean_out, torch.float64, "mean_out"),
                                  _stream(stream)), "cnr_quant_error")


# ---- several tables per launch -------------------------------------------------------------------

_JOB_TENSORS = {"table": F32, "bitmap": U32, "indices": None, "mark_scratch": None, "row_ids": U32,
                "n_dirty_dev": U64, "compact_scratch": None, "scale": F32, "bias": F32, "row_min": F32,
                "row_max": F32, "codes_u8": U8, "packed": U8}


def make_jobs(jobs):
    """A ctypes array of ``cnr_table_job`` from a list of dicts.  Keys are the struct's field names;
    tensor-valued fields take GPU tensors (checked for dtype and contiguity, resolved to device
    pointers here), ``n_rows`` / ``n_indices`` / ``capacity`` take ints; ``n_indices`` defaults to the
    length of ``indices``.  The caller keeps the tensors alive while the array is in use."""
    arr = (cnr_table_job * max(1, len(jobs)))()
    for j, d in zip(arr, jobs):
        unknown = set(d) - {f for f, _ in cnr_table_job._fields_}
        if unknown:
            raise KeyError("unknown cnr_table_job fields: %s" % sorted(unknown))
        for name, dtype in _JOB_TENSORS.items():
            t = d.get(name)
            if t is not None:
                p = _dev(t, t.dtype if dtype is None else dtype, name)
                setattr(j, name, p.value)
        j.n_rows = int(d.get("n_rows", 0))
        j.capacity = int(d.get("capacity", 0))
        idx = d.get("indices")
        j.n_indices = int(d.get("n_indices", idx.numel() if idx is not None else 0))
    return arr


def _jobs_arg(jobs):
    if isinstance(jobs, (list, tuple)):
        return make_jobs(jobs), len(jobs)
    return jobs, len(jobs)


def cnr_clear_bitmap_batch(ctx, jobs, stream=None) -> None:
    arr, n = _jobs_arg(jobs)
    _check(load().cnr_clear_bitmap_batch(ctx, arr, n, _stream(stream)), "cnr_clear_bitmap_batch")


def cnr_mark_touched_batch(ctx, jobs, index_type: int, stream=None) -> None:
    arr, n = _jobs_arg(jobs)
    _check(load().cnr_mark_touched_batch(ctx, arr, n, index_type, _stream(stream)), "cnr_mark_touched_batch")


def cnr_compact_dirty_batch(ctx, jobs, stream=None) -> None:
    arr, n = _jobs_arg(jobs)
    _check(load().cnr_compact_dirty_batch(ctx, arr, n, _stream(stream)), "cnr_compact_dirty_batch")


def cnr_quantize_rows_batch(ctx, jobs, dim: int, bits: int, mode: int, greedy=None, stream=None) -> None:
    arr, n = _jobs_arg(jobs)
    gp = None
    if greedy is not None:
        gp = ctypes.pointer(cnr_greedy_params(int(greedy[0]), float(greedy[1])))
    _check(load().cnr_quantize_rows_batch(ctx, arr, n, dim, bits, mode, gp, _stream(stream)),
           "cnr_quantize_rows_batch")


def cnr_restore_rows_batch(ctx, jobs, dim: int, bits: int, stream=None) -> None:
    arr, n = _jobs_arg(jobs)
    _check(load().cnr_restore_rows_batch(ctx, arr, n, dim, bits, _stream(stream)), "cnr_restore_rows_batch")


# ---- greedy parameters by profiling ----------------------------------------------------------------

def cnr_select_scratch_bytes(n_sample: int, dim: int, bits: int) -> int:
    return int(load().cnr_select_scratch_bytes(n_sample, dim, bits))


def cnr_select_greedy_params(ctx, table, n_rows: int, dim: int, sample_ids, bits: int, bins_grid, ratio_grid,
                             taper: float, scratch, stream=None):
    """Returns ((num_bins, ratio), report) with report = [E_minmax, E(bins...)..., E(ratios...)...]."""
    n = sample_ids.numel()
    if scratch.numel() * scratch.element_size() < cnr_select_scratch_bytes(n, dim, bits):
        raise ValueError("scratch smaller than cnr_select_scratch_bytes")
    bins = (ctypes.c_uint32 * len(bins_grid))(*[int(b) for b in bins_grid])
    ratios = (ctypes.c_float * len(ratio_grid))(*[float(r) for r in ratio_grid])
    report = (ctypes.c_double * (1 + len(bins_grid) + len(ratio_grid)))()
    chosen = cnr_greedy_params()
    _check(load().cnr_select_greedy_params(ctx, _dev(table, F32, "table"), n_rows, dim, _dev(sample_ids, U32, "sample_ids"),
                                           n, bits, bins, len(bins_grid), ratios, len(ratio_grid), float(taper),
                                           _dev(scratch, scratch.dtype, "scratch"), ctypes.byref(chosen), report,
                                           _stream(stream)), "cnr_select_greedy_params")
    return (int(chosen.num_bins), float(chosen.ratio)), list(report)


# ---- chunked encode into host memory --------------------------------------------------------------

def cnr_host_writer_device_bytes(dim: int, bits: int, chunk_rows: int) -> int:
    return int(load().cnr_host_writer_device_bytes(dim, bits, chunk_rows))


def cnr_host_writer_create(ctx, dim: int, bits: int, chunk_rows: int) -> ctypes.c_void_p:
    w = ctypes.c_void_p()
    _check(load().cnr_host_writer_create(ctx, dim, bits, chunk_rows, ctypes.byref(w)), "cnr_host_writer_create")
    return w


def cnr_host_writer_destroy(writer) -> None:
    _check(load().cnr_host_writer_destroy(writer), "cnr_host_writer_destroy")


def _host(t, dtype, name: str, n_items: int):
    """Pointer of a contiguous CPU tensor with room for n_items elements."""
    if t is None:
        return None
    if not isinstance(t, torch.Tensor) or t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise TypeError("%s must be a contiguous CPU tensor of %s" % (name, dtype))
    if t.numel() < n_items:
        raise ValueError("%s too small" % name)
    return ctypes.c_void_p(t.data_ptr())


def cnr_encode_to_host(writer, table, n_rows: int, dim: int, bits: int, row_ids, n: int, mode: int, greedy,
                       host_row_ids, host_scale, host_bias, host_packed, overlap=CNR_HOST_OVERLAP, stream=None) -> None:
    """``dim`` and ``bits`` are the writer's (used here to check the host buffers' sizes); ``overlap`` is
    CNR_HOST_SERIAL, CNR_HOST_OVERLAP (False and True mean the same) or CNR_HOST_DIRECT."""
    gp = None
    if greedy is not None:
        gp = ctypes.pointer(cnr_greedy_params(int(greedy[0]), float(greedy[1])))
    if table.numel() < n_rows * dim:
        raise ValueError("table smaller than n_rows * dim")
    if row_ids is not None and row_ids.numel() < n:
        raise ValueError("row_ids shorter than n")
    _check(load().cnr_encode_to_host(writer, _dev(table, F32, "table"), n_rows, _dev(row_ids, U32, "row_ids"), n, mode,
                                     gp, _host(host_row_ids, U32, "host_row_ids", n),
                                     _host(host_scale, F32, "host_scale", n), _host(host_bias, F32, "host_bias", n),
                                     _host(host_packed, U8, "host_packed", n * cnr_packed_row_bytes(dim, bits)),
                                     int(overlap), _stream(stream)), "cnr_encode_to_host")


def cnr_restore_from_host(writer, table, n_rows: int, dim: int, bits: int, host_row_ids, host_scale, host_bias,
                          host_packed, n: int, overlap=CNR_HOST_OVERLAP, stream=None) -> None:
    """``dim`` and ``bits`` are the writer's (used here to check the buffers' sizes); ``overlap`` is
    CNR_HOST_SERIAL, CNR_HOST_OVERLAP (False and True mean the same) or CNR_HOST_DIRECT."""
    if table.numel() < n_rows * dim:
        raise ValueError("table smaller than n_rows * dim")
    _check(load().cnr_restore_from_host(writer, _dev(table, F32, "table"), n_rows,
                                        _host(host_row_ids, U32, "host_row_ids", n),
                                        _host(host_scale, F32, "host_scale", n), _host(host_bias, F32, "host_bias", n),
                                        _host(host_packed, U8, "host_packed", n * cnr_packed_row_bytes(dim, bits)),
                                        n, int(overlap), _stream(stream)), "cnr_restore_from_host")


def cnr_host_writer_wait(writer, stream=None) -> None:
    _check(load().cnr_host_writer_wait(writer, _stream(stream)), "cnr_host_writer_wait")


def cnr_poll_errors(ctx, stream=None):
    """Returns (status, n_bad_indices, flags); synchronises the stream."""
    bad, flags = ctypes.c_uint64(0), ctypes.c_uint32(0)
    st = load().cnr_poll_errors(ctx, _stream(stream), ctypes.byref(bad), ctypes.byref(flags))
    if st in (CNR_E_HIP, CNR_E_INVALID):
        raise CnrError(st, "cnr_poll_errors")
    return st, int(bad.value), int(flags.value)


def prepare(name: str, *args):
    """A zero-argument callable that repeats one library call with fixed arguments.

    ``args`` are given as for the binding function ``name`` except that every tensor is resolved to
    its device pointer once, here, and ``stream`` (last argument, may be None = the current stream
    at preparation time) to its handle.  The returned callable only crosses into C and checks the
    status, so a tight loop of launches is not slowed down by per-call argument checks.  The caller
    keeps the tensors alive and unchanged in place."""
    fn = getattr(load(), name)
    *body, stream = args
    cargs = []
    for a in body:
        if isinstance(a, torch.Tensor):
            if not a.is_cuda or not a.is_contiguous():
                raise ValueError("prepared arguments must be contiguous GPU tensors")
            cargs.append(ctypes.c_void_p(a.data_ptr()))
        elif isinstance(a, tuple):                       # (num_bins, ratio)
            cargs.append(ctypes.pointer(cnr_greedy_params(int(a[0]), float(a[1]))))
        else:
            cargs.append(a)
    cargs.append(_stream(stream))

    def call():
        st = fn(*cargs)
        if st != CNR_OK:
            raise CnrError(st, name)
    return call


def cnr_last_hip_error(ctx) -> int:
    return int(load().cnr_last_hip_error(ctx))


def cnr_full_checkpoint_due(sizes) -> bool:
    arr = (ctypes.c_double * len(sizes))(*[float(s) for s in sizes])
    return bool(load().cnr_full_checkpoint_due(arr, len(sizes)))


def cnr_select_bits(expected_resumes: int, observed_resumes: int = 0) -> int:
    return int(load().cnr_select_bits(int(expected_resumes), int(observed_resumes)))


def cnr_policy_init(kind: int) -> cnr_policy:
    p = cnr_policy()
    _check(load().cnr_policy_init(ctypes.byref(p), int(kind)), "cnr_policy_init")
    return p


def cnr_policy_next(policy: cnr_policy, dirty_fraction: float):
    """Returns (take_full, clear_bitmap) for the checkpoint at the end of this interval."""
    d = load().cnr_policy_next(ctypes.byref(policy), float(dirty_fraction))
    return bool(d.take_full), bool(d.clear_bitmap)
