"""Device buffers for one table's checkpoints and the order of the library calls.

Plumbing only: torch allocates the memory and provides the stream, every step of the path runs in
libcnr's kernels.  One :class:`TableCheckpointer` serves one embedding table (one shard of the
model on this GPU, Section 4.1): it keeps the tracking bit-vector between iterations
(Section 5.1.1) and, at checkpoint time, produces the incremental, quantized view of the table
(Sections 5.1 and 5.2).
"""
from __future__ import annotations

from dataclasses import dataclass

import torch

from . import binding as B


@dataclass
class EncodedRows:
    """One table's incremental checkpoint as it sits in device memory (valid up to ``n`` rows)."""
    n_dev: torch.Tensor      # int64 [1]: number of dirty rows
    row_ids: torch.Tensor    # int32 (uint32 bits) [capacity]
    scale: torch.Tensor      # float32 [capacity]
    bias: torch.Tensor       # float32 [capacity]
    packed: torch.Tensor     # uint8 [capacity * packed_row_bytes]
    bits: int
    dim: int
    row_min: torch.Tensor | None = None
    row_max: torch.Tensor | None = None

    def count(self) -> int:
        """Number of rows encoded (synchronises)."""
        return int(self.n_dev.item())


class TableCheckpointer:
    def __init__(self, ctx, n_rows: int, dim: int, capacity: int | None = None, device="cuda:0",
                 mark_scratch: torch.Tensor | None = None):
        self.ctx, self.n_rows, self.dim = ctx, int(n_rows), int(dim)
        self.capacity = self.n_rows if capacity is None else int(capacity)
        self.device = torch.device(device)
        dev = self.device
        self.bitmap = torch.zeros(max(1, B.cnr_bitmap_words(n_rows)), dtype=torch.int32, device=dev)
        self.scratch = torch.empty((B.cnr_scratch_bytes(n_rows) + 7) // 8, dtype=torch.int64, device=dev)
        self.row_ids = torch.empty(max(1, self.capacity), dtype=torch.int32, device=dev)
        self.n_dirty = torch.zeros(1, dtype=torch.int64, device=dev)
        # zero-filled scratch for marking long index streams; may be shared between the tables of
        # one stream (pass the same tensor), the library leaves it zeroed after every call
        self.mark_scratch = mark_scratch
        if mark_scratch is not None and mark_scratch.numel() * mark_scratch.element_size() < B.cnr_mark_scratch_bytes(n_rows):
            raise ValueError("mark_scratch too small for this table")

    @staticmethod
    def new_mark_scratch(max_rows: int, device="cuda:0") -> torch.Tensor:
        return torch.zeros((B.cnr_mark_scratch_bytes(max_rows) + 7) // 8, dtype=torch.int64, device=device)

    # -- tracking ---------------------------------------------------------------------------
    def clear(self, stream=None) -> None:
        B.cnr_clear_bitmap(self.ctx, self.bitmap, self.n_rows, stream)

    def mark(self, indices: torch.Tensor, stream=None) -> None:
        B.cnr_mark_touched(self.ctx, self.bitmap, self.n_rows, indices.reshape(-1), self.mark_scratch, stream)

    # -- checkpoint -------------------------------------------------------------------------
    def compact(self, stream=None) -> None:
        B.cnr_compact_dirty(self.ctx, self.bitmap, self.n_rows, self.row_ids, self.capacity,
                            self.n_dirty, self.scratch, stream)

    def alloc_output(self, bits: int, want_range: bool = False) -> EncodedRows:
        cap, dev = max(1, self.capacity), self.device
        f = lambda: torch.empty(cap, dtype=torch.float32, device=dev)  # noqa: E731
        return EncodedRows(self.n_dirty, self.row_ids, f(), f(),
                           torch.empty(cap * B.cnr_packed_row_bytes(self.dim, bits), dtype=torch.uint8,
                                       device=dev),
                           bits, self.dim, f() if want_range else None, f() if want_range else None)

    def encode(self, table: torch.Tensor, out: EncodedRows, mode: int = B.CNR_RANGE_MINMAX,
               greedy=None, codes_u8=None, fused: bool = True, stream=None) -> EncodedRows:
        """Quantizes the rows listed by the last :meth:`compact` into ``out``."""
        B.cnr_quantize_rows(self.ctx, table, self.n_rows, self.dim, self.row_ids, self.n_dirty,
                            self.capacity, out.bits, mode, greedy, out.scale, out.bias, out.row_min,
                            out.row_max, codes_u8, out.packed if fused else None, stream)
        if not fused:
            B.cnr_pack(self.ctx, codes_u8, self.n_dirty, self.capacity, self.dim, out.bits, out.packed,
                       stream)
        return out

    def restore(self, table: torch.Tensor, enc: EncodedRows, stream=None) -> None:
        """Writes the de-quantized rows of ``enc`` over the same rows of ``table`` in place."""
        B.cnr_restore_rows(self.ctx, table, self.n_rows, self.dim, enc.row_ids, enc.n_dev, self.capacity,
                           enc.bits, enc.packed, enc.scale, enc.bias, stream)

    # -- repeated checkpoints of the same buffers ---------------------------------------------------
    def prepare_step(self, indices: torch.Tensor, table: torch.Tensor, out: EncodedRows,
                     restore_into: torch.Tensor | None = None, mode: int = B.CNR_RANGE_MINMAX,
                     greedy=None, stream=None):
        """The calls of one checkpoint of this table (clear, mark, compact, encode and, when
        ``restore_into`` is given, restore) as a list of (label, zero-argument callable), with all
        arguments resolved once (see :func:`binding.prepare`)."""
        idx = indices.reshape(-1)
        kind = B.CNR_IDX_I64 if idx.dtype == torch.int64 else B.CNR_IDX_I32
        steps = [
            ("clear", B.prepare("cnr_clear_bitmap", self.ctx, self.bitmap, self.n_rows, stream)),
            ("mark", B.prepare("cnr_mark_touched", self.ctx, self.bitmap, self.n_rows, idx, idx.numel(), kind,
                               self.mark_scratch, stream)),
            ("compact", B.prepare("cnr_compact_dirty", self.ctx, self.bitmap, self.n_rows, self.row_ids,
                                  self.capacity, self.n_dirty, self.scratch, stream)),
            ("encode", B.prepare("cnr_quantize_rows", self.ctx, table, self.n_rows, self.dim, self.row_ids,
                                 self.n_dirty, self.capacity, out.bits, mode, greedy, out.scale, out.bias,
                                 out.row_min, out.row_max, None, out.packed, stream)),
        ]
        if restore_into is not None:
            steps.append(("restore", B.prepare("cnr_restore_rows", self.ctx, restore_into, self.n_rows, self.dim,
                                               out.row_ids, out.n_dev, self.capacity, out.bits, out.packed,
                                               out.scale, out.bias, stream)))
        return steps


class BatchCheckpointer:
    """Several tables of one row length checkpointed together: every stage is one ``*_batch`` call
    (one launch per kernel for up to ``CNR_MAX_BATCH`` tables) instead of one call per table.

    Built from per-table :class:`TableCheckpointer` objects, which keep owning the buffers; each
    needs a mark scratch of its own if the bulk marking route is wanted (the tables of a batch are
    marked side by side)."""

    def __init__(self, ctx, checkpointers):
        self.ctx = ctx
        self.cks = list(checkpointers)
        if not self.cks:
            raise ValueError("no tables")
        if len({c.dim for c in self.cks}) != 1:
            raise ValueError("the tables of a batch share one row length")
        self.dim = self.cks[0].dim
        scratches = [c.mark_scratch.data_ptr() for c in self.cks if c.mark_scratch is not None]
        if len(set(scratches)) != len(scratches):
            raise ValueError("tables of a batch must not share a mark scratch")

    def _track_fields(self, c):
        return dict(n_rows=c.n_rows, bitmap=c.bitmap, mark_scratch=c.mark_scratch, row_ids=c.row_ids,
                    capacity=c.capacity, n_dirty_dev=c.n_dirty, compact_scratch=c.scratch)

    def jobs(self, indices=None, tables=None, outs=None):
        """The job array for these tables; ``indices`` / ``tables`` / ``outs`` are per-table lists
        (look-up tensors, fp32 tables, :class:`EncodedRows`) or None where a call does not need them."""
        jobs = []
        for i, c in enumerate(self.cks):
            d = self._track_fields(c)
            if indices is not None and indices[i] is not None:
                d["indices"] = indices[i].reshape(-1)
            if tables is not None:
                if tables[i].numel() < c.n_rows * c.dim:
                    raise ValueError("table %d smaller than n_rows * dim" % i)
                d["table"] = tables[i]
            if outs is not None:
                o = outs[i]
                cap = max(1, c.capacity)
                if (o.scale.numel() < cap or o.bias.numel() < cap
                        or o.packed.numel() < cap * B.cnr_packed_row_bytes(c.dim, o.bits)):
                    raise ValueError("output %d too small for the table's capacity" % i)
                d.update(scale=o.scale, bias=o.bias, row_min=o.row_min, row_max=o.row_max, packed=o.packed)
            jobs.append(d)
        return B.make_jobs(jobs)

    @staticmethod
    def _index_type(indices):
        kinds = {t.dtype for t in indices if t is not None}
        if len(kinds) > 1:
            raise TypeError("the index streams of a batch share one dtype")
        return B.CNR_IDX_I32 if kinds == {torch.int32} else B.CNR_IDX_I64

    def clear(self, stream=None) -> None:
        B.cnr_clear_bitmap_batch(self.ctx, self.jobs(), stream)

    def mark(self, indices, stream=None) -> None:
        B.cnr_mark_touched_batch(self.ctx, self.jobs(indices=indices), self._index_type(indices), stream)

    def compact(self, stream=None) -> None:
        B.cnr_compact_dirty_batch(self.ctx, self.jobs(), stream)

    def encode(self, tables, outs, mode: int = B.CNR_RANGE_MINMAX, greedy=None, stream=None) -> None:
        bits = outs[0].bits
        if any(o.bits != bits for o in outs):
            raise ValueError("the outputs of a batch share one bit-width")
        B.cnr_quantize_rows_batch(self.ctx, self.jobs(tables=tables, outs=outs), self.dim, bits, mode, greedy,
                                  stream)

    def restore(self, tables, encs, stream=None) -> None:
        """Writes the rows of ``encs[i]`` over the same rows of ``tables[i]``."""
        B.cnr_restore_rows_batch(self.ctx, self.jobs(tables=tables, outs=encs), self.dim, encs[0].bits, stream)

    def prepare_step(self, indices, tables, outs, restore_into=None, mode: int = B.CNR_RANGE_MINMAX,
                     greedy=None, stream=None):
        """One checkpoint of all tables (clear, mark, compact, encode and, when ``restore_into`` lists
        one destination table per table, restore) as (label, zero-argument callable) pairs with the
        job arrays built once."""
        n = len(self.cks)
        track = self.jobs(indices=indices)
        enc = self.jobs(tables=tables, outs=outs)
        kind = self._index_type(indices)
        bits = outs[0].bits
        steps = [
            ("clear", B.prepare("cnr_clear_bitmap_batch", self.ctx, track, n, stream)),
            ("mark", B.prepare("cnr_mark_touched_batch", self.ctx, track, n, kind, stream)),
            ("compact", B.prepare("cnr_compact_dirty_batch", self.ctx, track, n, stream)),
            ("encode", B.prepare("cnr_quantize_rows_batch", self.ctx, enc, n, self.dim, bits, mode, greedy, stream)),
        ]
        if restore_into is not None:
            back = self.jobs(tables=restore_into, outs=outs)
            steps.append(("restore", B.prepare("cnr_restore_rows_batch", self.ctx, back, n, self.dim, bits, stream)))
        return steps


class HostCheckpointWriter:
    """Chunked encode with the device-to-host copy of chunk c overlapping the encode of chunk c+1
    (Section 4.4 and 5.2: the optimized checkpoint is built chunk by chunk and every finished chunk
    is handed on while the next one is being quantized).

    Plumbing only: the library's writer (``cnr_host_writer_*``, ``cnr_encode_to_host``) owns the two
    device staging sets and the copy stream and orders the chunks; this class owns the pinned host
    buffers the chunks land in (where a storage writer would pick them up)."""

    def __init__(self, ctx, dim: int, bits: int, capacity: int, chunk_rows: int = 1 << 20, device="cuda:0"):
        if chunk_rows % 16:
            raise ValueError("chunk_rows must be a multiple of 16 (keeps every slice 16-byte aligned)")
        self.ctx, self.dim, self.bits, self.capacity, self.chunk = ctx, dim, bits, int(capacity), int(chunk_rows)
        self.prb = B.cnr_packed_row_bytes(dim, bits)
        with torch.cuda.device(torch.device(device)):
            self.writer = B.cnr_host_writer_create(ctx, dim, bits, self.chunk)
        cap = max(1, self.capacity)
        self.host = dict(row_ids=torch.empty(cap, dtype=torch.int32, pin_memory=True),
                         scale=torch.empty(cap, dtype=torch.float32, pin_memory=True),
                         bias=torch.empty(cap, dtype=torch.float32, pin_memory=True),
                         packed=torch.empty(cap * self.prb, dtype=torch.uint8, pin_memory=True))
        self.n_host = torch.zeros(1, dtype=torch.int64, pin_memory=True)

    def close(self) -> None:
        if self.writer is not None:
            B.cnr_host_writer_destroy(self.writer)
            self.writer = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _to_host_path(self, overlap):
        """None: the faster way for this row length (the kernel's own stores for rows of up to 64
        elements, staged copies that overlap the encode for longer ones)."""
        if overlap is None:
            return B.CNR_HOST_DIRECT if self.dim <= 64 else B.CNR_HOST_OVERLAP
        return int(overlap)

    def encode_to_host(self, ck: TableCheckpointer, table: torch.Tensor, mode: int = B.CNR_RANGE_MINMAX,
                       greedy=None, overlap=None) -> int:
        """Encodes the rows listed by ``ck.compact()`` and leaves ids, scale, bias and packed codes in
        the pinned host buffers; returns the number of rows.  ``overlap`` is a ``CNR_HOST_*`` path
        (True and False mean OVERLAP and SERIAL), None picks by row length.  Synchronises at the start
        (the row count has to reach the host to size the copies) and at the end."""
        overlap = self._to_host_path(overlap)
        main = torch.cuda.current_stream()
        self.n_host.copy_(ck.n_dirty, non_blocking=True)
        main.synchronize()
        n = min(int(self.n_host.item()), ck.capacity, self.capacity)
        B.cnr_encode_to_host(self.writer, table, ck.n_rows, self.dim, self.bits, ck.row_ids, n, mode, greedy,
                             self.host["row_ids"], self.host["scale"], self.host["bias"], self.host["packed"],
                             overlap, main)
        B.cnr_host_writer_wait(self.writer, main)
        return n

    def encode_table_to_host(self, table: torch.Tensor, n_rows: int, mode: int = B.CNR_RANGE_MINMAX,
                             greedy=None, overlap=None) -> int:
        """A full (baseline) checkpoint: every row of ``table``, no id list, into the pinned host
        buffers; returns ``n_rows``.  Synchronises at the end."""
        overlap = self._to_host_path(overlap)
        if n_rows > self.capacity:
            raise ValueError("the writer's host buffers hold %d rows" % self.capacity)
        main = torch.cuda.current_stream()
        B.cnr_encode_to_host(self.writer, table, n_rows, self.dim, self.bits, None, n_rows, mode, greedy,
                             None, self.host["scale"], self.host["bias"], self.host["packed"], overlap, main)
        B.cnr_host_writer_wait(self.writer, main)
        return n_rows

    def restore_from_host(self, table: torch.Tensor, n_rows: int, n: int, overlap=B.CNR_HOST_DIRECT,
                          with_ids: bool = True) -> None:
        """Writes the first ``n`` rows held in the pinned host buffers (as :meth:`encode_to_host` left
        them, or as a loader filled them) over ``table``.  By default the restore kernel reads the
        pinned buffers itself over the host link (``CNR_HOST_DIRECT``); with ``CNR_HOST_OVERLAP`` (or
        True) the copy of chunk c+1 from host memory overlaps the de-quantize-and-scatter of chunk c,
        with ``CNR_HOST_SERIAL`` (or False) copies and kernels alternate on one stream.  Synchronises
        at the end."""
        main = torch.cuda.current_stream()
        B.cnr_restore_from_host(self.writer, table, n_rows, self.dim, self.bits,
                                self.host["row_ids"] if with_ids else None, self.host["scale"], self.host["bias"],
                                self.host["packed"], n, overlap, main)
        B.cnr_host_writer_wait(self.writer, main)
