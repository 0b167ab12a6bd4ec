#!/usr/bin/env python3
"""Benchmark of the checkpoint-encoder hot path on one MI355X.

One step = one checkpoint of the whole workload: for every table, clear the tracking bitmap, mark
it from the table's look-up stream, compact it into the dirty-row list, gather + quantize + pack the
dirty rows (fused kernel), and restore them into a stale baseline table.  Inputs (tables, index
streams) are resident in HBM before the timed region.  The reported value is fp32 table bytes
checkpointed per second over the whole step.

Default workload: the 8 x 5M x 64 outlier-mix tables with 30 % dirty rows, 4 bits, min/max range.
The same tables are also encoded once per run with the greedy range search (100 bins, ratio 1),
reported separately against the vector-ALU roofline, and the CPU oracle is timed on a bounded
sample of the same workload.

Prints one JSON line.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import paper_2010_08679_amd as P  # noqa: E402
from paper_2010_08679_amd import synth  # noqa: E402

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published
FP32_VECTOR_PEAK_TFLOPS = 157.3  # MI355X fp32 vector, published
# SIMD time the greedy search needs per element and candidate range: 26 clocks of a 16-lane SIMD for a
# wave of 64 (add / subtract / multiply occupy it for 2 clocks, every other vector instruction of the
# loop for 4: bench_ceilings.hip measures that), with 256 CUs x 4 SIMDs at 2.4 GHz
GREEDY_SIMD_CLOCKS_PER_ELEMENT = 26.0
SIMD_CLOCKS_PER_S = 256 * 4 * 2.4e9

# HBM traffic of the two bandwidth-bound kernels from rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE, each
# scaled by what a 1 GiB device copy reads on the same counter: 2.000 and 1.000), in bytes per dirty row,
# valid only for the kernel source whose hash is recorded with it (profiles/hbm_traffic.txt).
TRAFFIC_PER_ROW = {
    # _kernel_hash() : {workload/bits : bytes per dirty row}
    "a2e6a8cd8520d9e7bb6344cdfd2a382c27d08e95db09fef0a95bfb9a9a5ff999": {"cfg4/b4": 300.96, "cfg3/b2": 558.98, "cfg3/b3": 581.12, "cfg5/b8": 658.98, "cfg5/b4": 592.55},
}
RESTORE_TRAFFIC_PER_ROW = {
    "0a151c3fed73be1daf849a41a37f121a6c0b73202cd2806cb848ad2850c9bc6b": {"cfg4/b4": 300.01, "cfg3/b2": 556.09, "cfg3/b3": 572.08, "cfg5/b8": 652.09, "cfg5/b4": 588.04},
}


def _source_hash(name: str, upto: str | None = None) -> str:
    """Hash of a kernel source file (up to the line that starts the section `upto`), without comments
    and white space."""
    with open(os.path.join(ROOT, "paper_2010_08679_amd", "csrc", name), "r") as f:
        text = f.read()
    if upto is not None:
        text = text[:text.index(upto)]
    code = "".join(line.split("//")[0] for line in text.splitlines(True))
    return hashlib.sha256("".join(code.split()).encode()).hexdigest()


def _kernel_hash() -> str:
    """The tile kernel's source: everything in its file above the greedy kernel's section."""
    return _source_hash("cnr_quantize.hip", "// Greedy range search")


def _restore_kernel_hash() -> str:
    return _source_hash("cnr_restore.hip")


def encode_bytes_per_row(dim: int, bits: int) -> int:
    """Algorithmic bytes of the fused encode per dirty row: row id + gathered row + packed codes +
    scale and bias."""
    return 4 + 4 * dim + dim * bits // 8 + 8


def restore_bytes_per_row(dim: int, bits: int) -> int:
    return 4 + dim * bits // 8 + 8 + 4 * dim


def B_prepare_mark(batch, indices):
    """One prepared batched mark of `indices` (a list of tensors, one per table of `batch`)."""
    jobs = batch.jobs(indices=indices)
    return P.prepare("cnr_mark_touched_batch", batch.ctx, jobs, len(indices), P.CNR_IDX_I64, None)


class Timer:
    """Pairs of events on the current stream, summed per label.  Events are created up front so that
    the timed loop only records them."""

    def __init__(self, labels, n_spans_per_label):
        self.pool = {k: [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
                         for _ in range(n_spans_per_label)] for k in labels}
        self.used = {k: 0 for k in labels}

    def span(self, label):
        i = self.used[label]
        self.used[label] = i + 1
        return self.pool[label][i]

    def totals_ms(self):
        return {k: sum(a.elapsed_time(b) for a, b in v[:self.used[k]]) for k, v in self.pool.items() if self.used[k]}

    def counts(self):
        return dict(self.used)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="cfg4", choices=sorted(synth.WORKLOADS))
    ap.add_argument("--tables", type=int, default=0, help="use only the first N tables (0 = all)")
    ap.add_argument("--bits", type=int, default=4)
    ap.add_argument("--per-table", action="store_true",
                    help="one library call per table and stage instead of one batched call per stage")
    ap.add_argument("--no-greedy", action="store_true", help="skip the greedy-range extra")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline")
    ap.add_argument("--no-host-copy", action="store_true", help="skip the chunked encode-to-host extra")
    ap.add_argument("--no-full", action="store_true", help="skip the full-checkpoint extra")
    ap.add_argument("--iterations", type=int, default=0,
                    help="look-up iterations per table of a Zipf workload (0 = the workload's own count, "
                         "stopping early at the share of dirty rows it names)")
    ap.add_argument("--seed", type=int, default=4)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (each GPU checkpoints its own table "
              "shard independently); --gpus %d is not supported" % args.gpus, file=sys.stderr)
        return 2
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2

    dev = "cuda:0"
    torch.cuda.set_device(0)
    w = synth.WORKLOADS[args.workload]
    n_tables = w.n_tables if args.tables <= 0 else min(args.tables, w.n_tables)
    bits = args.bits
    ctx = P.cnr_create(0)

    # ---- resident inputs ------------------------------------------------------------------------
    tables, streams, cks, encs = [], [], [], []
    batched = not args.per_table
    # the batched form restores every table into a stale table of its own; where that does not fit the
    # GPU's memory (configuration 5 at full size: 197 GB of tables), fall back to per-table calls
    table_bytes = w.n_rows * w.dim * 4
    per_row_extra = 12 + P.cnr_packed_row_bytes(w.dim, bits) + 1 + 8       # outputs, ids, mark scratch, look-ups (about)
    need_batched = n_tables * (2 * table_bytes + w.n_rows * per_row_extra)
    free_bytes = torch.cuda.mem_get_info()[0]
    if batched and need_batched > 0.92 * free_bytes:
        print("bench.py: the batched form needs about %.0f GB, %.0f GB are free: one call per table and stage instead"
              % (need_batched / 1e9, free_bytes / 1e9), file=sys.stderr)
        batched = False
    # per-table calls run one after the other and can share the scratch of the bulk mark
    # and the stale table that restore writes into; batched calls work on all tables at once
    shared_scratch = None if batched else P.TableCheckpointer.new_mark_scratch(w.n_rows, dev)
    # Look-up streams first.  A Zipf workload runs its own number of iterations (rounds of 16 M look-ups
    # for the until-coverage kind, at most 64) and stops early once the share of dirty rows it names is
    # reached, measured with the library's own mark + compact on a probe bitmap; --iterations overrides
    # the count (and then nothing stops early).  What was run is spelled out in config.workload.
    iters_run, probe_dirty = [], []
    for ti in range(n_tables):
        if w.lookups == "bernoulli":
            batches = list(synth.lookup_batches(w, ti, args.seed, dev))
        else:
            limit = args.iterations if args.iterations > 0 else (w.iterations or 64)
            target = w.dirty_fraction * w.n_rows if (w.dirty_fraction and args.iterations <= 0) else None
            probe = P.TableCheckpointer(ctx, w.n_rows, w.dim, device=dev, mark_scratch=shared_scratch)
            probe.clear()
            batches = []
            for idx in synth.lookup_batches(w, ti, args.seed, dev, iterations=limit):
                batches.append(idx)
                if target is not None:
                    probe.mark(idx)
                    probe.compact()
                    if int(probe.n_dirty.item()) >= target:
                        break
            del probe
        iters_run.append(len(batches))
        streams.append(torch.cat([b.reshape(-1) for b in batches]))
        del batches
    for ti in range(n_tables):
        tables.append(synth.make_table(w, ti, args.seed, dev))
        scratch = P.TableCheckpointer.new_mark_scratch(w.n_rows, dev) if batched else shared_scratch
        # room for 1.25 x the share of dirty rows the workload names (all rows when it names none)
        cap = w.n_rows if not w.dirty_fraction or args.iterations > 0 else min(
            w.n_rows, (int(1.25 * w.dirty_fraction * w.n_rows) + 1023) & ~1023)
        ck = P.TableCheckpointer(ctx, w.n_rows, w.dim, capacity=cap, device=dev, mark_scratch=scratch)
        cks.append(ck)
        encs.append(ck.alloc_output(bits))
    stale = [torch.zeros((w.n_rows, w.dim), dtype=torch.float32, device=dev) for _ in range(n_tables if batched else 1)]
    torch.cuda.synchronize()

    # one checkpoint of every table as a flat list of prepared launches (arguments resolved once, so
    # that the host keeps ahead of the GPU)
    if batched:
        batch = P.BatchCheckpointer(ctx, cks)
        calls = batch.prepare_step(streams, tables, encs, restore_into=stale)
    else:
        calls = []
        for ti in range(n_tables):
            calls += cks[ti].prepare_step(streams[ti], tables[ti], encs[ti], restore_into=stale[0])
    launches_per_stage = 1 if batched else n_tables

    def step(timer, bracket):
        for label, fn in calls:
            if timer is not None and label in bracket:
                a, b = timer.span(label)
                a.record()
                fn()
                b.record()
            else:
                fn()

    for _ in range(args.warmup):
        step(None, ())
    torch.cuda.synchronize()
    st, bad, flags = P.cnr_poll_errors(ctx)
    assert (st, bad, flags) == (P.CNR_OK, 0, 0), (st, bad, flags)
    n_dirty = [int(c.n_dirty.item()) for c in cks]

    # timed region: only the dominant kernel is bracketed by events, so that the host issues the
    # launches of a step faster than the GPU runs them
    timer = Timer(("encode",), args.steps * launches_per_stage)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(timer, ("encode",))
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    # per-stage split from a second, untimed run of the same steps with every launch bracketed
    stage_labels = ("clear", "mark", "compact", "encode", "restore")
    stage_timer = Timer(stage_labels, args.steps * launches_per_stage)
    for _ in range(args.steps):
        step(stage_timer, stage_labels)
    torch.cuda.synchronize()

    # what an event pair around nothing reads: the part of avg_launch_ms that is not the kernel
    null_timer = Timer(("null",), 64)
    for _ in range(64):
        a, b = null_timer.span("null")
        a.record()
        b.record()
    torch.cuda.synchronize()
    null_ms = null_timer.totals_ms()["null"] / 64

    ms_per_step = wall * 1e3 / args.steps
    table_bytes = sum(n_dirty) * w.dim * 4
    value = table_bytes / (ms_per_step * 1e-3) / 1e9
    stage_ms = {k: v / args.steps for k, v in stage_timer.totals_ms().items()}
    launches = timer.counts()

    # dominant kernel: the fused gather + quantize + pack.  A span of events holds one launch: one
    # table (per-table calls), or all tables of the batched call (up to 16 tables per launch).
    tables_per_launch = n_tables // launches_per_stage
    launches_per_span = -(-tables_per_launch // P.CNR_MAX_BATCH)
    enc_launch_ms = timer.totals_ms()["encode"] / (launches["encode"] * launches_per_span)
    rows_per_launch = sum(n_dirty) / n_tables * tables_per_launch / launches_per_span
    enc_bytes = encode_bytes_per_row(w.dim, bits) * rows_per_launch
    achieved = enc_bytes / (enc_launch_ms * 1e-3) / 1e9
    traffic = None
    rec = TRAFFIC_PER_ROW.get(_kernel_hash(), {}).get("%s/b%d" % (w.name, bits))
    if rec:
        traffic = round(rec * rows_per_launch, 1)
    roofline = {"bound": "hbm", "kernel": "quantize_tile_kernel<%d, %d>" % (w.dim // 16, bits),
                "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": traffic,
                "bytes_per_launch": int(enc_bytes), "avg_launch_ms": round(enc_launch_ms, 5),
                "tables_per_launch": tables_per_launch // launches_per_span,
                "launches_per_event_span": launches_per_span, "empty_event_pair_ms": round(null_ms, 5)}
    res_ms = stage_timer.totals_ms()["restore"] / (stage_timer.counts()["restore"] * launches_per_span)
    res_bytes = restore_bytes_per_row(w.dim, bits) * rows_per_launch
    res_achieved = res_bytes / (res_ms * 1e-3) / 1e9
    res_traffic = None
    rec = RESTORE_TRAFFIC_PER_ROW.get(_restore_kernel_hash(), {}).get("%s/b%d" % (w.name, bits))
    if rec:
        res_traffic = round(rec * rows_per_launch, 1)
    # the other long kernel of a step, measured the same way (from the per-stage run)
    roofline_restore = {"bound": "hbm", "kernel": "restore_rows16_kernel<%d, %d>" % (w.dim // 16, bits),
                        "achieved": round(res_achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                        "frac": round(res_achieved / HBM_PEAK_GBPS, 4), "traffic": res_traffic,
                        "bytes_per_launch": int(res_bytes), "avg_launch_ms": round(res_ms, 5),
                        "tables_per_launch": tables_per_launch // launches_per_span,
                        "launches_per_event_span": launches_per_span}
    stages = {k: round(v, 4) for k, v in stage_ms.items()}
    stages["encode_only_GBps_table_bytes"] = round(table_bytes / ((stage_ms["compact"] + stage_ms["encode"]) * 1e-3) / 1e9, 1)
    stages["restore_hbm_GBps"] = round(res_bytes / (res_ms * 1e-3) / 1e9, 1)
    stages["mark_Gidx_per_s"] = round(sum(s.numel() for s in streams) / (stage_ms["mark"] * 1e-3) / 1e9, 2)

    if w.lookups == "bernoulli":
        lookups_desc = "Bernoulli(%.2f) row selection with repeats" % w.dirty_fraction
    else:
        per = "%d x %d" % (w.batch, w.pooling) if w.lookups == "zipf_batches" else "%d" % (streams[0].numel() // iters_run[0])
        stop = ("--iterations %d" % args.iterations if args.iterations > 0 else
                "stopped at %.0f%% coverage" % (100 * w.dirty_fraction) if w.dirty_fraction else "the workload's count")
        lookups_desc = "Zipf(%.2f) look-ups, %d-%d iterations of %s per table (%s)" % (
            w.zipf_s, min(iters_run), max(iters_run), per, stop)
    out = {
        "metric": "checkpoint encode GB/s (fp32 table bytes)", "value": round(value, 1), "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": "%s: %d tables x %d rows x dim %d, %s values, %s, %.1f%% dirty, %d-bit min/max "
                               "range, step = clear+mark+compact+encode+restore of all tables, %s"
                               % (w.name, n_tables, w.n_rows, w.dim, w.values, lookups_desc,
                                  100.0 * sum(n_dirty) / (n_tables * w.n_rows), bits,
                                  "one batched call per stage" if batched else "one call per table and stage"),
                   "dirty_rows": sum(n_dirty), "lookups_per_step": int(sum(s.numel() for s in streams)),
                   "index_dtype": "int64"},
        "roofline": roofline,
        "roofline_restore": roofline_restore,
        "stages_ms_per_step": stages,
    }

    # ---- a launch-bound step replayed from a HIP graph (the calls only enqueue kernels, so a step can be
    #      captured once): reported where the eager step is short enough for launch overhead to matter
    if ms_per_step < 0.5:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step(None, ())
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):                           # the calls are prepared on the capturing stream
            if batched:
                gcalls = batch.prepare_step(streams, tables, encs, restore_into=stale)
            else:
                gcalls = []
                for ti in range(n_tables):
                    gcalls += cks[ti].prepare_step(streams[ti], tables[ti], encs[ti], restore_into=stale[0])
            for _, fn in gcalls:
                fn()
        for _ in range(max(3, args.warmup)):
            graph.replay()
        torch.cuda.synchronize()
        reps = max(args.steps, 200)
        t0 = time.perf_counter()
        for _ in range(reps):
            graph.replay()
        torch.cuda.synchronize()
        g_ms = (time.perf_counter() - t0) * 1e3 / reps
        assert [int(c.n_dirty.item()) for c in cks] == n_dirty
        out["graph_replay"] = {"ms_per_step": round(g_ms, 4), "value": round(table_bytes / (g_ms * 1e-3) / 1e9, 1),
                               "unit": "GB/s", "replays": reps}

    # ---- context for the roofline: what a plain device-to-device copy reaches on this machine -----------
    src = torch.empty(1 << 28, dtype=torch.float32, device=dev).fill_(1.0)
    dst = torch.empty_like(src)
    dst.copy_(src)
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(5):
        dst.copy_(src)
    b.record()
    torch.cuda.synchronize()
    out["roofline"]["copy_ceiling_GBps"] = round(5 * 2 * src.numel() * 4 / (a.elapsed_time(b) * 1e-3) / 1e9, 1)
    del src, dst

    # ---- marking as training issues it: one short index stream per table and iteration -------------
    per_iter = 40960                                            # 2048 x 20 look-ups (configuration 2)
    small = [s_[:per_iter].contiguous() for s_ in streams]
    if batched:
        small_batched = B_prepare_mark(batch, small)
    small_single = [P.prepare("cnr_mark_touched", ctx, cks[ti].bitmap, w.n_rows, small[ti], per_iter, P.CNR_IDX_I64,
                              None, None) for ti in range(n_tables)]

    def time_calls(fns, reps=50):
        for f in fns:
            f()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            for f in fns:
                f()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / reps * 1e6
    mark_us = {"per_table_calls_us": round(time_calls(small_single), 2)}
    if batched:
        mark_us["batched_call_us"] = round(time_calls([small_batched]), 2)
    out["mark_per_iteration"] = dict(workload="%d tables x %d int64 look-ups per iteration into %d-row bitmaps"
                                              % (n_tables, per_iter, w.n_rows), **mark_us)

    # ---- greedy range search on the same tables (ALU-bound) ---------------------------------------
    if not args.no_greedy and w.num_bins:
        g_ms = []
        for rep in range(2):
            a = torch.cuda.Event(enable_timing=True)
            b = torch.cuda.Event(enable_timing=True)
            a.record()
            if batched:
                batch.encode(tables, encs, mode=P.CNR_RANGE_GREEDY, greedy=(w.num_bins, w.ratio))
            else:
                for ti in range(n_tables):
                    cks[ti].encode(tables[ti], encs[ti], mode=P.CNR_RANGE_GREEDY, greedy=(w.num_bins, w.ratio))
            b.record()
            torch.cuda.synchronize()
            g_ms.append(a.elapsed_time(b))
        g = min(g_ms)
        n_iter = P.cnr_greedy_iterations(w.num_bins, w.ratio)
        # arithmetic the search itself prescribes, per element and candidate range: clip (2), subtract,
        # divide, round, multiply, add, subtract, square, accumulate = 10
        flops = sum(n_dirty) * w.dim * (1 + 2 * n_iter) * 10.0
        issue_ms = sum(n_dirty) * w.dim * (1 + 2 * n_iter) / 64.0 * GREEDY_SIMD_CLOCKS_PER_ELEMENT / SIMD_CLOCKS_PER_S * 1e3
        out["greedy"] = {
            "workload": "%d-bit greedy range, num_bins=%d, ratio=%.2f (%d candidate ranges per row)"
                        % (bits, w.num_bins, w.ratio, 1 + 2 * n_iter),
            "ms": round(g, 3), "value": round(table_bytes / (g * 1e-3) / 1e9, 2), "unit": "GB/s",
            "roofline": {"bound": "alu", "achieved": round(flops / (g * 1e-3) / 1e12, 2),
                         "peak": FP32_VECTOR_PEAK_TFLOPS, "unit": "TFLOP/s",
                         "frac": round(flops / (g * 1e-3) / 1e12 / FP32_VECTOR_PEAK_TFLOPS, 4),
                         # the same launch against the time its own instruction mix needs at full issue rate
                         "issue_bound_ms": round(issue_ms, 3), "issue_frac": round(issue_ms / g, 4), "traffic": None},
        }

    # ---- a full (baseline) checkpoint: every row of a table, no id list (Section 5.1) ---------------
    if not args.no_full:
        prb = P.cnr_packed_row_bytes(w.dim, bits)
        f_scale = torch.empty(w.n_rows, dtype=torch.float32, device=dev)
        f_bias = torch.empty(w.n_rows, dtype=torch.float32, device=dev)
        f_packed = torch.empty(w.n_rows * prb, dtype=torch.uint8, device=dev)
        full = {}
        for label in ("encode", "restore"):
            def run(ti):
                if label == "encode":
                    P.cnr_quantize_rows(ctx, tables[ti], w.n_rows, w.dim, None, None, w.n_rows, bits,
                                        P.CNR_RANGE_MINMAX, None, f_scale, f_bias, None, None, None, f_packed, None)
                else:
                    P.cnr_restore_rows(ctx, stale[ti % len(stale)], w.n_rows, w.dim, None, None, w.n_rows, bits,
                                       f_packed, f_scale, f_bias, None)
            run(0)
            torch.cuda.synchronize()
            a = torch.cuda.Event(enable_timing=True)
            b = torch.cuda.Event(enable_timing=True)
            reps = 5
            a.record()
            for r in range(reps):
                run((r + 1) % n_tables)
            b.record()
            torch.cuda.synchronize()
            full[label] = a.elapsed_time(b) / reps
        row_bytes = 4 * w.dim + prb + 8
        out["full_checkpoint"] = {
            "workload": "all %d rows of one table, %d-bit min/max, no id list" % (w.n_rows, bits),
            "encode_ms": round(full["encode"], 4), "restore_ms": round(full["restore"], 4),
            "encode_GBps_table_bytes": round(w.n_rows * w.dim * 4 / (full["encode"] * 1e-3) / 1e9, 1),
            "encode_hbm_GBps": round(w.n_rows * row_bytes / (full["encode"] * 1e-3) / 1e9, 1),
            "restore_hbm_GBps": round(w.n_rows * row_bytes / (full["restore"] * 1e-3) / 1e9, 1)}
        del f_scale, f_bias, f_packed

    # ---- chunked encode with the device-to-host copy overlapped (what follows the path) -----------
    if not args.no_host_copy:
        writer = P.HostCheckpointWriter(ctx, w.dim, bits, capacity=w.n_rows, chunk_rows=1 << 20, device=dev)
        cks[0].clear(); cks[0].mark(streams[0]); cks[0].compact()
        def median_s(fn, reps=7, warm=1):
            """Median and largest wall time of `reps` calls (each call ends synchronized), after `warm`
            untimed ones; the largest of those is returned as well."""
            warm_ts = []
            for _ in range(warm):
                t0 = time.perf_counter()
                fn()
                warm_ts.append(time.perf_counter() - t0)
            ts = []
            for _ in range(reps):
                t0 = time.perf_counter()
                fn()
                ts.append(time.perf_counter() - t0)
            ts.sort()
            return ts[len(ts) // 2], ts[-1], max(warm_ts)
        res, back, n_h = {}, {}, 0
        for label, overlap in (("direct", P.CNR_HOST_DIRECT), ("overlapped", P.CNR_HOST_OVERLAP),
                               ("serialized", P.CNR_HOST_SERIAL)):
            def to_host():
                nonlocal n_h
                n_h = writer.encode_to_host(cks[0], tables[0], overlap=overlap)
            res[label] = median_s(to_host)
        # and the way back: the same chunks from host memory into the stale table.  The first dozen or so
        # overlapped calls of a process can contain one that takes 4-10 ms (the host blocks once inside
        # the runtime's hipMemcpyAsync while it sets up the second stream's copy path, the GPU idle
        # meanwhile; it does not recur), so 16 calls run untimed first and their slowest is reported apart.
        # The direct way (the restore kernel reads the pinned buffers itself) has no copies at all.
        for label, overlap in (("direct", P.CNR_HOST_DIRECT), ("overlapped", P.CNR_HOST_OVERLAP),
                               ("serialized", P.CNR_HOST_SERIAL)):
            back[label] = median_s(lambda: writer.restore_from_host(stale[0], w.n_rows, n_h, overlap=overlap), reps=50, warm=16)
        # `value` is the way the writer takes by default for this row length
        to_path = "direct" if writer._to_host_path(None) == P.CNR_HOST_DIRECT else "overlapped"
        out["to_host"] = {"workload": "table 0: %d dirty rows encoded into pinned host memory, by the encode kernel's "
                                      "own stores (direct) or in chunks of %d rows with staged copies; median of 7 "
                                      "calls" % (n_h, writer.chunk),
                          "direct_ms": round(res["direct"][0] * 1e3, 3),
                          "overlapped_ms": round(res["overlapped"][0] * 1e3, 3),
                          "serialized_ms": round(res["serialized"][0] * 1e3, 3),
                          "slowest_call_ms": round(max(r[1] for r in res.values()) * 1e3, 3),
                          "path": to_path,
                          "host_link_GBps": round(n_h * (12 + writer.prb) / res[to_path][0] / 1e9, 1),
                          "value": round(n_h * w.dim * 4 / res[to_path][0] / 1e9, 1), "unit": "GB/s",
                          "host_bytes": int(n_h * (12 + writer.prb))}
        out["from_host"] = {"workload": "table 0: the same %d rows restored from pinned host memory, read by the "
                                        "restore kernel itself (direct) or copied in chunks of %d rows first; median "
                                        "of 50 calls after 16 untimed ones" % (n_h, writer.chunk),
                            "direct_ms": round(back["direct"][0] * 1e3, 3),
                            "overlapped_ms": round(back["overlapped"][0] * 1e3, 3),
                            "serialized_ms": round(back["serialized"][0] * 1e3, 3),
                            "slowest_call_ms": round(max(b[1] for b in back.values()) * 1e3, 3),
                            "slowest_direct_call_ms": round(max(back["direct"][1], back["direct"][2]) * 1e3, 3),
                            "slowest_warmup_call_ms": round(max(b[2] for b in back.values()) * 1e3, 3),
                            "host_link_GBps": round(n_h * (12 + writer.prb) / back["direct"][0] / 1e9, 1),
                            "value": round(n_h * w.dim * 4 / back["direct"][0] / 1e9, 1), "unit": "GB/s"}
        del writer

    # ---- CPU oracle on a bounded sample -----------------------------------------------------------
    if not args.no_cpu:
        import oracle as O
        threads = int(os.environ.get("OMP_NUM_THREADS", "0")) or (os.cpu_count() or 1)
        threads = max(1, min(threads, os.cpu_count() or 1))
        n_cpu_tables = min(n_tables, 4)
        cpu_s, cpu_rows = 0.0, 0
        for ti in range(n_cpu_tables):
            host_table = tables[ti].cpu().numpy()
            host_idx = streams[ti].cpu().numpy()
            t0 = time.perf_counter()
            bm = O.new_bitmap(w.n_rows)
            O.mark_touched(bm, w.n_rows, host_idx)
            ids, n = O.compact_dirty(bm, w.n_rows)
            q = O.quantize_rows(host_table, ids, bits, n_threads=threads)
            packed = O.pack(q["codes"], bits)
            host_stale = np.zeros_like(host_table)
            O.restore_rows(host_stale, ids, bits, packed, q["scale"], q["bias"], n_threads=threads)
            cpu_s += time.perf_counter() - t0
            cpu_rows += n
            assert n == n_dirty[ti]
            if ti + 1 < n_cpu_tables:
                del host_table, host_stale, q, packed
        out["cpu_baseline"] = {"value": round(cpu_rows * w.dim * 4 / cpu_s / 1e9, 4), "unit": "GB/s", "cores": threads,
                               "kind": "oracle", "seconds": round(cpu_s, 2),
                               "sample": "tables 0-%d of %d (%d rows each, %d dirty in all): mark+compact+%d-bit "
                                         "min/max quantize+pack+restore; quantize and restore on %d threads, "
                                         "the rest on one" % (n_cpu_tables - 1, n_tables, w.n_rows, cpu_rows, bits, threads)}
        # the same oracle on one thread, on a smaller sample of the last table's dirty rows
        m1 = min(n, 200_000)
        t0 = time.perf_counter()
        q1 = O.quantize_rows(host_table, ids[:m1], bits, n_threads=1)
        pk1 = O.pack(q1["codes"], bits)
        O.restore_rows(host_stale, ids[:m1], bits, pk1, q1["scale"], q1["bias"], n_threads=1)
        s1 = time.perf_counter() - t0
        out["cpu_baseline"]["one_thread"] = {"value": round(m1 * w.dim * 4 / s1 / 1e9, 4), "unit": "GB/s", "cores": 1,
                                             "sample": "quantize+pack+restore of the first %d dirty rows of table %d"
                                                       % (m1, n_cpu_tables - 1)}
        del q1, pk1
        ti = n_cpu_tables - 1
        # the GPU result for the same table must be what the oracle produced
        cks[ti].clear(); cks[ti].mark(streams[ti]); cks[ti].compact(); cks[ti].encode(tables[ti], encs[ti])
        torch.cuda.synchronize()
        assert np.array_equal(encs[ti].row_ids.cpu().numpy().view(np.uint32)[:n], ids)
        assert np.array_equal(encs[ti].scale.cpu().numpy()[:n], q["scale"])
        gp = encs[ti].packed.cpu().numpy()[:n * packed.shape[1]].reshape(n, -1)
        assert np.mean(gp != packed) <= 1e-4
        if "greedy" in out:
            m = min(n, 20000)
            t0 = time.perf_counter()
            O.quantize_rows(host_table, ids[:m], bits, mode=O.RANGE_GREEDY, num_bins=w.num_bins,
                            ratio=w.ratio, n_threads=threads, want_codes=False)
            gs = time.perf_counter() - t0
            out["greedy"]["cpu_baseline"] = {"value": round(m * w.dim * 4 / gs / 1e9, 5), "unit": "GB/s",
                                             "cores": threads, "kind": "oracle",
                                             "sample": "first %d dirty rows of table %d" % (m, ti)}

    P.cnr_destroy(ctx)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
