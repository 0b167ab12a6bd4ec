"""GPU parity of the several-tables-per-launch calls: every table of a batch against the CPU oracle,
and against the single-table calls bit for bit."""
import numpy as np
import pytest
import torch

import oracle as O
import paper_2010_08679_amd as P
from paper_2010_08679_amd import synth
from util_parity import compare_quantized, u32

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
BITS = (2, 3, 4, 8)


@pytest.fixture(scope="module")
def ctx():
    c = P.cnr_create(0)
    yield c
    torch.cuda.synchronize()
    P.cnr_destroy(c)


def _poll_clean(ctx):
    assert P.cnr_poll_errors(ctx) == (P.CNR_OK, 0, 0)


class _Tables:
    """A few tables of one row length with ragged sizes, their look-up streams, and both per-table
    and batched checkpointers on the same kind of buffers."""

    def __init__(self, ctx, sizes, dim, seed, n_idx, with_scratch=True, idx_dtype=torch.int64):
        g = torch.Generator(device=DEV).manual_seed(seed)
        self.sizes, self.dim = sizes, dim
        self.tables = [synth.table_outlier_mix(n, dim, 0.02, seed * 100 + i, DEV) for i, n in enumerate(sizes)]
        self.host = [t.cpu().numpy() for t in self.tables]
        self.idx = [None if m == 0 else torch.randint(0, n, (m,), generator=g, device=DEV).to(idx_dtype)
                    for n, m in zip(sizes, n_idx)]

        def cks():
            return [P.TableCheckpointer(ctx, n, dim, device=DEV,
                                        mark_scratch=P.TableCheckpointer.new_mark_scratch(n, DEV) if with_scratch else None)
                    for n in sizes]
        self.single, self.batched = cks(), cks()
        self.batch = P.BatchCheckpointer(ctx, self.batched)

    def oracle_track(self, i):
        bm = O.new_bitmap(self.sizes[i])
        if self.idx[i] is not None:
            O.mark_touched(bm, self.sizes[i], self.idx[i].cpu().numpy())
        ids, n = O.compact_dirty(bm, self.sizes[i])
        return bm, ids, n


def _outputs(cks, bits):
    return [c.alloc_output(bits, want_range=True) for c in cks]


def _host(enc, n, dim, bits):
    prb = P.cnr_packed_row_bytes(dim, bits)
    packed = enc.packed.cpu().numpy()[:n * prb].reshape(n, prb)
    return dict(scale=enc.scale.cpu().numpy()[:n], bias=enc.bias.cpu().numpy()[:n],
                row_min=enc.row_min.cpu().numpy()[:n], row_max=enc.row_max.cpu().numpy()[:n],
                packed=packed, codes=O.unpack(packed, dim, bits))


# small tables share one encode / restore launch, a table of more than 64 MB takes its own
SIZES = {"small": ([70_001, 5_000, 33, 16_384, 1], [300_000, 2_000, 0, 9_000, 3]),   # look-ups: bulk, atomic, none, ...
         "mixed": ([5_000, 300_007, 40_000, 140_000], [4_000, 200_000, 30_000, 90_000])}


@pytest.mark.parametrize("bits", BITS)
@pytest.mark.parametrize("dim,which", [(64, "small"), (128, "small"), (64, "mixed"), (256, "mixed"), (32, "small")])
def test_batched_checkpoint_equals_oracle_and_single_calls(ctx, bits, dim, which):
    sizes, n_idx = SIZES[which]
    print("case batch %s dim=%d bits=%d" % (which, dim, bits), flush=True)
    T = _Tables(ctx, sizes, dim, seed=bits * 10 + dim, n_idx=n_idx)
    # --- batched path
    T.batch.clear()
    T.batch.mark(T.idx)
    T.batch.compact()
    outs_b = _outputs(T.batched, bits)
    T.batch.encode(T.tables, outs_b)
    stale_b = [torch.zeros_like(t) for t in T.tables]
    T.batch.restore(stale_b, outs_b)
    # --- the same through the single-table calls
    outs_s = _outputs(T.single, bits)
    stale_s = [torch.zeros_like(t) for t in T.tables]
    for c, idx, t, o, st in zip(T.single, T.idx, T.tables, outs_s, stale_s):
        c.clear()
        if idx is not None:
            c.mark(idx)
        c.compact()
        c.encode(t, o)
        c.restore(st, o)
    torch.cuda.synchronize()
    for i, n_rows in enumerate(sizes):
        bm, ids, n = T.oracle_track(i)
        cb, cs = T.batched[i], T.single[i]
        assert np.array_equal(u32(cb.bitmap)[:bm.size], bm), "table %d bitmap" % i
        assert int(cb.n_dirty.item()) == n and np.array_equal(u32(cb.row_ids)[:n], ids)
        if cb.mark_scratch is not None:
            assert not cb.mark_scratch.any()
        got = _host(outs_b[i], n, dim, bits)
        one = _host(outs_s[i], n, dim, bits)
        for k in ("scale", "bias", "row_min", "row_max", "packed"):
            assert np.array_equal(got[k], one[k]), "table %d %s differs from the single-table call" % (i, k)
        assert torch.equal(stale_b[i], stale_s[i])
        if n:
            ora = O.quantize_rows(T.host[i], ids, bits, n_threads=8)
            compare_quantized(T.host[i][ids], got, ora, bits, what="batch table %d b%d d%d" % (i, bits, dim))
            want = np.zeros_like(T.host[i])
            O.restore_rows(want, ids, bits, got["packed"], got["scale"], got["bias"])
            assert np.array_equal(stale_b[i].cpu().numpy(), want)
    _poll_clean(ctx)


@pytest.mark.parametrize("dtype", [torch.int64, torch.int32])
def test_batched_mark_takes_each_table_by_its_own_route(ctx, dtype):
    # one batch whose tables need all three routes of the mark: bitmap slices in LDS with teams of one,
    # two and three workgroups (four tables with long streams, so that the call's estimate favours the
    # slices for them), flag bytes for a table too large for that, atomics for short streams
    slice_rows = 32 * 40960
    sizes = [3 * slice_rows - 5, 100, 16 * slice_rows + 77, slice_rows + 1, 40_000, slice_rows, 2 * slice_rows + 3, slice_rows - 1]
    n_idx = [400_001, 50, 500_003, 300_000, 100, 0, 390_000, 380_003]
    print("case mixed-route mark dtype=%s" % dtype, flush=True)
    g = torch.Generator(device=DEV).manual_seed(77)
    cks = [P.TableCheckpointer(ctx, n, 16, device=DEV, mark_scratch=P.TableCheckpointer.new_mark_scratch(n, DEV))
           for n in sizes]
    batch = P.BatchCheckpointer(ctx, cks)
    idx = [None if m == 0 else torch.randint(-1, n + 1, (m,), generator=g, device=DEV).to(dtype)
           for n, m in zip(sizes, n_idx)]
    batch.clear()
    batch.mark(idx)
    batch.mark(idx)                                            # marks accumulate; the same streams again
    batch.compact()
    torch.cuda.synchronize()
    skipped = 0
    for i, n_rows in enumerate(sizes):
        bm = O.new_bitmap(n_rows)
        if idx[i] is not None:
            skipped += 2 * O.mark_touched(bm, n_rows, idx[i].cpu().numpy())
        ids, n = O.compact_dirty(bm, n_rows)
        assert np.array_equal(u32(cks[i].bitmap)[:bm.size], bm), "table %d bitmap" % i
        assert int(cks[i].n_dirty.item()) == n and np.array_equal(u32(cks[i].row_ids)[:n], ids)
        assert not cks[i].mark_scratch.any()
    st, bad, flags = P.cnr_poll_errors(ctx)
    assert st == P.CNR_E_INDEX_RANGE and bad == skipped and skipped > 0 and flags == 0
    _poll_clean(ctx)


@pytest.mark.parametrize("bits,dim", [(4, 64), (2, 128), (3, 256)])
def test_batched_greedy(ctx, bits, dim):
    sizes = [3_001, 700, 64]
    T = _Tables(ctx, sizes, dim, seed=7 + bits, n_idx=[2_500, 900, 64])
    T.batch.clear()
    T.batch.mark(T.idx)
    T.batch.compact()
    outs = _outputs(T.batched, bits)
    T.batch.encode(T.tables, outs, mode=P.CNR_RANGE_GREEDY, greedy=(20, 0.6))
    torch.cuda.synchronize()
    for i in range(len(sizes)):
        _, ids, n = T.oracle_track(i)
        got = _host(outs[i], n, dim, bits)
        ora = O.quantize_rows(T.host[i], ids, bits, mode=O.RANGE_GREEDY, num_bins=20, ratio=0.6, n_threads=8)
        compare_quantized(T.host[i][ids], got, ora, bits, greedy=True, what="batch greedy table %d" % i)
    _poll_clean(ctx)


def test_more_tables_than_one_launch_takes(ctx):
    n_tables = P.CNR_MAX_BATCH + 3
    sizes = [1_000 + 37 * i for i in range(n_tables)]
    T = _Tables(ctx, sizes, 64, seed=3, n_idx=[400 + i for i in range(n_tables)], with_scratch=False,
                idx_dtype=torch.int32)
    T.batch.clear()
    T.batch.mark(T.idx)
    T.batch.compact()
    outs = _outputs(T.batched, 4)
    T.batch.encode(T.tables, outs)
    stale = [torch.zeros_like(t) for t in T.tables]
    T.batch.restore(stale, outs)
    torch.cuda.synchronize()
    for i in range(n_tables):
        bm, ids, n = T.oracle_track(i)
        assert np.array_equal(u32(T.batched[i].bitmap)[:bm.size], bm)
        assert int(T.batched[i].n_dirty.item()) == n and np.array_equal(u32(T.batched[i].row_ids)[:n], ids)
        got = _host(outs[i], n, 64, 4)
        ora = O.quantize_rows(T.host[i], ids, 4)
        compare_quantized(T.host[i][ids], got, ora, 4, what="table %d of %d" % (i, n_tables))
        want = np.zeros_like(T.host[i])
        O.restore_rows(want, ids, 4, got["packed"], got["scale"], got["bias"])
        assert np.array_equal(stale[i].cpu().numpy(), want)
    _poll_clean(ctx)


def test_other_row_lengths_go_table_by_table(ctx):
    sizes = [900, 2_000]
    T = _Tables(ctx, sizes, 40, seed=11, n_idx=[500, 1_500])
    T.batch.clear()
    T.batch.mark(T.idx)
    T.batch.compact()
    outs = _outputs(T.batched, 4)
    T.batch.encode(T.tables, outs)
    stale = [torch.zeros_like(t) for t in T.tables]
    T.batch.restore(stale, outs)
    torch.cuda.synchronize()
    for i in range(2):
        _, ids, n = T.oracle_track(i)
        got = _host(outs[i], n, 40, 4)
        ora = O.quantize_rows(T.host[i], ids, 4)
        compare_quantized(T.host[i][ids], got, ora, 4, what="dim 40 table %d" % i)
        want = np.zeros_like(T.host[i])
        O.restore_rows(want, ids, 4, got["packed"], got["scale"], got["bias"])
        assert np.array_equal(stale[i].cpu().numpy(), want)
    _poll_clean(ctx)


def test_bad_job_rejects_the_whole_call_before_any_launch(ctx):
    T = _Tables(ctx, [2_000, 2_000], 64, seed=5, n_idx=[1_000, 1_000])
    T.batch.clear()
    torch.cuda.synchronize()
    jobs = T.batch.jobs(indices=T.idx)
    jobs[1].n_rows = 1 << 32
    with pytest.raises(P.CnrError) as e:
        P.cnr_mark_touched_batch(ctx, jobs, P.CNR_IDX_I64)
    assert e.value.status == P.CNR_E_INVALID
    jobs = T.batch.jobs(indices=T.idx)
    jobs[1].indices += 4                                       # int64 stream at a 4-byte boundary
    with pytest.raises(P.CnrError) as e:
        P.cnr_mark_touched_batch(ctx, jobs, P.CNR_IDX_I64)
    assert e.value.status == P.CNR_E_ALIGN
    torch.cuda.synchronize()
    assert not T.batched[0].bitmap.any() and not T.batched[1].bitmap.any()
    outs = _outputs(T.batched, 4)
    with pytest.raises(P.CnrError) as e:
        P.cnr_quantize_rows_batch(ctx, T.batch.jobs(tables=T.tables, outs=outs), 64, 5, P.CNR_RANGE_MINMAX)
    assert e.value.status == P.CNR_E_BITS
    with pytest.raises(P.CnrError) as e:
        P.cnr_restore_rows_batch(ctx, T.batch.jobs(tables=T.tables, outs=outs), 12, 3)
    assert e.value.status == P.CNR_E_DIM
    _poll_clean(ctx)


def test_capacity_overflow_in_one_table_of_a_batch(ctx):
    sizes = [4_000, 4_000]
    cks = [P.TableCheckpointer(ctx, sizes[0], 64, device=DEV),
           P.TableCheckpointer(ctx, sizes[1], 64, capacity=100, device=DEV)]
    batch = P.BatchCheckpointer(ctx, cks)
    g = torch.Generator(device=DEV).manual_seed(9)
    idx = [torch.randint(0, n, (3_000,), generator=g, device=DEV) for n in sizes]
    batch.clear()
    batch.mark(idx)
    cks[1].row_ids.fill_(-1)
    batch.compact()
    st, bad, flags = P.cnr_poll_errors(ctx)
    assert st == P.CNR_E_CAPACITY and flags == P.CNR_FLAG_CAPACITY and bad == 0
    for c, ix in zip(cks, idx):
        bm = O.new_bitmap(c.n_rows)
        O.mark_touched(bm, c.n_rows, ix.cpu().numpy())
        ids, n = O.compact_dirty(bm, c.n_rows)
        assert int(c.n_dirty.item()) == n                      # the true count, also when truncated
        m = min(n, c.capacity)
        assert np.array_equal(u32(c.row_ids)[:m], ids[:m])
    _poll_clean(ctx)


def test_batched_step_replays_from_a_hip_graph(ctx):
    # the batched calls only enqueue kernels on the caller's stream (job descriptors travel by value in
    # the launch), so a whole step over several tables can be captured once and replayed; inputs are
    # refreshed in place between replays and every replay is checked against the oracle
    sizes, dim, bits = [90_001, 20_000, 50], 64, 4
    T = _Tables(ctx, sizes, dim, seed=21, n_idx=[200_000, 5_000, 40])
    outs = _outputs(T.batched, bits)
    stale = [torch.zeros_like(t) for t in T.tables]

    def step():                                                 # prepared calls hold the stream that is
        for _, call in T.batch.prepare_step(T.idx, T.tables, outs, restore_into=stale):  # current here
            call()

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                                  # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    g = torch.Generator(device=DEV).manual_seed(77)
    for rep in range(3):
        for i, n_rows in enumerate(sizes):                      # eager work between the replays
            T.idx[i].copy_(torch.randint(0, n_rows, (T.idx[i].numel(),), generator=g, device=DEV))
            T.tables[i].mul_(1.0 + 0.1 * (rep + 1))
            stale[i].fill_(float(rep))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for i, n_rows in enumerate(sizes):
            host = T.tables[i].cpu().numpy()
            _, ids, n = T.oracle_track(i)
            c = T.batched[i]
            assert int(c.n_dirty.item()) == n and np.array_equal(u32(c.row_ids)[:n], ids)
            got = _host(outs[i], n, dim, bits)
            ora = O.quantize_rows(host, ids, bits, n_threads=8)
            compare_quantized(host[ids], got, ora, bits, what="replay %d table %d" % (rep, i))
            want = np.full_like(host, float(rep))
            O.restore_rows(want, ids, bits, got["packed"], got["scale"], got["bias"])
            assert np.array_equal(stale[i].cpu().numpy(), want)
            assert not c.mark_scratch.any()
    _poll_clean(ctx)
