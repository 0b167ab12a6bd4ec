"""GPU parity at the full sizes of the benchmark configurations, in the launch configurations the
benchmark times: one prepared batched call per stage over all tables (its default), and prepared
per-table calls with a shared scratch for marking; device-side row counts in both.
The tracking bitmap and the dirty-row list are compared in full; the encoded rows on a sample the
oracle can quantize row by row (every position of the first and last wave batches plus a random
draw); restored tables on the same sample plus rows that must stay untouched."""
import numpy as np
import pytest
import torch

import oracle as O
import paper_2010_08679_amd as P
from paper_2010_08679_amd import synth
from util_parity import compare_quantized, u32

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def ctx():
    c = P.cnr_create(0)
    yield c
    torch.cuda.synchronize()
    P.cnr_destroy(c)


def _sample_positions(n, count, seed):
    rng = np.random.default_rng(seed)
    edge = np.concatenate([np.arange(min(n, 64)), np.arange(max(0, n - 64), n)])
    rnd = rng.integers(0, n, size=count)
    return np.unique(np.concatenate([edge, rnd])).astype(np.int64)


def _encoded_sample(enc, pos, dim, bits):
    """Host copies of the GPU outputs at dirty-list positions ``pos``."""
    p = torch.from_numpy(pos).to(DEV)
    prb = P.cnr_packed_row_bytes(dim, bits)
    packed = enc.packed.reshape(-1, prb).index_select(0, p).cpu().numpy()
    out = dict(scale=enc.scale.index_select(0, p).cpu().numpy(), bias=enc.bias.index_select(0, p).cpu().numpy(),
               packed=packed, codes=O.unpack(packed, dim, bits))
    if enc.row_min is not None:
        out["row_min"] = enc.row_min.index_select(0, p).cpu().numpy()
        out["row_max"] = enc.row_max.index_select(0, p).cpu().numpy()
    return out


def _check_table(ctx, w, table, batches, bits_list, greedy=None, sample=100_000, greedy_sample=None,
                 scratch=None, what=""):
    n_rows, dim = table.shape
    ck = P.TableCheckpointer(ctx, n_rows, dim, device=DEV, mark_scratch=scratch)
    bm = O.new_bitmap(n_rows)
    ck.clear()
    for b in batches:                       # batches may be a generator that looks at ck (coverage)
        ck.mark(b)
        O.mark_touched(bm, n_rows, b.cpu().numpy())
    ck.compact()
    torch.cuda.synchronize()
    ids, n = O.compact_dirty(bm, n_rows)
    assert np.array_equal(u32(ck.bitmap)[:bm.size], bm), what + " bitmap"
    assert int(ck.n_dirty.item()) == n, what + " dirty count"
    assert np.array_equal(u32(ck.row_ids)[:n], ids), what + " dirty list"
    print("%s: %d of %d rows dirty (%.1f %%)" % (what, n, n_rows, 100.0 * n / n_rows), flush=True)

    pos = _sample_positions(n, sample, 1)
    rows_t = table.index_select(0, torch.from_numpy(ids[pos].astype(np.int64)).to(DEV))
    rows = rows_t.cpu().numpy()
    stale = torch.full_like(table, -3.0)      # one reusable stale table, whatever the size (up to 20.5 GB)
    for bits in bits_list:
        enc = ck.alloc_output(bits, want_range=True)
        for _, call in ck.prepare_step(torch.zeros(1, dtype=torch.int64, device=DEV), table, enc)[3:]:
            call()                          # the prepared encode launch, as the benchmark issues it
        torch.cuda.synchronize()
        got = _encoded_sample(enc, pos, dim, bits)
        ora = O.quantize_rows(rows, None, bits, n_threads=8)
        compare_quantized(rows, got, ora, bits, what="%s b%d" % (what, bits))
        ck.restore(stale, enc)
        torch.cuda.synchronize()
        back = stale.index_select(0, torch.from_numpy(ids[pos].astype(np.int64)).to(DEV)).cpu().numpy()
        assert np.array_equal(back, O.dequantize(got["codes"], got["scale"], got["bias"])), what + " restore"
        untouched = np.setdiff1d(np.arange(0, n_rows, max(1, n_rows // 50_000)), ids)
        assert torch.all(stale.index_select(0, torch.from_numpy(untouched).to(DEV)) == -3.0)
        # every listed row was written and no other: the restored table differs from the stale fill in
        # exactly the dirty rows (a row of a real table never de-quantizes to -3.0 throughout)
        assert int((stale != -3.0).any(dim=1).sum().item()) == n, what + " rows written"
        stale.fill_(-3.0)
        if greedy is not None:
            # the whole sample when greedy_sample is None (>= 100,000 rows: enough to resolve the 1e-4 bars)
            gpos = pos if greedy_sample is None else pos[:: max(1, len(pos) // greedy_sample)]
            ck.encode(table, enc, mode=P.CNR_RANGE_GREEDY, greedy=greedy)
            torch.cuda.synchronize()
            sel = np.searchsorted(pos, gpos)
            got_g = _encoded_sample(enc, gpos, dim, bits)
            ora_g = O.quantize_rows(rows[sel], None, bits, mode=O.RANGE_GREEDY, num_bins=greedy[0],
                                    ratio=greedy[1], n_threads=8)
            compare_quantized(rows[sel], got_g, ora_g, bits, greedy=True, what="%s greedy b%d" % (what, bits))
    st, bad, flags = P.cnr_poll_errors(ctx)
    assert (st, bad, flags) == (P.CNR_OK, 0, 0)


def test_cfg4_table_full_size(ctx):
    w = synth.WORKLOADS["cfg4"]
    table = synth.make_table(w, 0, 4, DEV)
    scratch = P.TableCheckpointer.new_mark_scratch(w.n_rows, DEV)
    _check_table(ctx, w, table, list(synth.lookup_batches(w, 0, 4, DEV)), (4,), greedy=(w.num_bins, w.ratio),
                 sample=125_000, scratch=scratch, what="cfg4 table 0")
    assert not scratch.any()


def test_table_beyond_4GB_addresses(ctx):
    # 9.5 M rows x 128 floats = 4.9 GB: row offsets pass 2^32 bytes; dirty rows cluster at the far end
    n_rows, dim = 9_500_000, 128
    table = synth.table_normal(n_rows, dim, 0.05, 77, DEV)
    g = torch.Generator(device=DEV).manual_seed(3)
    tail = torch.randint(n_rows - 600_000, n_rows, (400_000,), generator=g, device=DEV)
    head = torch.randint(0, n_rows, (100_000,), generator=g, device=DEV)
    w = synth.WORKLOADS["cfg3"]
    _check_table(ctx, w, table, [tail, head], (2, 3), sample=60_000, what="4.9 GB table")


def test_cfg3_table_zipf_until_coverage(ctx):
    # configuration 3 at full shape: 40 M x 128 (20.5 GB); Zipf(1.2) rounds of 16 M look-ups, marked
    # with the kernel under test, until 10 % of the rows are dirty (bounded at 64 rounds)
    w = synth.WORKLOADS["cfg3"]
    table = synth.make_table(w, 0, 3, DEV)
    scratch = P.TableCheckpointer.new_mark_scratch(w.n_rows, DEV)
    probe = P.TableCheckpointer(ctx, w.n_rows, w.dim, device=DEV, mark_scratch=scratch)
    probe.clear()
    rounds = []
    for idx in synth.lookup_batches(w, 0, 3, DEV, iterations=64):
        rounds.append(idx)
        probe.mark(idx)
        probe.compact()
        if int(probe.n_dirty.item()) >= w.dirty_fraction * w.n_rows:
            break
    del probe
    _check_table(ctx, w, table, rounds, (2, 3), sample=60_000, scratch=scratch, what="cfg3 table")


def test_cfg5_table_8bit_and_4bit(ctx):
    # one of configuration 5's twelve tables (32 M x 128, 16.4 GB), all 1000 iterations of 4,096 x 32 look-ups
    w = synth.WORKLOADS["cfg5"]
    table = synth.make_table(w, 0, 5, DEV)
    batches = list(synth.lookup_batches(w, 0, 5, DEV, iterations=1000))
    _check_table(ctx, w, table, batches, (8, 4), sample=60_000, what="cfg5 table 0")


def test_cfg4_all_tables_through_the_batched_calls(ctx):
    # the launch configuration the benchmark times by default: all eight tables of configuration 4
    # through one prepared batched call per stage, each table with a flag-byte scratch and a stale
    # table of its own
    w = synth.WORKLOADS["cfg4"]
    bits, seed = 4, 4
    tables = [synth.make_table(w, ti, seed, DEV) for ti in range(w.n_tables)]
    streams = [torch.cat([b.reshape(-1) for b in synth.lookup_batches(w, ti, seed, DEV)]) for ti in range(w.n_tables)]
    cks = [P.TableCheckpointer(ctx, w.n_rows, w.dim, device=DEV,
                               mark_scratch=P.TableCheckpointer.new_mark_scratch(w.n_rows, DEV))
           for _ in range(w.n_tables)]
    encs = [c.alloc_output(bits, want_range=True) for c in cks]
    stale = [torch.full_like(t, -3.0) for t in tables]
    batch = P.BatchCheckpointer(ctx, cks)
    for _ in range(2):                                          # a second step must give the same result
        for _, call in batch.prepare_step(streams, tables, encs, restore_into=stale):
            call()
    torch.cuda.synchronize()
    for ti in range(w.n_tables):
        what = "cfg4 batched table %d" % ti
        bm = O.new_bitmap(w.n_rows)
        O.mark_touched(bm, w.n_rows, streams[ti].cpu().numpy())
        ids, n = O.compact_dirty(bm, w.n_rows)
        assert np.array_equal(u32(cks[ti].bitmap)[:bm.size], bm), what + " bitmap"
        assert int(cks[ti].n_dirty.item()) == n and np.array_equal(u32(cks[ti].row_ids)[:n], ids), what
        assert not cks[ti].mark_scratch.any()
        pos = _sample_positions(n, 30_000, ti)
        sel = torch.from_numpy(ids[pos].astype(np.int64)).to(DEV)
        rows = tables[ti].index_select(0, sel).cpu().numpy()
        got = _encoded_sample(encs[ti], pos, w.dim, bits)
        ora = O.quantize_rows(rows, None, bits, n_threads=8)
        compare_quantized(rows, got, ora, bits, what=what)
        back = stale[ti].index_select(0, sel).cpu().numpy()
        assert np.array_equal(back, O.dequantize(got["codes"], got["scale"], got["bias"])), what + " restore"
        untouched = np.setdiff1d(np.arange(0, w.n_rows, 100), ids)
        assert torch.all(stale[ti].index_select(0, torch.from_numpy(untouched).to(DEV)) == -3.0)
    st, bad, flags = P.cnr_poll_errors(ctx)
    assert (st, bad, flags) == (P.CNR_OK, 0, 0)


@pytest.mark.parametrize("with_ids", [False, True])
def test_host_counted_lists_are_encoded_and_restored_in_slices(ctx, with_ids):
    # A list whose length the host passes (no count on the device) is cut into several launches; with no
    # id list either, that is a full checkpoint of the table.  The result must be, bit for bit, what the
    # single launch over a device-side count gives, and the oracle's on a sample that includes the rows
    # on either side of every cut.
    n_rows, dim, bits = 4_000_037, 64, 4
    print("case sliced launches with_ids=%s" % with_ids, flush=True)
    table = synth.table_outlier_mix(n_rows, dim, 0.02, 9, DEV)
    if with_ids:
        g = torch.Generator(device=DEV).manual_seed(3)
        ids = torch.nonzero(torch.rand(n_rows, generator=g, device=DEV) < 0.85).reshape(-1).to(torch.int32)
        n = ids.numel()
    else:
        ids, n = None, n_rows
    target = ((512 << 20) // (4 * dim)) & ~1023
    assert n > target + target // 2                            # long enough to be cut
    n_slices = -(-n // target)
    step = (-(-n // n_slices) + 1023) & ~1023
    prb = P.cnr_packed_row_bytes(dim, bits)
    n_dev = torch.tensor([n], dtype=torch.int64, device=DEV)

    def outputs():
        f = lambda: torch.full((n,), -1.0, dtype=torch.float32, device=DEV)  # noqa: E731
        return dict(scale=f(), bias=f(), row_min=f(), row_max=f(),
                    packed=torch.zeros(n * prb, dtype=torch.uint8, device=DEV))
    cut, one = outputs(), outputs()
    for o, count in ((cut, None), (one, n_dev)):
        P.cnr_quantize_rows(ctx, table, n_rows, dim, ids, count, n, bits, P.CNR_RANGE_MINMAX, None,
                            o["scale"], o["bias"], o["row_min"], o["row_max"], None, o["packed"], None)
    torch.cuda.synchronize()
    for k in cut:
        assert torch.equal(cut[k], one[k]), k

    edges = np.concatenate([np.arange(c - 3, c + 3) for c in range(step, n, step)])
    pos = np.unique(np.concatenate([_sample_positions(n, 20_000, 5), edges])).astype(np.int64)
    p = torch.from_numpy(pos).to(DEV)
    row_of = p if ids is None else ids.index_select(0, p).to(torch.int64)
    rows = table.index_select(0, row_of).cpu().numpy()
    packed = cut["packed"].reshape(-1, prb).index_select(0, p).cpu().numpy()
    got = dict(packed=packed, codes=O.unpack(packed, dim, bits),
               **{k: cut[k].index_select(0, p).cpu().numpy() for k in ("scale", "bias", "row_min", "row_max")})
    compare_quantized(rows, got, O.quantize_rows(rows, None, bits, n_threads=8), bits, what="sliced encode")

    stale_cut, stale_one = torch.full_like(table, -3.0), torch.full_like(table, -3.0)
    for st, count in ((stale_cut, None), (stale_one, n_dev)):
        P.cnr_restore_rows(ctx, st, n_rows, dim, ids, count, n, bits, cut["packed"], cut["scale"], cut["bias"], None)
    torch.cuda.synchronize()
    assert torch.equal(stale_cut, stale_one)
    back = stale_cut.index_select(0, row_of).cpu().numpy()
    assert np.array_equal(back, O.dequantize(got["codes"], got["scale"], got["bias"]))
    if ids is not None:
        written = torch.zeros(n_rows, dtype=torch.bool, device=DEV)
        written[ids.to(torch.int64)] = True
        assert torch.all(stale_cut[~written] == -3.0)
    st, bad, flags = P.cnr_poll_errors(ctx)
    assert (st, bad, flags) == (P.CNR_OK, 0, 0)
