"""GPU parity: libcnr (through its C ABI) against the CPU oracle, element by element, on the same
seeded inputs.  Sizes span several 16-row wave batches, several workgroups and ragged tails."""
import numpy as np
import pytest
import torch

import oracle as O
import paper_2010_08679_amd as P
from paper_2010_08679_amd import synth
from util_parity import (CODE_MISMATCH_FRACTION, GpuTable, assert_near_ties, compare_quantized,
                         gpu_encode_all_outputs, u32)

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
    st, bad, flags = P.cnr_poll_errors(ctx)
    assert (st, bad, flags) == (P.CNR_OK, 0, 0)


def _oracle_track(n_rows, batches):
    bm = O.new_bitmap(n_rows)
    skipped = 0
    for b in batches:
        skipped += O.mark_touched(bm, n_rows, b)
    ids, n = O.compact_dirty(bm, n_rows)
    return bm, ids, n, skipped


# ------------------------------------------------------------------ tracking + compaction

@pytest.mark.parametrize("n_rows", [1, 31, 32, 33, 63, 64, 65, 1000, 16384, 16385, 100_000, 1_000_003])
@pytest.mark.parametrize("dtype", [torch.int64, torch.int32])
def test_mark_and_compact_bit_exact(ctx, n_rows, dtype):
    print("case n_rows=%d dtype=%s" % (n_rows, dtype), flush=True)
    g = torch.Generator(device=DEV).manual_seed(n_rows)
    ck = P.TableCheckpointer(ctx, n_rows, 64, device=DEV)
    ck.clear()
    batches = []
    for it in range(3):
        n_idx = max(1, min(200_000, n_rows // 4 + 5))
        idx = torch.randint(0, n_rows, (n_idx,), generator=g, device=DEV).to(dtype)
        batches.append(idx)
        ck.mark(idx)
    ck.compact()
    torch.cuda.synchronize()
    bm, ids, n, _ = _oracle_track(n_rows, [b.cpu().numpy() for b in batches])
    assert np.array_equal(u32(ck.bitmap)[:bm.size], bm)
    assert int(ck.n_dirty.item()) == n
    assert np.array_equal(u32(ck.row_ids)[:n], ids)
    _poll_clean(ctx)


# rows per LDS bitmap slice of the bulk mark, and the table size beyond which it uses flag bytes instead
SLICE_ROWS = 32 * 40960
FLAG_ROUTE_ROWS = 16 * SLICE_ROWS + 1


@pytest.mark.parametrize("n_rows", [1, 33, 1000, 16385, 100_000, 1_000_003, SLICE_ROWS - 1, SLICE_ROWS, SLICE_ROWS + 1,
                                    2 * SLICE_ROWS + 33, 5_000_000, FLAG_ROUTE_ROWS])
@pytest.mark.parametrize("dtype", [torch.int64, torch.int32])
def test_bulk_mark_through_scratch(ctx, n_rows, dtype):
    # long streams with a scratch buffer take a bulk route (bitmap slices in LDS, or flag bytes for the
    # largest table here); the bitmap must be the same, the scratch must come back zeroed, and marks
    # must accumulate over calls and over the routes
    print("case bulk n_rows=%d dtype=%s" % (n_rows, dtype), flush=True)
    g = torch.Generator(device=DEV).manual_seed(n_rows + 1)
    scratch = P.TableCheckpointer.new_mark_scratch(n_rows, DEV)
    ck = P.TableCheckpointer(ctx, n_rows, 64, device=DEV, mark_scratch=scratch)
    ck.clear()
    batches = []
    for n_idx in (300_000 + n_rows // 256, 1000, 150_001 + n_rows // 256):   # bulk, atomic, bulk
        idx = torch.randint(-2, n_rows + 2, (n_idx,), generator=g, device=DEV).to(dtype)
        idx[-1] = n_rows - 1                                   # the last row, at the very end of a stream
        idx[0], idx[1] = -1, n_rows                            # and two that are outside for certain
        batches.append(idx)
        ck.mark(idx)
    ck.compact()
    torch.cuda.synchronize()
    bm, ids, n, skipped = _oracle_track(n_rows, [b.cpu().numpy() for b in batches])
    assert np.array_equal(u32(ck.bitmap)[:bm.size], bm)
    assert int(ck.n_dirty.item()) == n and np.array_equal(u32(ck.row_ids)[:n], ids)
    assert not scratch.any()
    st, bad, flags = P.cnr_poll_errors(ctx)
    assert st == P.CNR_E_INDEX_RANGE and bad == skipped and flags == 0
    _poll_clean(ctx)


@pytest.mark.parametrize("dtype", [torch.int64, torch.int32])
@pytest.mark.parametrize("offset,length", [(1, 200_001), (2, 200_002), (3, 199_999), (0, 200_003), (1, 70_000)])
def test_bulk_mark_any_stream_alignment_and_length(ctx, dtype, offset, length):
    # the index stream may start at any naturally aligned address and have any length: the elements
    # before the first and after the last whole 16-byte unit are marked as well
    n_rows = 3_000_017
    print("case bulk alignment dtype=%s offset=%d length=%d" % (dtype, offset, length), flush=True)
    g = torch.Generator(device=DEV).manual_seed(offset * 7 + length)
    scratch = P.TableCheckpointer.new_mark_scratch(n_rows, DEV)
    ck = P.TableCheckpointer(ctx, n_rows, 64, device=DEV, mark_scratch=scratch)
    ck.clear()
    base = torch.randint(0, n_rows, (offset + length + 5,), generator=g, device=DEV).to(dtype)
    idx = base[offset:offset + length]
    idx[0] = 0
    idx[-1] = n_rows - 1
    assert idx.data_ptr() == base.data_ptr() + offset * base.element_size()
    ck.mark(idx)
    ck.compact()
    torch.cuda.synchronize()
    bm, ids, n, skipped = _oracle_track(n_rows, [idx.cpu().numpy()])
    assert skipped == 0
    assert np.array_equal(u32(ck.bitmap)[:bm.size], bm)
    assert int(ck.n_dirty.item()) == n and np.array_equal(u32(ck.row_ids)[:n], ids)
    assert not scratch.any()
    _poll_clean(ctx)


@pytest.mark.parametrize("dtype", [torch.int64, torch.int32])
@pytest.mark.parametrize("offset,length", [(0, 400_000), (1, 400_001), (3, 399_998)])
def test_flag_route_mark_with_heavy_repeats(ctx, dtype, offset, length):
    # tables beyond the slice route: look-ups go through a table of lately flagged rows that drops
    # repeats.  A stream that is mostly repeats of a few thousand hot rows (in bursts and spread out),
    # rows whose slot content is the empty marker (they bypass the table), rows that collide in one
    # slot, indices outside the table, any alignment and length; and a second call on top of the first
    n_rows = FLAG_ROUTE_ROWS + 17
    print("case flag route repeats dtype=%s offset=%d length=%d" % (dtype, offset, length), flush=True)
    rng = np.random.default_rng(length + offset)
    hot = rng.choice(n_rows, size=3000, replace=False)
    h = (np.arange(n_rows, dtype=np.uint64) * np.uint64(0x9E3779B1)) & np.uint64(0xFFFFFFFF)
    bypass = np.flatnonzero((h & np.uint64(0xFFFF)) == np.uint64(0xFFFF))[:50]            # empty-marker rows
    same_slot = np.flatnonzero((h >> np.uint64(16)) == (h[hot[0]] >> np.uint64(16)))[:40]   # collide with a hot row
    parts = [hot[rng.integers(0, 3000, size=length // 2)], np.repeat(hot[:200], 100), np.repeat(bypass, 20),
             np.tile(same_slot, 30), rng.integers(0, n_rows, size=length // 8), np.array([-1, -5, n_rows, n_rows + 7, n_rows - 1, 0])]
    stream = np.concatenate(parts)
    rng.shuffle(stream[: length // 2])                                                     # keep the bursts that follow
    stream = np.resize(stream, offset + length + 3).astype(np.int64)
    if dtype == torch.int32:
        stream[5] = -(2 ** 31)                                                             # looks like a row when cast to unsigned
    base = torch.from_numpy(stream).to(DEV).to(dtype)
    idx = base[offset:offset + length]
    scratch = P.TableCheckpointer.new_mark_scratch(n_rows, DEV)
    ck = P.TableCheckpointer(ctx, n_rows, 64, capacity=600_000, device=DEV, mark_scratch=scratch)
    ck.clear()
    ck.mark(idx)
    second = torch.from_numpy(rng.integers(0, n_rows, size=length)).to(DEV).to(dtype)
    ck.mark(second)
    ck.compact()
    torch.cuda.synchronize()
    bm, ids, n, skipped = _oracle_track(n_rows, [idx.cpu().numpy(), second.cpu().numpy()])
    assert skipped >= 4
    assert np.array_equal(u32(ck.bitmap)[:bm.size], bm)
    assert int(ck.n_dirty.item()) == n and np.array_equal(u32(ck.row_ids)[:n], ids)
    assert not scratch.any()
    st, bad, flags = P.cnr_poll_errors(ctx)
    assert st == P.CNR_E_INDEX_RANGE and bad == skipped and flags == 0


def test_mark_skips_and_counts_out_of_range(ctx):
    n_rows = 5000
    ck = P.TableCheckpointer(ctx, n_rows, 64, device=DEV)
    ck.clear()
    g = torch.Generator(device=DEV).manual_seed(5)
    idx = torch.randint(-50, n_rows + 50, (20_000,), generator=g, device=DEV)
    ck.mark(idx)
    ck.compact()
    bm, ids, n, skipped = _oracle_track(n_rows, [idx.cpu().numpy()])
    st, bad, flags = P.cnr_poll_errors(ctx)
    assert st == P.CNR_E_INDEX_RANGE and bad == skipped and skipped > 0 and flags == 0
    assert np.array_equal(u32(ck.bitmap)[:bm.size], bm)
    assert np.array_equal(u32(ck.row_ids)[:n], ids)
    _poll_clean(ctx)                                            # counters were reset by the poll


def test_compact_empty_full_garbage_padding_and_capacity(ctx):
    n_rows = 40_001
    ck = P.TableCheckpointer(ctx, n_rows, 64, device=DEV)
    ck.clear()
    ck.compact()
    assert int(ck.n_dirty.item()) == 0
    ck.bitmap.fill_(-1)                                         # every bit, padding bits included
    ck.compact()
    torch.cuda.synchronize()
    assert int(ck.n_dirty.item()) == n_rows
    assert np.array_equal(u32(ck.row_ids)[:n_rows], np.arange(n_rows, dtype=np.uint32))
    small = P.TableCheckpointer(ctx, n_rows, 64, capacity=1000, device=DEV)
    small.bitmap.fill_(-1)
    small.row_ids.fill_(-1)
    small.compact()
    st, bad, flags = P.cnr_poll_errors(ctx)
    assert st == P.CNR_E_CAPACITY and flags & P.CNR_FLAG_CAPACITY
    assert int(small.n_dirty.item()) == n_rows                  # true count is still reported
    assert np.array_equal(u32(small.row_ids), np.arange(1000, dtype=np.uint32))
    _poll_clean(ctx)


def test_clear_bitmap_after_marking(ctx):
    n_rows = 70_000
    ck = P.TableCheckpointer(ctx, n_rows, 64, device=DEV)
    ck.mark(torch.arange(0, n_rows, 3, device=DEV))
    ck.clear()
    torch.cuda.synchronize()
    assert not ck.bitmap.any()


# ------------------------------------------------------------------ quantize + pack + restore

def _table(n_rows, dim, seed, kind="normal"):
    if kind == "normal":
        return synth.table_normal(n_rows, dim, 0.05, seed, DEV)
    return synth.table_outlier_mix(n_rows, dim, 0.02, seed, DEV)


def _dirty(gt, frac, seed):
    idx = synth.bernoulli_lookup_stream(gt.n_rows, frac, seed, DEV)
    gt.ck.clear()
    gt.ck.mark(idx)
    gt.ck.compact()
    return idx


@pytest.mark.parametrize("bits", BITS)
@pytest.mark.parametrize("dim", [64, 128, 256, 8, 40, 96])
def test_minmax_encode_and_restore(ctx, bits, dim):
    print("case bits=%d dim=%d" % (bits, dim), flush=True)
    n_rows = 3001
    gt = GpuTable(ctx, _table(n_rows, dim, 100 + dim + bits))
    idx = _dirty(gt, 0.37, bits * 7 + dim)
    got = gpu_encode_all_outputs(gt, bits)
    _, ids, n, _ = _oracle_track(n_rows, [idx.cpu().numpy()])
    assert got["n"] == n
    ora = O.quantize_rows(gt.host, ids, bits)
    compare_quantized(gt.host[ids], got, ora, bits, what="minmax b%d d%d" % (bits, dim))
    # the fused pack is the dense layout of the codes the same kernel reports
    assert np.array_equal(got["packed"], O.pack(got["codes"], bits))
    # restore into a stale copy: listed rows are scale*q+bias bit for bit, the rest untouched
    stale = torch.full_like(gt.table, 123.0)
    d = got["dev"]
    P.cnr_restore_rows(ctx, stale, n_rows, dim, d["row_ids"], d["n_dev"], d["n_max"], bits,
                       d["packed"], d["scale"], d["bias"])
    torch.cuda.synchronize()
    want = np.full_like(gt.host, 123.0)
    O.restore_rows(want, ids, bits, got["packed"], got["scale"], got["bias"])
    assert np.array_equal(stale.cpu().numpy().view(np.uint32), want.view(np.uint32))
    _poll_clean(ctx)


@pytest.mark.parametrize("bits", BITS)
@pytest.mark.parametrize("dim", [64, 128, 24])
def test_unfused_pack_equals_fused(ctx, bits, dim):
    n_rows = 1500
    gt = GpuTable(ctx, _table(n_rows, dim, 7))
    _dirty(gt, 0.5, 3)
    got = gpu_encode_all_outputs(gt, bits)
    n = got["n"]
    codes = torch.from_numpy(got["codes"].copy()).to(DEV).reshape(-1)
    out = torch.zeros(max(1, n) * P.cnr_packed_row_bytes(dim, bits), dtype=torch.uint8, device=DEV)
    n_dev = torch.tensor([n], dtype=torch.int64, device=DEV)
    P.cnr_pack(ctx, codes, n_dev, n, dim, bits, out)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy().reshape(n, -1), got["packed"])
    assert np.array_equal(got["packed"], O.pack(got["codes"], bits))


@pytest.mark.parametrize("n", [0, 1, 3, 15, 16, 17, 63, 64, 65, 1000])
def test_row_counts_without_row_ids(ctx, n):
    # row_ids == NULL quantizes rows 0..n-1; n is chosen around the 16-row batch of a wavefront
    dim, bits = 64, 4
    gt = GpuTable(ctx, _table(max(n, 1), dim, 11 + n))
    got = gpu_encode_all_outputs(gt, bits, row_ids=None, n=n)
    if n == 0:
        return
    ora = O.quantize_rows(gt.host[:n].copy(), None, bits)
    compare_quantized(gt.host[:n], got, ora, bits, what="n=%d" % n)
    assert np.array_equal(got["packed"], O.pack(got["codes"], bits))


def test_device_count_overrides_n_max(ctx):
    dim, bits, n_rows = 128, 3, 900
    gt = GpuTable(ctx, _table(n_rows, dim, 5))
    ids = torch.arange(0, n_rows, 2, dtype=torch.int32, device=DEV)
    n_dev = torch.tensor([37], dtype=torch.int64, device=DEV)
    scale = torch.full((ids.numel(),), -7.0, device=DEV)
    bias = torch.full((ids.numel(),), -7.0, device=DEV)
    packed = torch.full((ids.numel() * 48,), 0xEE, dtype=torch.uint8, device=DEV)
    P.cnr_quantize_rows(ctx, gt.table, n_rows, dim, ids, n_dev, ids.numel(), bits, P.CNR_RANGE_MINMAX,
                        None, scale, bias, packed=packed)
    torch.cuda.synchronize()
    ora = O.quantize_rows(gt.host, ids.cpu().numpy().view(np.uint32)[:37], bits)
    assert np.array_equal(scale.cpu().numpy()[:37], ora["scale"])
    assert torch.all(scale[37:] == -7.0) and torch.all(packed[37 * 48:] == 0xEE)
    assert np.array_equal(packed.cpu().numpy()[:37 * 48].reshape(37, 48), O.pack(ora["codes"], bits))


def test_special_rows(ctx):
    dim = 64
    rows = np.zeros((8, dim), dtype=np.float32)
    rows[0] = 0.375                                    # constant
    rows[1, ::2] = -0.0                                # zeros of both signs
    rows[2] = np.linspace(-1, 1, dim)                  # exact-tie prone, symmetric
    rows[3] = np.float32(1e-41) * np.arange(dim)       # denormals
    rows[4] = np.float32(1e30) * np.cos(np.arange(dim))
    rows[5, 7] = 5.0                                   # single spike
    rows[6] = -np.arange(dim, dtype=np.float32)
    rows[7] = np.arange(dim) % 4                       # exactly on a 2-bit grid
    gt = GpuTable(ctx, torch.from_numpy(rows).to(DEV))
    for bits in BITS:
        for mode in (P.CNR_RANGE_MINMAX, P.CNR_RANGE_SYMMETRIC):
            got = gpu_encode_all_outputs(gt, bits, mode=mode, row_ids=None, n=8)
            ora = O.quantize_rows(rows, None, bits, mode=mode)
            for k in ("scale", "bias", "row_min", "row_max"):
                assert np.array_equal(got[k].view(np.uint32), ora[k].view(np.uint32)), (bits, mode, k)
            # codes come from a reciprocal multiply on the GPU and a division in the oracle: they may
            # differ by one step, and only where the quotient is shown to sit at a half-integer (rows 2
            # and 7 are built to put many quotients exactly there)
            diff = np.abs(got["codes"].astype(np.int16) - ora["codes"].astype(np.int16))
            assert_near_ties(rows, ora, diff, what="special rows b%d mode %d" % (bits, mode))


@pytest.mark.parametrize("bits", (2, 3, 4))
@pytest.mark.parametrize("dim", [64, 128, 40, 16, 32, 256])
@pytest.mark.parametrize("params", [(25, 1.0), (45, 0.6), (100, 1.0)])
def test_greedy_encode(ctx, bits, dim, params):
    print("case greedy bits=%d dim=%d params=%s" % (bits, dim, params), flush=True)
    n_rows = 1237
    gt = GpuTable(ctx, _table(n_rows, dim, 31 + bits, kind="outlier"))
    idx = _dirty(gt, 0.3, dim + bits)
    got = gpu_encode_all_outputs(gt, bits, mode=P.CNR_RANGE_GREEDY, greedy=params)
    _, ids, n, _ = _oracle_track(n_rows, [idx.cpu().numpy()])
    assert got["n"] == n
    ora = O.quantize_rows(gt.host, ids, bits, mode=O.RANGE_GREEDY, num_bins=params[0], ratio=params[1],
                          n_threads=8)
    compare_quantized(gt.host[ids], got, ora, bits, greedy=True, what="greedy b%d d%d" % (bits, dim))
    assert np.array_equal(got["packed"], O.pack(got["codes"], bits))
    # the search must have moved a fair share of the outlier rows off their min/max range
    plain = O.quantize_rows(gt.host, ids, bits)
    assert np.mean(got["scale"] < plain["scale"]) > 0.2


@pytest.mark.parametrize("dim,bits,params", [(64, 4, (100, 1.0)), (64, 3, (45, 0.6)), (64, 2, (25, 1.0)), (64, 8, (20, 1.0)),
                                             (128, 4, (100, 1.0)), (128, 3, (25, 1.0)), (256, 4, (45, 0.6)), (256, 2, (100, 1.0)),
                                             (32, 4, (100, 1.0)), (32, 3, (25, 1.0)), (32, 2, (45, 0.6)), (32, 8, (20, 1.0)),
                                             (128, 2, (45, 0.6)), (128, 8, (20, 1.0)), (256, 3, (25, 1.0)), (256, 8, (20, 0.5))])
def test_greedy_on_long_lists(ctx, dim, bits, params):
    # A list of 8 M elements or more is searched with 64 elements per lane (32 at dim 32) instead of 16:
    # the same results are due.  Ordinary outlier rows with rows a few float spacings wide, constant
    # rows and rows of huge and tiny magnitude among them (waves that hold one divide as F_Q is
    # written); the oracle checks a sample that contains all of those, the pack and the row ranges are
    # checked on every row.
    print("case greedy long list bits=%d dim=%d params=%s" % (bits, dim, params), flush=True)
    n_rows = (1 << 23) // dim * 10 // 9 + 4321
    table = synth.table_outlier_mix(n_rows, dim, 0.02, 51 + dim + bits, DEV)
    rng = np.random.default_rng(dim * 8 + bits)
    special = []
    for mag in (1.0, 1000.0, -7.5):
        base = np.float32(mag)
        u = np.spacing(np.abs(base))
        for span in (1, 2, 7, 100, 40000):
            x = (base + u * rng.integers(0, span + 1, size=(6, dim)).astype(np.float32)).astype(np.float32)
            x[:, 0], x[:, 1] = base, base + u * span
            special.append(x)
    special.append(np.full((5, dim), 0.25, dtype=np.float32))
    special.append(np.float32(rng.normal(0, 1e30, size=(5, dim))))
    special.append(np.float32(rng.normal(0, 1e-36, size=(5, dim))))
    special = np.concatenate(special)
    where = np.sort(rng.choice(n_rows, size=special.shape[0], replace=False))
    table[torch.from_numpy(where).to(DEV)] = torch.from_numpy(special).to(DEV)
    gt = GpuTable(ctx, table)
    idx = torch.nonzero(torch.rand(n_rows, device=DEV, generator=torch.Generator(device=DEV).manual_seed(dim + bits)) < 0.93).reshape(-1)
    idx = torch.unique(torch.cat([idx, torch.from_numpy(where).to(DEV)]))
    gt.ck.clear(); gt.ck.mark(idx); gt.ck.compact()
    got = gpu_encode_all_outputs(gt, bits, mode=P.CNR_RANGE_GREEDY, greedy=params)
    n = got["n"]
    ids = idx.cpu().numpy()
    assert n == ids.size and n * dim >= 1 << 23
    rows = gt.host[ids]
    assert np.array_equal(got["row_min"], rows.min(axis=1)) and np.array_equal(got["row_max"], rows.max(axis=1))
    assert np.array_equal(got["packed"], O.pack(got["codes"], bits))
    pos = np.unique(np.concatenate([np.arange(200), np.arange(n - 200, n), np.searchsorted(ids, where),
                                    rng.integers(0, n, size=24_000)]))
    ora = O.quantize_rows(rows[pos], None, bits, mode=O.RANGE_GREEDY, num_bins=params[0], ratio=params[1], n_threads=8)
    sub = {k: got[k][pos] for k in ("scale", "bias", "row_min", "row_max", "codes")}
    compare_quantized(rows[pos], sub, ora, bits, greedy=True, what="greedy long list b%d d%d" % (bits, dim))
    plain = O.quantize_rows(rows[pos], None, bits)
    if bits <= 4:   # the search must have moved a fair share of the rows (at 8 bits clipping hardly ever pays)
        assert np.mean(sub["scale"] < plain["scale"]) > 0.2
    # the same buffers (their capacity allows a long list) with a short list, its length known on the
    # device alone: the kernel for short lists must be the one that runs, and nothing else may write
    few = torch.from_numpy(np.sort(rng.choice(n_rows, size=3001, replace=False))).to(DEV)
    gt.ck.clear(); gt.ck.mark(few); gt.ck.compact()
    got = gpu_encode_all_outputs(gt, bits, mode=P.CNR_RANGE_GREEDY, greedy=params)
    assert got["n"] == 3001
    rows = gt.host[few.cpu().numpy()]
    ora = O.quantize_rows(rows, None, bits, mode=O.RANGE_GREEDY, num_bins=params[0], ratio=params[1], n_threads=8)
    compare_quantized(rows, got, ora, bits, greedy=True, what="greedy short list in long buffers b%d d%d" % (bits, dim))
    assert np.array_equal(got["packed"], O.pack(got["codes"], bits))
    _poll_clean(ctx)


@pytest.mark.parametrize("dim", [64, 128, 16, 40])
def test_greedy_on_rows_spanning_a_few_float_spacings(ctx, dim):
    # rows a few representable values wide around a large magnitude: the cumulative bounds of the
    # search move by whole spacings and late candidate ranges close or turn inside out; the result
    # must still be the oracle's, bit for bit
    rng = np.random.default_rng(dim)
    blocks = []
    for mag in (1.0, 1000.0, 3e-3, -7.5):
        base = np.float32(mag)
        u = np.spacing(np.abs(base))
        for span in (1, 2, 4, 7, 20, 100, 3000, 40000):
            x = (base + u * rng.integers(0, span + 1, size=(24, dim)).astype(np.float32)).astype(np.float32)
            x[:, 0], x[:, 1] = base, base + u * span
            blocks.append(x)
    blocks.append(np.float32(rng.normal(0, 0.02, size=(40, dim))))     # ordinary rows in the same waves
    rows = np.concatenate(blocks)[rng.permutation(sum(b.shape[0] for b in blocks))]
    gt = GpuTable(ctx, torch.from_numpy(rows).to(DEV))
    n = rows.shape[0]
    for bits in (2, 3, 4):
        if (dim * bits) % 8:
            continue
        for params in ((3, 1.0), (6, 1.0), (25, 1.0), (100, 1.0), (45, 0.6)):
            got = gpu_encode_all_outputs(gt, bits, mode=P.CNR_RANGE_GREEDY, greedy=params, row_ids=None, n=n)
            ora = O.quantize_rows(rows, None, bits, mode=O.RANGE_GREEDY, num_bins=params[0], ratio=params[1])
            for k in ("scale", "bias", "row_min", "row_max"):
                assert np.array_equal(got[k].view(np.uint32), ora[k].view(np.uint32)), (bits, params, k)
            assert np.array_equal(got["codes"], ora["codes"]), (bits, params)


def test_greedy_zero_ratio_is_minmax(ctx):
    gt = GpuTable(ctx, _table(500, 64, 3, kind="outlier"))
    a = gpu_encode_all_outputs(gt, 4, row_ids=None, n=500)
    b = gpu_encode_all_outputs(gt, 4, mode=P.CNR_RANGE_GREEDY, greedy=(50, 0.0), row_ids=None, n=500)
    for k in ("scale", "bias", "codes", "packed"):
        assert np.array_equal(a[k], b[k])


def test_bad_row_ids_are_skipped_and_flagged(ctx):
    dim, bits, n_rows = 64, 4, 100
    gt = GpuTable(ctx, _table(n_rows, dim, 9))
    ids_np = np.array([5, 7, 100, 9, 4_000_000_000, 11], dtype=np.uint32)
    ids = torch.from_numpy(ids_np.view(np.int32)).to(DEV)
    scale = torch.full((6,), -7.0, device=DEV)
    bias = torch.full((6,), -7.0, device=DEV)
    packed = torch.full((6 * 32,), 0xEE, dtype=torch.uint8, device=DEV)
    P.cnr_quantize_rows(ctx, gt.table, n_rows, dim, ids, None, 6, bits, P.CNR_RANGE_MINMAX, None, scale,
                        bias, packed=packed)
    st, _, flags = P.cnr_poll_errors(ctx)
    assert st == P.CNR_E_ROW_ID and flags == P.CNR_FLAG_ROW_ID
    good = [0, 1, 3, 5]
    ora = O.quantize_rows(gt.host, ids_np[good], bits)
    assert np.array_equal(scale.cpu().numpy()[good], ora["scale"])
    assert np.array_equal(packed.cpu().numpy().reshape(6, 32)[good], O.pack(ora["codes"], bits))
    assert torch.all(scale[[2, 4]] == -7.0) and torch.all(packed.reshape(6, 32)[[2, 4]] == 0xEE)
    # restore: bad ids are skipped too, nothing outside the table is written
    stale = torch.zeros_like(gt.table)
    P.cnr_restore_rows(ctx, stale, n_rows, dim, ids, None, 6, bits, packed, scale, bias)
    st, _, flags = P.cnr_poll_errors(ctx)
    assert st == P.CNR_E_ROW_ID
    touched = torch.nonzero(stale.abs().sum(dim=1)).reshape(-1).cpu().tolist()
    assert set(touched) <= {5, 7, 9, 11}
    _poll_clean(ctx)


def test_argument_errors(ctx):
    t = torch.zeros((16, 64), device=DEV)
    s = torch.zeros(16, device=DEV)
    with pytest.raises(P.CnrError) as e:
        P.cnr_quantize_rows(ctx, t, 16, 64, None, None, 16, 5, P.CNR_RANGE_MINMAX, None, s, s)
    assert e.value.status == P.CNR_E_BITS
    t2 = torch.zeros((16, 12), device=DEV)
    with pytest.raises(P.CnrError) as e:
        P.cnr_quantize_rows(ctx, t2, 16, 12, None, None, 16, 3, P.CNR_RANGE_MINMAX, None, s, s)
    assert e.value.status == P.CNR_E_DIM                       # 36 bits per row: not whole bytes
    with pytest.raises(P.CnrError) as e:
        P.cnr_quantize_rows(ctx, t, 16, 64, None, None, 16, 4, P.CNR_RANGE_GREEDY, None, s, s)
    assert e.value.status == P.CNR_E_INVALID                   # greedy without parameters
    with pytest.raises(P.CnrError) as e:
        P.cnr_quantize_rows(ctx, t.reshape(-1)[1:], 15, 64, None, None, 15, 4, P.CNR_RANGE_MINMAX, None, s, s)
    assert e.value.status == P.CNR_E_ALIGN
    _poll_clean(ctx)


# ------------------------------------------------------------------ the small benchmark configurations

def test_cfg1_end_to_end(ctx):
    w = synth.WORKLOADS["cfg1"]
    gt = GpuTable(ctx, synth.make_table(w, 0, 1, DEV))
    batches = list(synth.lookup_batches(w, 0, 1, DEV))
    gt.ck.clear()
    for b in batches:
        gt.ck.mark(b)
    gt.ck.compact()
    got = gpu_encode_all_outputs(gt, 4)
    bm, ids, n, _ = _oracle_track(w.n_rows, [b.cpu().numpy() for b in batches])
    assert np.array_equal(u32(gt.ck.bitmap)[:bm.size], bm)
    assert got["n"] == n and np.array_equal(u32(gt.ck.row_ids)[:n], ids) and 0 < n <= 4096
    ora = O.quantize_rows(gt.host, ids, 4)
    compare_quantized(gt.host[ids], got, ora, 4, what="cfg1")
    assert np.array_equal(got["packed"], O.pack(ora["codes"], 4))
    stale = torch.zeros_like(gt.table)
    d = got["dev"]
    P.cnr_restore_rows(ctx, stale, w.n_rows, w.dim, d["row_ids"], d["n_dev"], d["n_max"], 4, d["packed"],
                       d["scale"], d["bias"])
    want = np.zeros_like(gt.host)
    O.restore_rows(want, ids, 4, O.pack(ora["codes"], 4), ora["scale"], ora["bias"])
    assert np.array_equal(stale.cpu().numpy().view(np.uint32), want.view(np.uint32))
    _poll_clean(ctx)


def test_cfg2_two_tables_accumulated_tracking(ctx):
    # configuration 2 at reduced length: 2 of the 8 tables, 12 of the 200 iterations, full shapes
    w = synth.WORKLOADS["cfg2"]
    for ti in range(2):
        gt = GpuTable(ctx, synth.make_table(w, ti, 2, DEV))
        batches = list(synth.lookup_batches(w, ti, 2, DEV, iterations=12))
        gt.ck.clear()
        for b in batches:
            gt.ck.mark(b)
        gt.ck.compact()
        got = gpu_encode_all_outputs(gt, 4)
        bm, ids, n, _ = _oracle_track(w.n_rows, [b.cpu().numpy() for b in batches])
        assert np.array_equal(u32(gt.ck.bitmap)[:bm.size], bm)
        assert got["n"] == n and np.array_equal(u32(gt.ck.row_ids)[:n], ids)
        ora = O.quantize_rows(gt.host, ids, 4, n_threads=8)
        compare_quantized(gt.host[ids], got, ora, 4, what="cfg2 table %d" % ti)
        assert np.array_equal(got["packed"], O.pack(got["codes"], 4))
    _poll_clean(ctx)


# ------------------------------------------------------------------ error metric and parameter selection

@pytest.mark.parametrize("bits", BITS)
@pytest.mark.parametrize("dim", [64, 128, 40])
def test_quant_error_matches_oracle_l2(ctx, bits, dim):
    n_rows = 2000
    gt = GpuTable(ctx, _table(n_rows, dim, 50 + bits, kind="outlier"))
    idx = _dirty(gt, 0.4, 9)
    got = gpu_encode_all_outputs(gt, bits)
    n, d = got["n"], got["dev"]
    err = torch.full((max(1, d["n_max"]),), -1.0, dtype=torch.float64, device=DEV)
    mean = torch.full((1,), -1.0, dtype=torch.float64, device=DEV)
    P.cnr_quant_error(ctx, gt.table, n_rows, dim, d["row_ids"], d["n_dev"], d["n_max"], bits, d["packed"],
                      d["scale"], d["bias"], err, mean)
    torch.cuda.synchronize()
    ids = u32(d["row_ids"])[:n]
    want, want_mean = O.row_l2(gt.host[ids], O.dequantize(got["codes"], got["scale"], got["bias"]))
    e = err.cpu().numpy()
    assert np.allclose(e[:n], want, rtol=1e-12, atol=0) and np.all(e[n:] == -1.0)
    assert float(mean.item()) == pytest.approx(want_mean, rel=1e-12)
    _poll_clean(ctx)


def test_greedy_parameter_selection_matches_oracle(ctx):
    # Section 5.2 "Parameter selection": profile a uniform sample of the dirty rows over a grid of
    # num_bins and ratio values; both sides must see the same error curves and make the same choice
    n_rows, dim, bits = 200_000, 64, 3
    gt = GpuTable(ctx, _table(n_rows, dim, 21, kind="outlier"))
    _dirty(gt, 0.3, 2)
    n = int(gt.ck.n_dirty.item())
    pos = synth.sample_positions(n, 0.005, 7, DEV, min_rows=256)
    sample_ids = gt.ck.row_ids[pos].contiguous()
    bins, ratios = (5, 10, 20, 30, 40, 50), (0.25, 0.5, 0.75, 1.0)
    choice, report = P.select_greedy_params(ctx, gt.table, n_rows, dim, sample_ids, bits, bins, ratios)
    rows = gt.host[u32(sample_ids)]
    want_choice, want_report = O.select_greedy_params(rows, bits, bins, ratios, n_threads=8)
    assert set(report) == set(want_report)
    for key in want_report:
        assert report[key] == pytest.approx(want_report[key], rel=1e-9), key
    assert choice == want_choice
    assert report[("bins", choice[0])] < report["naive"]
    _poll_clean(ctx)


# ------------------------------------------------------------------ chunked encode with overlapped copies

@pytest.mark.parametrize("overlap", [P.CNR_HOST_OVERLAP, P.CNR_HOST_SERIAL, P.CNR_HOST_DIRECT])
def test_chunked_encode_to_host_equals_one_shot_encode(ctx, overlap):
    # Sections 4.4 / 5.2: the checkpoint is built chunk by chunk, each chunk handed on while the next
    # is quantized.  The chunks must add up to exactly the unchunked result.
    n_rows, dim, bits = 300_000, 64, 4
    gt = GpuTable(ctx, _table(n_rows, dim, 8))
    _dirty(gt, 0.3, 4)
    enc = gt.ck.alloc_output(bits)
    gt.ck.encode(gt.table, enc)
    n = enc.count()
    writer = P.HostCheckpointWriter(ctx, dim, bits, capacity=n_rows, chunk_rows=16 * 1000, device=DEV)
    for _ in range(2):                                          # staging buffers are reused across calls
        got_n = writer.encode_to_host(gt.ck, gt.table, overlap=overlap)
        assert got_n == n and n > 5 * writer.chunk and n % writer.chunk != 0
        prb = P.cnr_packed_row_bytes(dim, bits)
        assert torch.equal(writer.host["row_ids"][:n], enc.row_ids[:n].cpu())
        assert torch.equal(writer.host["scale"][:n], enc.scale[:n].cpu())
        assert torch.equal(writer.host["bias"][:n], enc.bias[:n].cpu())
        assert torch.equal(writer.host["packed"][:n * prb], enc.packed[:n * prb].cpu())
    ora = O.quantize_rows(gt.host, u32(enc.row_ids)[:n], bits, n_threads=8)
    assert np.array_equal(writer.host["scale"][:n].numpy(), ora["scale"])
    assert np.mean(O.unpack(writer.host["packed"][:n * prb].numpy(), dim, bits) != ora["codes"]) <= 1e-4
    _poll_clean(ctx)


@pytest.mark.parametrize("overlap", [True, False, "direct"])
@pytest.mark.parametrize("with_ids", [True, False])
def test_round_trip_through_host_memory(ctx, overlap, with_ids):
    # checkpoint to host memory in chunks, then the way back: the table restored from the host buffers
    # (chunk by chunk through the staging sets, or by a kernel that reads the pinned buffers itself)
    # equals the one restored by a single call from the device-side encode, and the oracle's
    n_rows, dim, bits = 60_017, 64, 4
    print("case host round trip overlap=%s with_ids=%s" % (overlap, with_ids), flush=True)
    back_path = overlap = P.CNR_HOST_DIRECT if overlap == "direct" else int(overlap)
    table = synth.table_outlier_mix(n_rows, dim, 0.02, 41, DEV)
    ck = P.TableCheckpointer(ctx, n_rows, dim, device=DEV)
    ck.clear()
    if with_ids:
        ck.mark(synth.bernoulli_lookup_stream(n_rows, 0.4, 7, DEV))
    else:
        ck.bitmap.fill_(-1)                                     # every row: a full checkpoint
    ck.compact()
    writer = P.HostCheckpointWriter(ctx, dim, bits, capacity=n_rows, chunk_rows=4096, device=DEV)   # 6 to 15 chunks
    n = writer.encode_to_host(ck, table, overlap=overlap)
    assert n == int(ck.n_dirty.item()) and (with_ids or n == n_rows)
    ids = writer.host["row_ids"][:n].numpy().view(np.uint32).copy()
    if not with_ids:                                            # the same checkpoint without any list
        listed = {k: v[:n * (writer.prb if k == "packed" else 1)].clone() for k, v in writer.host.items()}
        assert writer.encode_table_to_host(table, n_rows, overlap=overlap) == n_rows
        for k in ("scale", "bias", "packed"):
            assert torch.equal(writer.host[k][:listed[k].numel()], listed[k]), k

    direct = torch.full_like(table, -3.0)
    enc = ck.alloc_output(bits)
    ck.encode(table, enc)
    ck.restore(direct, enc)
    for rep in range(2):                                        # twice: the staging sets are reused
        back = torch.full_like(table, -3.0)
        writer.restore_from_host(back, n_rows, n, overlap=back_path, with_ids=with_ids)
        assert torch.equal(back, direct)
    want = np.full((n_rows, dim), -3.0, dtype=np.float32)
    O.restore_rows(want, ids, bits, writer.host["packed"][:n * writer.prb].numpy().reshape(n, -1),
                   writer.host["scale"][:n].numpy(), writer.host["bias"][:n].numpy())
    assert np.array_equal(back.cpu().numpy(), want)
    # a write right after a read, then a read, with no wait between the first two
    main = torch.cuda.current_stream()
    back.fill_(-3.0)
    P.cnr_restore_from_host(writer.writer, back, n_rows, dim, bits, writer.host["row_ids"] if with_ids else None,
                            writer.host["scale"], writer.host["bias"], writer.host["packed"], n, back_path, main)
    assert writer.encode_to_host(ck, back, overlap=overlap) == n   # encodes the table just restored
    again = torch.full_like(table, -3.0)
    writer.restore_from_host(again, n_rows, n, overlap=back_path, with_ids=with_ids)
    torch.cuda.synchronize()
    q = O.quantize_rows(want, ids, bits, n_threads=4)           # the oracle's encode of its own restored table
    want2 = np.full((n_rows, dim), -3.0, dtype=np.float32)
    O.restore_rows(want2, ids, bits, O.pack(q["codes"], bits), q["scale"], q["bias"])
    got2 = again.cpu().numpy()
    assert np.mean(got2 != want2) <= 1e-4 and np.array_equal(got2[want2 == -3.0], want2[want2 == -3.0])
    writer.close()
    _poll_clean(ctx)


@pytest.mark.parametrize("dim,bits", [(64, 2), (64, 3), (64, 8), (128, 4), (128, 8), (256, 3), (32, 4), (8, 8)])
def test_restore_reading_pinned_host_memory_itself(ctx, dim, bits):
    # every restore kernel shape with its inputs in pinned host memory: the same table as from the
    # device-side copies of those inputs, and as the oracle's restore; a ragged row count, twice
    n_rows = 20_011
    print("case restore straight from host dim=%d bits=%d" % (dim, bits), flush=True)
    table = synth.table_outlier_mix(n_rows, dim, 0.02, 43, DEV)
    ck = P.TableCheckpointer(ctx, n_rows, dim, device=DEV)
    ck.clear()
    ck.mark(synth.bernoulli_lookup_stream(n_rows, 0.35, 9, DEV))
    ck.compact()
    writer = P.HostCheckpointWriter(ctx, dim, bits, capacity=n_rows, chunk_rows=4096, device=DEV)
    n = writer.encode_to_host(ck, table)
    enc = ck.alloc_output(bits)
    ck.encode(table, enc)
    from_device = torch.full_like(table, 7.0)
    ck.restore(from_device, enc)
    for rep in range(2):
        back = torch.full_like(table, 7.0)
        writer.restore_from_host(back, n_rows, n, overlap=P.CNR_HOST_DIRECT)
        assert torch.equal(back, from_device)
    ids = writer.host["row_ids"][:n].numpy().view(np.uint32)
    want = np.full((n_rows, dim), 7.0, dtype=np.float32)
    O.restore_rows(want, ids, bits, writer.host["packed"][:n * writer.prb].numpy().reshape(n, -1),
                   writer.host["scale"][:n].numpy(), writer.host["bias"][:n].numpy())
    assert np.array_equal(back.cpu().numpy(), want)
    writer.close()
    _poll_clean(ctx)


@pytest.mark.parametrize("dim,bits,mode", [(64, 2, "minmax"), (64, 3, "minmax"), (64, 8, "minmax"), (128, 4, "minmax"),
                                           (128, 8, "symmetric"), (256, 3, "minmax"), (32, 4, "minmax"), (8, 8, "minmax"),
                                           (64, 4, "greedy"), (48, 4, "minmax")])
def test_encode_writing_pinned_host_memory_itself(ctx, dim, bits, mode):
    # every encode kernel shape with its outputs in pinned host memory: byte for byte what the same
    # call leaves in device buffers, nothing written past the last row, with and without an id list
    n_rows = 20_011
    print("case encode straight to host dim=%d bits=%d %s" % (dim, bits, mode), flush=True)
    table = synth.table_outlier_mix(n_rows, dim, 0.02, 47, DEV)
    ck = P.TableCheckpointer(ctx, n_rows, dim, device=DEV)
    ck.clear()
    ck.mark(synth.bernoulli_lookup_stream(n_rows, 0.35, 13, DEV))
    ck.compact()
    m = {"minmax": P.CNR_RANGE_MINMAX, "symmetric": P.CNR_RANGE_SYMMETRIC, "greedy": P.CNR_RANGE_GREEDY}[mode]
    greedy = (20, 0.5) if mode == "greedy" else None
    enc = ck.alloc_output(bits)
    ck.encode(table, enc, mode=m, greedy=greedy)
    n = enc.count()
    writer = P.HostCheckpointWriter(ctx, dim, bits, capacity=n_rows, chunk_rows=4096, device=DEV)
    prb = writer.prb
    for rep in range(2):
        for v in writer.host.values():
            v.fill_(0x55 if v.dtype == torch.uint8 else 12345)
        assert writer.encode_to_host(ck, table, mode=m, greedy=greedy, overlap=P.CNR_HOST_DIRECT) == n
        assert torch.equal(writer.host["row_ids"][:n], enc.row_ids[:n].cpu())
        assert torch.equal(writer.host["scale"][:n].view(torch.int32), enc.scale[:n].cpu().view(torch.int32))
        assert torch.equal(writer.host["bias"][:n].view(torch.int32), enc.bias[:n].cpu().view(torch.int32))
        assert torch.equal(writer.host["packed"][:n * prb], enc.packed[:n * prb].cpu())
        assert bool((writer.host["row_ids"][n:] == 12345).all()) and bool((writer.host["scale"][n:] == 12345).all())
        assert bool((writer.host["bias"][n:] == 12345).all()) and bool((writer.host["packed"][n * prb:] == 0x55).all())
    assert writer.encode_table_to_host(table, n_rows, mode=m, greedy=greedy, overlap=P.CNR_HOST_DIRECT) == n_rows
    staged = {k: v.clone() for k, v in writer.host.items()}
    assert writer.encode_table_to_host(table, n_rows, mode=m, greedy=greedy, overlap=P.CNR_HOST_OVERLAP) == n_rows
    for k in ("scale", "bias", "packed"):
        assert torch.equal(writer.host[k].view(torch.uint8), staged[k].view(torch.uint8)), k
    writer.close()
    _poll_clean(ctx)


def test_restore_straight_from_host_refuses_pageable_memory(ctx):
    # a buffer the GPU cannot reach is refused on the host, nothing is launched, the table stays as it
    # was, and the runtime is left without a pending error: the same call with copies then works
    n_rows, dim, bits = 5_003, 64, 4
    print("case restore straight from host, pageable buffers", flush=True)
    table = synth.table_normal(n_rows, dim, 0.02, 45, DEV)
    ck = P.TableCheckpointer(ctx, n_rows, dim, device=DEV)
    ck.clear()
    ck.mark(synth.bernoulli_lookup_stream(n_rows, 0.5, 11, DEV))
    ck.compact()
    writer = P.HostCheckpointWriter(ctx, dim, bits, capacity=n_rows, chunk_rows=1024, device=DEV)
    n = writer.encode_to_host(ck, table)
    pinned = writer.host
    pageable = {k: v.clone() for k, v in pinned.items()}          # plain host memory
    assert not any(v.is_pinned() for v in pageable.values())
    main = torch.cuda.current_stream()
    for bad in ("row_ids", "scale", "bias", "packed"):
        bufs = dict(pinned)
        bufs[bad] = pageable[bad]
        back = torch.full_like(table, 7.0)
        with pytest.raises(P.CnrError) as e:
            P.cnr_restore_from_host(writer.writer, back, n_rows, dim, bits, bufs["row_ids"], bufs["scale"], bufs["bias"],
                                    bufs["packed"], n, P.CNR_HOST_DIRECT, main)
        assert e.value.status == P.CNR_E_HOST_MEMORY, bad
        torch.cuda.synchronize()
        assert bool((back == 7.0).all())
    want = torch.full_like(table, 7.0)
    writer.restore_from_host(want, n_rows, n, overlap=P.CNR_HOST_DIRECT)
    back = torch.full_like(table, 7.0)
    P.cnr_restore_from_host(writer.writer, back, n_rows, dim, bits, pageable["row_ids"], pageable["scale"],
                            pageable["bias"], pageable["packed"], n, P.CNR_HOST_SERIAL, main)
    P.cnr_host_writer_wait(writer.writer, main)
    assert torch.equal(back, want)
    for bad in ("row_ids", "scale", "bias", "packed"):            # the encode's direct way likewise
        bufs = dict(pinned)
        bufs[bad] = pageable[bad].clone()
        kept = bufs[bad].clone()
        with pytest.raises(P.CnrError) as e:
            P.cnr_encode_to_host(writer.writer, table, n_rows, dim, bits, ck.row_ids, n, P.CNR_RANGE_MINMAX, None,
                                 bufs["row_ids"], bufs["scale"], bufs["bias"], bufs["packed"], P.CNR_HOST_DIRECT, main)
        assert e.value.status == P.CNR_E_HOST_MEMORY, bad
        P.cnr_host_writer_wait(writer.writer, main)
        assert torch.equal(bufs[bad], kept)
    with pytest.raises(P.CnrError) as e:
        P.cnr_encode_to_host(writer.writer, table, n_rows, dim, bits, ck.row_ids, n, P.CNR_RANGE_MINMAX, None,
                             pinned["row_ids"], pinned["scale"], pinned["bias"], pinned["packed"], 3, main)
    assert e.value.status == P.CNR_E_INVALID
    writer.close()
    _poll_clean(ctx)


def test_misaligned_row_id_slice_is_refused(ctx):
    t = torch.zeros((64, 64), device=DEV)
    ids = torch.arange(64, dtype=torch.int32, device=DEV)
    s = torch.zeros(64, device=DEV)
    with pytest.raises(P.CnrError) as e:
        P.cnr_quantize_rows(ctx, t, 64, 64, ids[1:], None, 32, 4, P.CNR_RANGE_MINMAX, None, s, s)
    assert e.value.status == P.CNR_E_ALIGN


# ------------------------------------------------------------------ graph capture

def test_checkpoint_step_replays_from_a_hip_graph(ctx):
    # the whole step (clear, mark, compact, encode, restore) only enqueues kernels on the caller's
    # stream, allocates nothing and never synchronises, so it can be captured once and replayed; the
    # inputs are refreshed in place between replays and every replay is checked against the oracle
    n_rows, dim, bits = 120_000, 64, 4
    gt = GpuTable(ctx, _table(n_rows, dim, 40))
    scratch = P.TableCheckpointer.new_mark_scratch(n_rows, DEV)
    ck = P.TableCheckpointer(ctx, n_rows, dim, device=DEV, mark_scratch=scratch)
    enc = ck.alloc_output(bits)
    idx = synth.bernoulli_lookup_stream(n_rows, 0.25, 1, DEV)
    n_idx = idx.numel()
    stale = torch.zeros_like(gt.table)

    def step():
        ck.clear()
        ck.mark(idx)
        ck.compact()
        ck.encode(gt.table, enc)
        ck.restore(stale, enc)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                                  # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(3):
        # eager work between replays: new look-ups (same length), new table values, a dirtied target
        fresh = synth.bernoulli_lookup_stream(n_rows, 0.25, 10 + rep, DEV)
        m = min(n_idx, fresh.numel())
        idx[:m].copy_(fresh[:m])
        idx[m:] = fresh[0]
        gt.table.mul_(1.0 + 0.1 * (rep + 1))
        stale.fill_(float(rep))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        host = gt.table.cpu().numpy()
        bm, ids, n, _ = _oracle_track(n_rows, [idx.cpu().numpy()])
        assert int(ck.n_dirty.item()) == n and np.array_equal(u32(ck.row_ids)[:n], ids)
        ora = O.quantize_rows(host, ids, bits, n_threads=8)
        assert np.array_equal(enc.scale.cpu().numpy()[:n], ora["scale"])
        packed = enc.packed.cpu().numpy()[:n * 32].reshape(n, 32)
        assert np.mean(O.unpack(packed, dim, bits) != ora["codes"]) <= 1e-4
        want = np.full_like(host, float(rep))
        O.restore_rows(want, ids, bits, packed, ora["scale"], ora["bias"])
        assert np.array_equal(stale.cpu().numpy(), want)
        assert not scratch.any()
    _poll_clean(ctx)


# ------------------------------------------------------------------ further edges

@pytest.mark.parametrize("bits", BITS)
def test_largest_supported_row_dimension(ctx, bits):
    dim, n_rows = P.CNR_MAX_DIM, 300
    gt = GpuTable(ctx, _table(n_rows, dim, 60 + bits))
    got = gpu_encode_all_outputs(gt, bits, row_ids=None, n=n_rows)
    ora = O.quantize_rows(gt.host, None, bits, n_threads=8)
    for k in ("scale", "bias", "row_min", "row_max"):
        assert np.array_equal(got[k], ora[k])
    compare_quantized(gt.host, got, ora, bits, what="dim %d b%d" % (dim, bits))
    assert np.array_equal(got["packed"], O.pack(got["codes"], bits))
    d = got["dev"]
    stale = torch.zeros_like(gt.table)
    P.cnr_restore_rows(ctx, stale, n_rows, dim, None, None, n_rows, bits, d["packed"], d["scale"], d["bias"])
    assert np.array_equal(stale.cpu().numpy(), O.dequantize(got["codes"], got["scale"], got["bias"]))
    t = torch.zeros((4, dim + 4), device=DEV)
    s = torch.zeros(4, device=DEV)
    with pytest.raises(P.CnrError) as e:
        P.cnr_quantize_rows(ctx, t, 4, dim + 4, None, None, 4, bits, P.CNR_RANGE_MINMAX, None, s, s)
    assert e.value.status == P.CNR_E_DIM
    _poll_clean(ctx)


@pytest.mark.parametrize("bits", BITS)
@pytest.mark.parametrize("dim", [64, 128, 256, 24])
def test_symmetric_range(ctx, bits, dim):
    n_rows = 2500
    t = _table(n_rows, dim, 70 + bits) + 0.02                  # shifted: the symmetric range wastes codes
    gt = GpuTable(ctx, t)
    got = gpu_encode_all_outputs(gt, bits, mode=P.CNR_RANGE_SYMMETRIC, row_ids=None, n=n_rows)
    ora = O.quantize_rows(gt.host, None, bits, mode=O.RANGE_SYMMETRIC, n_threads=8)
    compare_quantized(gt.host, got, ora, bits, what="symmetric b%d d%d" % (bits, dim))
    assert np.array_equal(got["bias"], -np.abs(gt.host).max(axis=1))
    assert np.array_equal(got["packed"], O.pack(got["codes"], bits))


def test_row_count_limit_is_checked_on_the_host(ctx):
    bm = torch.zeros(4, dtype=torch.int32, device=DEV)
    idx = torch.zeros(4, dtype=torch.int64, device=DEV)
    with pytest.raises(P.CnrError) as e:
        P.cnr_mark_touched(ctx, bm, 1 << 32, idx)
    assert e.value.status == P.CNR_E_INVALID
    t = torch.zeros((4, 64), device=DEV)
    s = torch.zeros(4, device=DEV)
    with pytest.raises(ValueError):                            # the binding's own size check comes first
        P.cnr_quantize_rows(ctx, t, 1 << 32, 64, None, None, 4, 4, P.CNR_RANGE_MINMAX, None, s, s)
    _poll_clean(ctx)


@pytest.mark.parametrize("bits", BITS)
@pytest.mark.parametrize("dim", [64, 128, 256])
@pytest.mark.parametrize("n", [1, 5, 16, 19, 33])
def test_ragged_passes_with_ids_at_every_width(ctx, bits, dim, n):
    # a 16-row pass that is partly empty, with row ids given, one of them outside the table, and
    # output buffers exactly n rows long (nothing may be written past them: the next tensors would
    # catch it in their own checks, and the sentinel rows below do so here)
    n_rows = 300
    gt = GpuTable(ctx, _table(n_rows, dim, 90 + bits + dim + n))
    rng = np.random.default_rng(n * 1000 + dim + bits)
    ids_np = np.sort(rng.choice(n_rows, size=n, replace=False)).astype(np.uint32)
    bad_at = n // 2
    ids_bad = ids_np.copy()
    ids_bad[bad_at] = n_rows + 5
    prb = P.cnr_packed_row_bytes(dim, bits)
    pad = 2                                                     # sentinel rows behind the n real ones
    ids = torch.zeros(max(16, n), dtype=torch.int32, device=DEV)     # 16-byte aligned, >= n entries
    ids[:n] = torch.from_numpy(ids_bad.view(np.int32)).to(DEV)
    scale = torch.full((n + pad,), -7.0, device=DEV)
    bias = torch.full((n + pad,), -7.0, device=DEV)
    rmin = torch.full((n + pad,), -7.0, device=DEV)
    rmax = torch.full((n + pad,), -7.0, device=DEV)
    packed = torch.full(((n + pad) * prb,), 0xEE, dtype=torch.uint8, device=DEV)
    codes = torch.full(((n + pad) * dim,), 0xEE, dtype=torch.uint8, device=DEV)
    P.cnr_quantize_rows(ctx, gt.table, n_rows, dim, ids, None, n, bits, P.CNR_RANGE_MINMAX, None, scale, bias,
                        rmin, rmax, codes, packed)
    st, _, flags = P.cnr_poll_errors(ctx)
    assert st == P.CNR_E_ROW_ID and flags == P.CNR_FLAG_ROW_ID
    good = [k for k in range(n) if k != bad_at]
    for t in (scale, bias, rmin, rmax):
        assert torch.all(t[n:] == -7.0) and t[bad_at] == -7.0
    assert torch.all(packed.reshape(n + pad, prb)[[bad_at, n, n + 1]] == 0xEE)
    assert torch.all(codes.reshape(n + pad, dim)[[bad_at, n, n + 1]] == 0xEE)
    if good:
        ora = O.quantize_rows(gt.host, ids_np[good], bits)
        got = dict(scale=scale.cpu().numpy()[good], bias=bias.cpu().numpy()[good],
                   row_min=rmin.cpu().numpy()[good], row_max=rmax.cpu().numpy()[good],
                   codes=codes.cpu().numpy().reshape(n + pad, dim)[good])
        compare_quantized(gt.host[ids_np[good]], got, ora, bits, what="ragged n=%d d%d b%d" % (n, dim, bits))
        assert np.array_equal(packed.cpu().numpy().reshape(n + pad, prb)[good], O.pack(got["codes"], bits))
    _poll_clean(ctx)


@pytest.mark.parametrize("bits", BITS)
@pytest.mark.parametrize("dim", [4, 16, 32, 48, 72, 192, 320, 512, 1000, 2048])
def test_other_row_lengths(ctx, bits, dim):
    # row lengths beside 64 / 128 / 256: every lanes-per-row variant, full and partly used, rows past the end
    if (dim * bits) % 8:
        pytest.skip("dim * bits is not a whole number of bytes")
    n_rows, n = 700, 333
    gt = GpuTable(ctx, _table(n_rows, dim, 200 + dim + bits))
    rng = np.random.default_rng(dim * 10 + bits)
    ids_np = np.sort(rng.choice(n_rows, size=n, replace=False)).astype(np.uint32)
    ids = torch.from_numpy(ids_np.view(np.int32)).to(DEV)
    for mode, omode in ((P.CNR_RANGE_MINMAX, O.RANGE_MINMAX), (P.CNR_RANGE_SYMMETRIC, O.RANGE_SYMMETRIC)):
        got = gpu_encode_all_outputs(gt, bits, mode=mode, row_ids=ids, n=n)
        ora = O.quantize_rows(gt.host, ids_np, bits, mode=omode, n_threads=8)
        compare_quantized(gt.host[ids_np], got, ora, bits, what="dim %d b%d mode %d" % (dim, bits, mode))
        assert np.array_equal(got["packed"], O.pack(got["codes"], bits))
    d = got["dev"]
    stale = torch.zeros_like(gt.table)
    P.cnr_restore_rows(ctx, stale, n_rows, dim, ids, None, n, bits, d["packed"], d["scale"], d["bias"])
    want = np.zeros_like(gt.host)
    O.restore_rows(want, ids_np, bits, got["packed"], got["scale"], got["bias"])
    assert np.array_equal(stale.cpu().numpy(), want)
    _poll_clean(ctx)


def test_host_writer_back_to_back_tables_and_argument_errors(ctx):
    # two tables through one writer without waiting in between: the second call's first chunks go into
    # staging sets the first call's copies may still be reading, which the writer's events must order
    dim, bits, chunk = 64, 4, 16 * 500
    prb = P.cnr_packed_row_bytes(dim, bits)
    writer = P.cnr_host_writer_create(ctx, dim, bits, chunk)
    assert P.cnr_host_writer_device_bytes(dim, bits, chunk) == 2 * chunk * (prb + 12)
    jobs = []
    for seed, n_rows in ((1, 50_000), (2, 33_000)):
        gt = GpuTable(ctx, _table(n_rows, dim, 300 + seed))
        _dirty(gt, 0.5, seed)
        n = int(gt.ck.n_dirty.item())
        host = dict(ids=torch.empty(n, dtype=torch.int32, pin_memory=(seed == 1)),      # pinned and pageable
                    scale=torch.empty(n, dtype=torch.float32, pin_memory=(seed == 1)),
                    bias=torch.empty(n, dtype=torch.float32, pin_memory=(seed == 1)),
                    packed=torch.empty(n * prb, dtype=torch.uint8, pin_memory=(seed == 1)))
        jobs.append((gt, n, host))
    for gt, n, host in jobs:
        assert n > 2 * chunk
        P.cnr_encode_to_host(writer, gt.table, gt.n_rows, dim, bits, gt.ck.row_ids, n, P.CNR_RANGE_MINMAX, None,
                             host["ids"], host["scale"], host["bias"], host["packed"], overlap=True)
    P.cnr_host_writer_wait(writer)
    for gt, n, host in jobs:
        ids = u32(gt.ck.row_ids)[:n]
        ora = O.quantize_rows(gt.host, ids, bits, n_threads=8)
        assert np.array_equal(host["ids"].numpy().view(np.uint32), ids)
        got = dict(scale=host["scale"].numpy(), bias=host["bias"].numpy(),
                   codes=O.unpack(host["packed"].numpy().reshape(n, prb), dim, bits))
        compare_quantized(gt.host[ids], got, ora, bits, what="host writer, %d rows" % n)
    # rows 0 .. n-1 without a list (a full checkpoint): several chunks, the last one ragged; more rows than
    # the table has is an error
    gt = jobs[0][0]
    n_full = 2 * chunk + 336
    assert n_full <= gt.n_rows
    hs, hb = torch.empty(n_full), torch.empty(n_full)
    hp = torch.empty(n_full * prb, dtype=torch.uint8)
    P.cnr_encode_to_host(writer, gt.table, gt.n_rows, dim, bits, None, n_full, P.CNR_RANGE_MINMAX, None, None, hs, hb, hp)
    P.cnr_host_writer_wait(writer)
    ora = O.quantize_rows(gt.host[:n_full].copy(), None, bits, n_threads=8)
    got = dict(scale=hs.numpy(), bias=hb.numpy(), codes=O.unpack(hp.numpy().reshape(n_full, prb), dim, bits))
    compare_quantized(gt.host[:n_full], got, ora, bits, what="host writer, no list")
    with pytest.raises(P.CnrError) as e:
        m = gt.n_rows + 16
        P.cnr_encode_to_host(writer, gt.table, gt.n_rows, dim, bits, None, m, P.CNR_RANGE_MINMAX, None, None,
                             torch.empty(m), torch.empty(m), torch.empty(m * prb, dtype=torch.uint8))
    assert e.value.status == P.CNR_E_INVALID
    P.cnr_host_writer_destroy(writer)
    for bad_chunk, status in ((100, P.CNR_E_INVALID), (0, P.CNR_E_INVALID)):
        with pytest.raises(P.CnrError) as e:
            P.cnr_host_writer_create(ctx, dim, bits, bad_chunk)
        assert e.value.status == status
    with pytest.raises(P.CnrError) as e:
        P.cnr_host_writer_create(ctx, 12, 3, 1024)
    assert e.value.status == P.CNR_E_DIM
    _poll_clean(ctx)


def test_seeded_random_cases_against_the_oracle(ctx):
    # a sweep of seeded random shapes through every encode / restore kernel family: row length, bit
    # width, range mode, list length, with or without a row list, device-side count below n_max
    rng = np.random.default_rng(20240607)
    dims = [4, 8, 16, 24, 32, 40, 64, 72, 96, 128, 160, 256, 264, 512, 1024]
    n_cases = n_diff = n_elements = 0
    for case in range(160):
        dim = int(rng.choice(dims))
        bits = int(rng.choice(BITS))
        if (dim * bits) % 8:
            continue
        n_rows = int(rng.integers(1, 900))
        n = int(rng.integers(1, n_rows + 1))
        mode, omode = [(P.CNR_RANGE_MINMAX, O.RANGE_MINMAX), (P.CNR_RANGE_SYMMETRIC, O.RANGE_SYMMETRIC)][int(rng.integers(2))]
        with_ids = bool(rng.integers(2))
        n_live = int(rng.integers(1, n + 1))                   # what the device-side count says
        table = torch.from_numpy((rng.standard_normal((n_rows, dim)) * 10.0 ** rng.uniform(-3, 2)).astype(np.float32)).to(DEV)
        host = table.cpu().numpy()
        ids_np = np.sort(rng.choice(n_rows, size=n, replace=False)).astype(np.uint32) if with_ids else np.arange(n, dtype=np.uint32)
        ids = torch.zeros(max(16, n), dtype=torch.int32, device=DEV)
        ids[:n] = torch.from_numpy(ids_np.view(np.int32)).to(DEV)
        n_dev = torch.tensor([n_live], dtype=torch.int64, device=DEV)
        prb = P.cnr_packed_row_bytes(dim, bits)
        scale = torch.full((n,), -7.0, device=DEV)
        bias = torch.full((n,), -7.0, device=DEV)
        packed = torch.full((n * prb,), 0xEE, dtype=torch.uint8, device=DEV)
        P.cnr_quantize_rows(ctx, table, n_rows, dim, ids if with_ids else None, n_dev, n, bits, mode, None, scale, bias,
                            packed=packed)
        stale = torch.full_like(table, -3.0)
        P.cnr_restore_rows(ctx, stale, n_rows, dim, ids if with_ids else None, n_dev, n, bits, packed, scale, bias)
        torch.cuda.synchronize()
        what = "case %d: dim %d b%d n_rows %d n %d live %d ids %d mode %d" % (case, dim, bits, n_rows, n, n_live, with_ids, mode)
        assert torch.all(scale[n_live:] == -7.0) and torch.all(packed[n_live * prb:] == 0xEE), what
        ora = O.quantize_rows(host, ids_np[:n_live], bits, mode=omode)
        got = dict(scale=scale.cpu().numpy()[:n_live], bias=bias.cpu().numpy()[:n_live],
                   codes=O.unpack(packed.cpu().numpy()[:n_live * prb].reshape(n_live, prb), dim, bits))
        assert np.array_equal(got["scale"].view(np.uint32), ora["scale"].view(np.uint32)), what
        assert np.array_equal(got["bias"].view(np.uint32), ora["bias"].view(np.uint32)), what
        diff = np.abs(got["codes"].astype(np.int16) - ora["codes"].astype(np.int16))
        # cases are far too small for a share of 1e-4 to allow one element: every differing code has to
        # be a proven near-tie, and the share is checked over the whole sweep
        n_diff += assert_near_ties(host[ids_np[:n_live].astype(np.int64)], ora, diff, what=what)
        n_elements += diff.size
        want = np.full_like(host, -3.0)
        O.restore_rows(want, ids_np[:n_live], bits, packed.cpu().numpy()[:n_live * prb].reshape(n_live, prb), got["scale"], got["bias"])
        assert np.array_equal(stale.cpu().numpy(), want), what
        n_cases += 1
    assert n_cases > 100
    assert n_diff <= CODE_MISMATCH_FRACTION * n_elements, (n_diff, n_elements)
    print("random sweep: %d cases, %d of %d codes differ (all near-ties)" % (n_cases, n_diff, n_elements), flush=True)
    _poll_clean(ctx)
