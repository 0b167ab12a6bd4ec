"""The compaction for callers that cannot allocate (cnr_compact_dirty_noalloc) against the plain call
(cnr_compact_dirty): same dirty-row list and count, bit for bit, through the C ABI, on calls in a row
that share the library's fixed scratch array -- the second on a smaller table, so that whatever the
first left in the array would show.  Collected last on purpose (file name)."""
import numpy as np
import pytest
import torch

import paper_2010_08679_amd as P

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _bitmap(n_rows, p, seed):
    g = torch.Generator(device=DEV).manual_seed(seed)
    words = P.cnr_bitmap_words(n_rows)
    bits = torch.rand(words * 32, generator=g, device=DEV) < p
    bits[n_rows:] = True                                       # padding bits must be ignored
    w = (bits.reshape(words, 32).to(torch.int64) << torch.arange(32, device=DEV)).sum(dim=1)
    return w.to(torch.int32)                                   # wraps to the same 32 bits


def _both(ctx, bm, n_rows, capacity):
    out = []
    for noalloc in (False, True):
        ids = torch.full((max(1, capacity),), -1, dtype=torch.int32, device=DEV)
        n_dev = torch.full((1,), -1, dtype=torch.int64, device=DEV)
        if noalloc:
            P.cnr_compact_dirty_noalloc(ctx, bm, n_rows, ids, capacity, n_dev)
        else:
            scratch = torch.empty((P.cnr_scratch_bytes(n_rows) + 7) // 8, dtype=torch.int64, device=DEV)
            P.cnr_compact_dirty(ctx, bm, n_rows, ids, capacity, n_dev, scratch)
        torch.cuda.synchronize()
        out.append((ids.cpu().numpy(), int(n_dev.item())))
    return out


def test_noalloc_compaction_equals_the_plain_call_on_calls_in_a_row():
    ctx = P.cnr_create(0)
    try:
        # large first, then smaller ones: tiles 0 .. 305, then 13, then 1, then an empty table
        for n_rows, p, seed in ((5_000_003, 0.3, 1), (200_001, 0.7, 2), (777, 0.5, 3), (0, 0.0, 4), (1_000_000, 0.01, 5)):
            print("case noalloc compact n_rows=%d p=%.2f" % (n_rows, p), flush=True)
            bm = _bitmap(max(n_rows, 1), p, seed)
            (ids_a, n_a), (ids_b, n_b) = _both(ctx, bm, n_rows, n_rows)
            assert n_a == n_b, (n_rows, n_a, n_b)
            assert np.array_equal(ids_a, ids_b), n_rows
            if n_rows:
                want = torch.nonzero(torch.rand(P.cnr_bitmap_words(n_rows) * 32,
                                                generator=torch.Generator(device=DEV).manual_seed(seed),
                                                device=DEV)[:n_rows] < p).reshape(-1).cpu().numpy()
                assert n_a == want.size and np.array_equal(ids_a[:n_a].view(np.uint32), want.astype(np.uint32))
        # a list that does not fit: same truncation, same count, same flag
        bm = _bitmap(100_000, 0.5, 9)
        (ids_a, n_a), (ids_b, n_b) = _both(ctx, bm, 100_000, 1000)
        assert n_a == n_b and n_a > 1000 and np.array_equal(ids_a, ids_b)
        st, _, flags = P.cnr_poll_errors(ctx)
        assert st == P.CNR_E_CAPACITY and flags == P.CNR_FLAG_CAPACITY
        # beyond the fixed maximum: refused before anything is launched
        with pytest.raises(P.CnrError) as e:
            P.cnr_compact_dirty_noalloc(ctx, bm, P.CNR_NOALLOC_MAX_ROWS + 1, None, 0,
                                        torch.zeros(1, dtype=torch.int64, device=DEV))
        assert e.value.status == P.CNR_E_TOO_LARGE
        st, bad, flags = P.cnr_poll_errors(ctx)
        assert (st, bad, flags) == (P.CNR_OK, 0, 0)
    finally:
        torch.cuda.synchronize()
        P.cnr_destroy(ctx)
