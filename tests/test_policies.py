"""Incremental checkpoint policies (Section 5.1): the host-side state machine against a simulation
that uses the oracle's predictor, and - on the GPU - that a table restored from a baseline plus the
latest one-shot incremental equals the one restored from a baseline plus the whole chain of
consecutive incrementals, and that both equal what the oracle says a quantized checkpoint of the
final table must restore to."""
import numpy as np
import pytest
import torch

import oracle as O
import paper_2010_08679_amd as P
from paper_2010_08679_amd import synth


def _simulate(kind, fractions):
    """Reference state machine written from the paper's text, with the oracle's inequality."""
    out, history = [], []
    for f in fractions:
        if kind == "one_shot":
            out.append((False, False))
        elif kind == "consecutive":
            out.append((False, True))
        else:
            if O.full_checkpoint_due(history):
                out.append((True, True))
                history = []
            else:
                out.append((False, False))
                history.append(f)
    return out


@pytest.mark.parametrize("kind,code", [("one_shot", P.CNR_POLICY_ONE_SHOT), ("consecutive", P.CNR_POLICY_CONSECUTIVE),
                                       ("intermittent", P.CNR_POLICY_INTERMITTENT)])
def test_policy_state_machine(kind, code):
    rng = np.random.default_rng(3)
    for trial in range(20):
        # sizes that grow after every full checkpoint, as in the paper's measurements
        fractions, level = [], 0.2
        for _ in range(40):
            level = min(1.0, level + rng.uniform(0.0, 0.08))
            fractions.append(level)
        pol = P.cnr_policy_init(code)
        got = []
        for i, f in enumerate(fractions):
            d = P.cnr_policy_next(pol, f)
            got.append(d)
            if d[0]:
                # a full checkpoint resets the growth in this synthetic trace
                for j in range(i + 1, len(fractions)):
                    fractions[j] = min(1.0, 0.2 + (fractions[j] - fractions[i]))
        assert got == _simulate(kind, fractions)


def test_intermittent_switches_at_interval_eight_on_paper_like_growth():
    # Section 6.3.1: sizes from ~25 % growing past 50 % after ten intervals -> full checkpoint at 8
    pol = P.cnr_policy_init(P.CNR_POLICY_INTERMITTENT)
    decisions = [P.cnr_policy_next(pol, 0.25 + 0.03 * k) for k in range(10)]
    assert [d[0] for d in decisions].index(True) + 1 == 8


@pytest.mark.gpu
def test_one_shot_and_consecutive_chains_restore_the_same_table():
    dev = "cuda:0"
    ctx = P.cnr_create(0)
    n_rows, dim, bits, intervals = 60_000, 64, 8, 5
    table = synth.table_normal(n_rows, dim, 0.05, 1, dev)
    baseline = table.clone()
    one = P.TableCheckpointer(ctx, n_rows, dim, device=dev)
    con = P.TableCheckpointer(ctx, n_rows, dim, device=dev)
    one.clear()
    con.clear()
    pol_one = P.cnr_policy_init(P.CNR_POLICY_ONE_SHOT)
    pol_con = P.cnr_policy_init(P.CNR_POLICY_CONSECUTIVE)
    z = synth.ZipfSampler(n_rows, 1.05, 9, dev)
    g = torch.Generator(device=dev).manual_seed(5)
    chain, latest, touched = [], None, []

    def snapshot(ck, enc):
        n = enc.count()
        prb = P.cnr_packed_row_bytes(dim, bits)
        return dict(n=n, ids=enc.row_ids[:n].clone(), scale=enc.scale[:n].clone(), bias=enc.bias[:n].clone(),
                    packed=enc.packed[:n * prb].clone())

    for it in range(intervals):
        for _ in range(3):                                      # three training iterations per interval
            idx = z.draw(4096)
            touched.append(idx.cpu().numpy())
            one.mark(idx)
            con.mark(idx)
            rows = torch.unique(idx)
            table[rows] += 0.01 * torch.randn((rows.numel(), dim), device=dev, generator=g)
        for ck, pol, keep in ((one, pol_one, "latest"), (con, pol_con, "chain")):
            ck.compact()
            enc = ck.alloc_output(bits)
            ck.encode(table, enc)
            full, clear = P.cnr_policy_next(pol, enc.count() / n_rows)
            assert not full
            snap = snapshot(ck, enc)
            if keep == "latest":
                latest = snap
                assert not clear
            else:
                chain.append(snap)
                assert clear
                ck.clear()

    def apply(target, snap):
        n_dev = torch.tensor([snap["n"]], dtype=torch.int64, device=dev)
        P.cnr_restore_rows(ctx, target, n_rows, dim, snap["ids"], n_dev, snap["n"], bits, snap["packed"],
                           snap["scale"], snap["bias"])

    a = baseline.clone()
    apply(a, latest)
    b = baseline.clone()
    for snap in chain:
        apply(b, snap)
    torch.cuda.synchronize()
    assert torch.equal(a, b)                                    # same table either way, bit for bit
    assert sum(s["n"] for s in chain) > latest["n"]             # the chain stores some rows twice

    # against the oracle: rows ever looked up hold the de-quantized final values, the rest the baseline
    dirty = np.unique(np.concatenate(touched)).astype(np.uint32)
    assert latest["n"] == dirty.size and np.array_equal(latest["ids"].cpu().numpy().view(np.uint32), dirty)
    final = table.cpu().numpy()
    ref = O.quantize_rows(final, dirty, bits)
    want = baseline.cpu().numpy()
    want[dirty] = O.dequantize(ref["codes"], ref["scale"], ref["bias"])
    got = a.cpu().numpy()
    diff = got != want
    assert diff.mean() <= 1e-4
    step = np.zeros(n_rows, dtype=np.float32)
    step[dirty] = ref["scale"]
    assert np.all(np.abs(got - want)[diff] <= 1.0001 * np.broadcast_to(step[:, None], got.shape)[diff])
    st, bad, flags = P.cnr_poll_errors(ctx)
    assert (st, bad, flags) == (P.CNR_OK, 0, 0)
    P.cnr_destroy(ctx)
