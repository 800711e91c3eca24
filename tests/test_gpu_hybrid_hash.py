"""HybridHash (Sec. III-D, Alg. 1) on the GPU against the oracle: the Hot-storage never changes a value the
layer computes, and its content, FCounter and the hit counts follow the algorithm."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import pk_oracle as orc
from oracle.hybrid_hash import HybridHashOracle
from helpers import small_problem, stack_tables

pytestmark = pytest.mark.gpu


def close(got, ref, bf16=False):
    rel = 2e-2 if bf16 else 1e-5
    return bool(np.all(np.abs(got.astype(np.float64) - ref.astype(np.float64)) <= 1e-6 + rel * np.abs(ref)))


def logical_rows(layer, p):
    """Every row of pack p where it currently lives: the Hot-storage if it has a slot, else the Cold-storage."""
    h = layer.hh[p]
    slot = h["slot_of"].cpu().numpy()
    W = layer.W[p].float().cpu().numpy().copy()
    A = layer.A[p].cpu().numpy().copy()
    hot = slot >= 0
    Wh = h["W_hot"].float().cpu().numpy()
    Ah = h["A_hot"].cpu().numpy()
    W[hot] = Wh[slot[hot]]
    A[hot] = Ah[slot[hot]]
    return W, A, slot


@pytest.mark.parametrize("cold_on_host,dtype", [(True, 0), (False, 0), (True, 1)])
def test_hybrid_hash_follows_alg1_and_is_transparent(cold_on_host, dtype):
    from paper_2204_04903_amd.layer import HybridEmbedding
    tables = [(90, 8, dtype), (60, 16, dtype), (120, 8, dtype), (40, 16, dtype)]
    fields = [(0, 0), (1, 1), (2, 0), (0, 1), (3, 0), (2, 0)]
    n_steps, warmup, flush = 9, 2, 3
    steps = [small_problem(300 + s, B=24, tables=tables, fields=fields, max_len=6) for s in range(n_steps)]
    pl = orc.plan(tables, fields)
    hot_rows = [25, 0 if dtype else 400]          # pack 0: a real cache; pack 1: none / room for every row
    layer = HybridEmbedding(tables, fields, hot_rows, warmup, flush, cold_on_host=cold_on_host)
    try:
        for t, w in enumerate(steps[0]["Wt"]):
            layer.load_table(t, w)
        W = stack_tables(pl, [w.copy() for w in steps[0]["Wt"]])
        A = [np.zeros(w.shape, np.float32) for w in W]
        oracles = [HybridHashOracle(int(pl.pack_rows[p]), hot_rows[p], warmup, flush) for p in range(pl.n_packs)]
        f32 = lambda w: w if dtype == 0 else (w.astype(np.uint32) << 16).view(np.float32)
        for itr, pr in enumerate(steps):
            ids = torch.from_numpy(pr["ids"]).cuda()
            offsets = torch.from_numpy(pr["offsets"]).cuda()
            grad = torch.from_numpy(pr["grad"]).cuda()
            # bf16: the rows on the device may sit one bf16 step away from the oracle's after an update
            # (both are inside the row band, checked below), and pooled sums of such rows can cancel.  The
            # pooled output is therefore held, within the band for bf16 tables, against the oracle's
            # forward pass over the rows the device holds at this moment.
            W_now = W
            if dtype == 1:
                W_now = [(logical_rows(layer, p)[0].view(np.uint32) >> np.uint32(16)).astype(np.uint16)
                         for p in range(pl.n_packs)]
            out = layer.forward(ids, offsets, pr["B"])
            layer.backward_update(grad, 0.05, 1e-8)
            queried, hits, flushed = layer.end_iteration()
            torch.cuda.synchronize()
            assert layer.error_word() == 0
            ref_out, ctx = orc.forward(pl, W, pr["B"], pr["ids"], pr["offsets"])
            ref_now = ref_out if dtype == 0 else orc.forward(pl, W_now, pr["B"], pr["ids"], pr["offsets"])[0]
            assert close(out.cpu().numpy(), ref_now, bf16=dtype == 1), f"iteration {itr}: pooled output"
            orc.backward_update(pl, W, A, ctx, pr["B"], pr["grad"], 0.05, 1e-8)
            for p in range(pl.n_packs):
                hit, fl = oracles[p].iteration(ctx[p].unique.astype(np.int64), itr)
                assert queried[p] == len(ctx[p].unique) and hits[p] == int(hit.sum()), f"iteration {itr} pack {p}: hits"
                assert flushed == fl
                n_hot = layer.hot_count(p)
                got_hot = layer.hh[p]["hot_row"].cpu().numpy()[:n_hot].astype(np.int64)     # slots in any order
                assert np.array_equal(np.sort(got_hot), oracles[p].hot), f"iteration {itr} pack {p}: Hot-storage content"
                assert np.array_equal(layer.hh[p]["fcounter"].cpu().numpy().astype(np.int64), oracles[p].fcounter)
                Wl, Al, slot = logical_rows(layer, p)
                assert int((slot >= 0).sum()) == n_hot and np.array_equal(slot[got_hot], np.arange(n_hot))
                assert close(Wl, f32(W[p]), bf16=dtype == 1), f"iteration {itr} pack {p}: rows"
                assert close(Al, A[p]), f"iteration {itr} pack {p}: accumulators"
        assert sum(o.fcounter.sum() for o in oracles) > 0 and any(len(o.hot) for o in oracles)
    finally:
        layer.close()


def test_selection_at_the_count_cap_follows_the_oracle():
    # rows queried in 65535 iterations or more are equally hot: FCounter is set by hand (nobody runs that many
    # iterations in a test) and the reloads that follow must pick the rows the oracle picks
    from paper_2204_04903_amd.layer import HybridEmbedding
    tables, fields = [(64, 8, 0)], [(0, 0)]
    steps = [small_problem(700 + s, B=6, tables=tables, fields=fields, max_len=2) for s in range(3)]
    pl = orc.plan(tables, fields)
    layer = HybridEmbedding(tables, fields, [5], 0, 1, cold_on_host=False)
    try:
        layer.load_table(0, steps[0]["Wt"][0])
        oracle = HybridHashOracle(64, 5, 0, 1)
        preset = {3: 70000, 10: 65535, 11: 65534, 20: 900000, 30: 65535, 40: 65533, 41: 65536, 50: 12}
        fc = torch.zeros(64, dtype=torch.int32)
        for r, v in preset.items():
            fc[r] = v
            oracle.fcounter[r] = v
        torch.cuda.synchronize()
        layer.hh[0]["fcounter"].copy_(fc.cuda())
        W = stack_tables(pl, [steps[0]["Wt"][0].copy()])
        for itr, pr in enumerate(steps):
            out = layer.forward(torch.from_numpy(pr["ids"]).cuda(), torch.from_numpy(pr["offsets"]).cuda(), pr["B"])
            layer.backward_update(torch.from_numpy(pr["grad"]).cuda(), 0.05, 1e-8)
            queried, hits, flushed = layer.end_iteration()
            torch.cuda.synchronize()
            _, ctx = orc.forward(pl, W, pr["B"], pr["ids"], pr["offsets"])
            hit, fl = oracle.iteration(ctx[0].unique.astype(np.int64), itr)
            assert flushed == fl and hits[0] == int(hit.sum())
            n_hot = layer.hot_count(0)
            got_hot = layer.hh[0]["hot_row"].cpu().numpy()[:n_hot].astype(np.int64)
            assert np.array_equal(np.sort(got_hot), oracle.hot), f"iteration {itr}: {np.sort(got_hot)} vs {oracle.hot}"
            assert np.array_equal(layer.hh[0]["fcounter"].cpu().numpy().astype(np.int64), oracle.fcounter)
        assert len(oracle.hot) == 5 and all(oracle.fcounter[r] >= 65535 for r in oracle.hot)      # rows at the cap fill it
    finally:
        layer.close()
