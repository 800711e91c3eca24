"""Pins of the oracle's sparse driver (no GPU).

At full size the tables exist only as the input generator's value function, and
oracle/sparse_tables.py feeds the oracle's step functions with the rows of the
distinct keys.  It decides which W / A values enter every step after the first,
so it is checked here against the route that needs no such bookkeeping: the
same oracle step functions on dense host tables (pk_oracle.forward /
backward_update), on shrunk configurations, over enough steps that rows are
revisited.  Everything must agree to the bit: both routes call the same
arithmetic in the same order, only the storage differs.
"""
import numpy as np
import pytest

import synth
from oracle import pk_oracle as orc
from oracle.sparse_tables import SparseOracle


def _dense_tables(wl, pl):
    Wt = [synth.table_rows(wl, t) for t in range(len(wl.tables))]
    W = []
    for p in range(pl.n_packs):
        ts = [t for t in range(len(Wt)) if pl.table_pack[t] == p]
        W.append(np.ascontiguousarray(np.concatenate([Wt[t] for t in ts], axis=0)))
    return W


@pytest.mark.parametrize("idx,shrink", [
    (3, dict(batch=97, row_scale=0.0005, n_fields=24)),    # mean pooling, four packs
    (4, dict(batch=61, row_scale=0.01, n_fields=40)),      # raw 64-bit hashed IDs, two interleaved packs
    (5, dict(batch=16, row_scale=0.001, n_fields=6, len_scale=0.1)),   # bf16 tables, long bags
])
def test_sparse_driver_equals_dense_route_over_revisited_rows(idx, shrink):
    wl = synth.config(idx, **shrink)
    so = SparseOracle(orc, synth, wl)
    pl = so.pl
    W = _dense_tables(wl, pl)
    W0 = [w.copy() for w in W]
    A = [np.zeros(w.shape, np.float32) for w in W]
    batches = synth.make_batches(wl, 4)
    revisited = 0
    touched = [np.zeros(w.shape[0], bool) for w in W]
    for s, b in enumerate(batches):
        out_s, res = so.step(b, wl.lr, wl.eps)
        out_d, ctx = orc.forward(pl, W, wl.batch, b.ids, b.offsets)
        orc.backward_update(pl, W, A, ctx, wl.batch, b.grad_out, wl.lr, wl.eps)
        assert np.array_equal(out_s.view(np.uint32), out_d.view(np.uint32)), f"step {s}: pooled output"
        for p in range(pl.n_packs):
            r, c = res[p], ctx[p]
            assert np.array_equal(r["keys"], c.key)
            assert np.array_equal(r["packed_offsets"], c.packed_offsets)
            assert np.array_equal(r["unique"], c.unique)
            assert np.array_equal(r["inverse"], c.inverse)
            so_d, _ = orc.segments(c.inverse, len(c.unique))
            assert np.array_equal(r["seg_offsets"], so_d)
            rows = c.unique.astype(np.int64)
            revisited += int(touched[p][rows].sum())
            touched[p][rows] = True
            assert np.array_equal(r["W"].view(np.uint8), W[p][rows].view(np.uint8)), f"step {s} pack {p}: W rows"
            assert np.array_equal(r["A"].view(np.uint32), A[p][rows].view(np.uint32)), f"step {s} pack {p}: A rows"
            # what the driver remembers is the dense table's state on every row seen so far
            seen = so.keys_seen[p].astype(np.int64)
            assert np.array_equal(np.nonzero(touched[p])[0], seen)
            assert np.array_equal(so.W_seen[p].view(np.uint8), W[p][seen].view(np.uint8))
            assert np.array_equal(so.A_seen[p].view(np.uint32), A[p][seen].view(np.uint32))
    assert revisited > 0, "the case must revisit rows, or the bookkeeping is not exercised"
    # rows never touched are the generator's values on both routes
    for p in range(pl.n_packs):
        idle = np.nonzero(~touched[p])[0][:512]
        if len(idle):
            assert np.array_equal(so.init_rows(p, idle.astype(np.uint64)).view(np.uint8), W0[p][idle].view(np.uint8))
            assert np.array_equal(W[p][idle].view(np.uint8), W0[p][idle].view(np.uint8))


def test_current_rows_before_any_step_are_the_generator_values_with_zero_accumulators():
    wl = synth.config(3, batch=8, row_scale=0.0005, n_fields=8)
    so = SparseOracle(orc, synth, wl)
    W = _dense_tables(wl, so.pl)
    for p in range(so.pl.n_packs):
        R = W[p].shape[0]
        uq = np.unique(np.random.default_rng(p).integers(0, R, size=200)).astype(np.uint64)
        Wr, Ar = so.current_rows(p, uq)
        assert np.array_equal(Wr, W[p][uq.astype(np.int64)])
        assert (Ar == 0).all()


def test_widen_rows_is_the_oracles_own_widening_on_every_bf16_pattern():
    bits = np.arange(65536, dtype=np.uint16)
    got = orc.widen_rows(bits.reshape(-1, 16), orc.BF16).reshape(-1)
    ref = np.array([orc.lib().orc_bf16_widen(int(b)) for b in bits], np.float64)
    both_nan = np.isnan(got) & np.isnan(ref)
    assert np.array_equal(got[~both_nan], ref[~both_nan])
    assert both_nan.sum() == np.isnan(ref).sum() == np.isnan(got).sum()
    # and the same values as the gather step itself returns for a bf16 table
    tab = np.ascontiguousarray(bits.reshape(-1, 16))
    E = orc.gather(tab, orc.BF16, np.arange(tab.shape[0], dtype=np.uint64))
    assert np.array_equal(E[~np.isnan(E)], orc.widen_rows(tab, orc.BF16)[~np.isnan(E)])
    f = np.random.default_rng(0).standard_normal((7, 5)).astype(np.float32)
    assert np.array_equal(orc.widen_rows(f, orc.F32), f.astype(np.float64))
