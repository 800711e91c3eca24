"""Pins of the CPU oracle against things other than itself: library routines
(numpy.unique, torch embedding_bag, torch.optim.Adagrad), Python big-integer
arithmetic, closed forms, exactness on integer-valued data, invariants, and the
examples the paper states (see tests/golden/)."""
import os

import numpy as np
import pytest
import torch

import synth
from oracle import pk_oracle as orc
from helpers import small_problem, stack_tables

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# --------------------------------------------------------------------------- plan
def _read_golden(name):
    rows = []
    with open(os.path.join(GOLDEN, name)) as fh:
        for line in fh:
            line = line.split("#")[0].strip()
            if line:
                rows.append(line.split())
    return rows


def test_plan_fig7_three_same_dim_fields_make_one_pack():
    # Fig. 7: three embedding tables looked up by one packed set of operators.
    (n_tables, n_packs), = [(int(a), int(b)) for a, b in _read_golden("fig7_packing.txt")]
    pl = orc.plan([(100, 8, 0)] * n_tables, [(t, 0) for t in range(n_tables)])
    assert pl.n_packs == n_packs
    assert list(pl.table_base) == [0, 100, 200] and list(pl.field_col) == [0, 8, 16]


def test_plan_pack_counts_of_the_five_configurations():
    # stated with the workload configurations: 1 / 1 / 4 / 2 / 1 packs
    for idx, n in zip(range(1, 6), (1, 1, 4, 2, 1)):
        wl = synth.config(idx, row_scale=0.001)
        pl = orc.plan([(t.rows, t.dim, t.dtype) for t in wl.tables], [(f.table, f.pool) for f in wl.fields])
        assert pl.n_packs == n
        # number of packs depends on distinct dims, not on the number of fields (Sec. III-B)
        assert pl.n_packs == len({(t.dim, t.dtype) for t in wl.tables})


def test_plan_layout_closed_forms():
    tables = [(10, 16, 0), (20, 8, 0), (30, 16, 0), (40, 8, 1), (50, 8, 0)]
    fields = [(2, 0), (1, 1), (0, 0), (4, 0), (3, 0), (1, 0)]
    pl = orc.plan(tables, fields)
    # packs ascending by (dim, dtype): (8,f32) (8,bf16) (16,f32)
    assert list(zip(pl.pack_dim, pl.pack_dtype)) == [(8, 0), (8, 1), (16, 0)]
    assert list(pl.table_pack) == [2, 0, 2, 1, 0]
    assert list(pl.table_base) == [0, 0, 10, 0, 20]
    assert list(pl.pack_rows) == [70, 40, 40]
    assert list(pl.field_pack) == [2, 0, 2, 0, 1, 0]
    assert list(pl.field_slot) == [0, 0, 1, 1, 0, 2]
    assert list(pl.field_col) == [0, 16, 24, 40, 48, 56] and pl.out_dim == 64
    assert [list(x) for x in pl.pack_fields] == [[1, 3, 5], [4], [0, 2]]


def test_eq1_volume_ratio_of_the_worked_example():
    # Sec. III-B after Eq. 1: uniform data, equally many tables of dim 8 and of
    # dim 32 -> the dim-32 pack carries four times the volume (hence 4 shards).
    (d_small, d_large, ratio), = [(int(a), int(b), float(c)) for a, b, c in _read_golden("eq1_example.txt")]
    n = 6
    tables = [(1000, d_small, 0)] * n + [(1000, d_large, 0)] * n
    pl = orc.plan(tables, [(t, 0) for t in range(2 * n)])
    occ = [512.0] * (2 * n)
    v0, v1 = orc.calc_vparam(pl, occ, 0), orc.calc_vparam(pl, occ, 1)
    assert v0 == n * d_small * 512.0           # floats gathered: dim x occurrences, summed over tables
    assert v1 / v0 == ratio


def test_eq1_shard_split_reproduces_the_worked_example():
    # Sec. III-B after Eq. 1: uniform data, one packed operation for the dim-8 tables ->
    # the dim-32 tables get four shards, each holding a quarter of them.
    (d_small, d_large, ratio), = [(int(a), int(b), float(c)) for a, b, c in _read_golden("eq1_example.txt")]
    n = 8
    tables = [(1000 + t, d_small, 0) for t in range(n)] + [(2000 + t, d_large, 0) for t in range(n)]
    fields = [(t, 0) for t in range(2 * n)]
    pl = orc.plan(tables, fields, max_shards=8)                       # uniform volumes
    assert list(pl.shards) == [1, int(ratio)]
    assert pl.n_packs == 1 + int(ratio)
    assert list(pl.pack_dim) == [d_small] + [d_large] * int(ratio)
    per_shard = [int((pl.table_pack[n:] == 1 + s).sum()) for s in range(int(ratio))]
    assert per_shard == [n // int(ratio)] * int(ratio)                # a quarter of the tables each
    assert list(pl.table_pack[:n]) == [0] * n


def test_eq1_only_packs_above_the_average_are_split():
    # Sec. III-B: a packed operation is split when its volume is above the average.  Three packs with
    # volumes V, 1.6 V and 4 V (average 2.2 V): only the last one is split, into 4; a rule that split
    # every pack by its ratio to the lightest would cut the middle one in two as well.
    n = 8
    tables = [(100, 10, 0)] * n + [(100, 16, 0)] * n + [(100, 40, 0)] * n
    fields = [(t, 0) for t in range(3 * n)]
    pl = orc.plan(tables, fields, max_shards=8)
    occ = [1.0] * (3 * n)
    v = [orc.calc_vparam(pl0 := orc.plan(tables, fields), occ, p) for p in range(3)]
    assert v[1] / v[0] == 1.6 and v[2] / v[0] == 4.0
    assert list(pl.shards) == [1, 1, 4]
    assert pl.n_packs == 6


def test_eq1_shard_split_rule_against_plain_python():
    # the same rule written out in Python on an irregular problem: volumes from per-field
    # statistics, rounding, both caps, tables dealt in turn, stacking per shard
    rng = np.random.default_rng(5)
    dims = [4, 4, 16, 16, 16, 16, 16, 8, 8, 8, 64]
    tables = [(int(rng.integers(5, 50)), d, 0) for d in dims]
    fields = [(t, 0) for t in range(len(tables))] + [(2, 1), (10, 0)]
    vol = [float(v) for v in rng.integers(1, 100, size=len(fields))]
    for max_shards in (2, 3, 16):
        pl = orc.plan(tables, fields, max_shards=max_shards, field_volume=vol)
        occ = [0.0] * len(tables)
        for f, (t, _) in enumerate(fields):
            occ[t] += vol[f]
        base = sorted(set(dims))
        V = {d: sum(d * occ[t] for t in range(len(tables)) if dims[t] == d) for d in base}
        vmin = min(V.values())
        vmean = sum(V.values()) / len(V)
        exp_pack, exp_base, exp_rows, q0 = {}, {}, [], 0
        exp_shards = []
        for d in base:
            ts = [t for t in range(len(tables)) if dims[t] == d]
            s = max(1, min(int(np.floor(V[d] / vmin + 0.5)) if V[d] > vmean else 1, max_shards, len(ts)))
            exp_shards.append(s)
            rows_acc = [0] * s
            for i, t in enumerate(ts):
                exp_pack[t] = q0 + i % s
                exp_base[t] = rows_acc[i % s]
                rows_acc[i % s] += tables[t][0]
            exp_rows += rows_acc
            q0 += s
        assert list(pl.shards) == exp_shards
        assert pl.n_packs == q0
        assert [int(x) for x in pl.table_pack] == [exp_pack[t] for t in range(len(tables))]
        assert [int(x) for x in pl.table_base] == [exp_base[t] for t in range(len(tables))]
        assert [int(x) for x in pl.pack_rows] == exp_rows
        # fields follow their tables; slots count the pack's fields in field order
        for f, (t, _) in enumerate(fields):
            assert pl.field_pack[f] == exp_pack[t]
            assert pl.field_slot[f] == sum(1 for g in range(f) if exp_pack[fields[g][0]] == exp_pack[t])
    # a split changes where rows live, not what the layer computes
    pr = small_problem(31, B=5, tables=tables, fields=fields, max_len=3)
    outs = []
    for ms in (0, 16):
        pl = orc.plan(tables, fields, max_shards=ms, field_volume=vol)
        out, _ = orc.forward(pl, stack_tables(pl, pr["Wt"]), pr["B"], pr["ids"], pr["offsets"])
        outs.append(out)
    assert np.array_equal(outs[0], outs[1])


# --------------------------------------------------------------------------- keys
def test_eq2_micro_batch_size_hand_worked_and_brute_force():
    # Sec. III-C, Eq. 2.  By hand: 1000 samples; one operator may use 10000 units at 30 per sample (333
    # samples), another 8000 at 20 (400): the first one binds, 333 samples need 4 micro-batches, and an even
    # cut makes them 250 each.
    assert orc.micro_batch_size(1000, [10000, 8000], [30, 20]) == 250
    assert orc.micro_batch_size(1000, [8000, 10000], [20, 30]) == 250          # the order of operators is irrelevant
    assert orc.micro_batch_size(1000, [1e12], [1.0]) == 1000                   # nothing binds: the whole batch
    assert orc.micro_batch_size(10, [5.0], [7.0]) == 0                         # not even one sample fits
    assert orc.micro_batch_size(10, [7.0], [7.0]) == 1
    # brute force: the largest size within every bound, then the fewest equal micro-batches of at most that size
    rng = np.random.default_rng(5)
    for _ in range(200):
        B = int(rng.integers(1, 5000))
        n = int(rng.integers(1, 4))
        ri = rng.integers(1, 1000, size=n).astype(np.float64)
        rb = rng.integers(1, 2_000_000, size=n).astype(np.float64)
        fit = [b for b in range(1, B + 1) if all(b * ri[o] <= rb[o] for o in range(n))]
        want = 0
        if fit:
            M = min(m for m in range(1, B + 1) if -(-B // m) <= fit[-1])
            want = -(-B // M)
        assert orc.micro_batch_size(B, rb, ri) == want


def test_keys_match_python_bigint_arithmetic_on_wild_ids():
    pr = small_problem(3, B=9, wild_ids=True)
    pr["ids"][:4] = [-1, -2**63, 2**63 - 1, 0]
    pl = orc.plan(pr["tables"], pr["fields"])
    B = pr["B"]
    for p in range(pl.n_packs):
        key, po = orc.pack_keys(pl, p, B, pr["ids"], pr["offsets"])
        exp_keys, exp_po = [], []
        for f in pl.pack_fields[p]:
            t = pr["fields"][f][0]
            for b in range(B):
                exp_po.append(len(exp_keys))
                for i in range(pr["offsets"][f * B + b], pr["offsets"][f * B + b + 1]):
                    u = int(pr["ids"][i]) & ((1 << 64) - 1)            # reinterpret as unsigned
                    exp_keys.append(int(pl.table_base[t]) + u % pr["tables"][t][0])
        exp_po.append(len(exp_keys))
        assert [int(x) for x in key] == exp_keys
        assert list(po) == exp_po


def test_keys_in_range_ids_are_fixed_points_and_tables_do_not_collide():
    pr = small_problem(4, B=16)
    pl = orc.plan(pr["tables"], pr["fields"])
    B = pr["B"]
    for p in range(pl.n_packs):
        key, po = orc.pack_keys(pl, p, B, pr["ids"], pr["offsets"])
        for j, f in enumerate(pl.pack_fields[p]):
            t = pr["fields"][f][0]
            seg = key[po[j * B]:po[(j + 1) * B]].astype(np.int64)
            raw = pr["ids"][pr["offsets"][f * B]:pr["offsets"][(f + 1) * B]]
            assert (seg - pl.table_base[t] == raw).all()
            assert (seg >= pl.table_base[t]).all() and (seg < pl.table_base[t] + pr["tables"][t][0]).all()
        # packed offsets = the fields' own offsets, rebased and concatenated
        lens = np.concatenate([np.diff(pr["offsets"][f * B:(f + 1) * B + 1]) for f in pl.pack_fields[p]])
        assert (np.diff(po) == lens).all() and po[0] == 0


# --------------------------------------------------------------------------- unique
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_unique_matches_numpy_and_invariants(seed):
    rng = np.random.default_rng(seed)
    key = rng.integers(0, 50, size=400).astype(np.uint64)
    key[::7] = np.uint64(2**40 + 5)                     # wide keys too
    uq, inv = orc.unique(key)
    nu, ninv = np.unique(key, return_inverse=True)
    assert (uq == nu).all() and (inv == ninv).all()
    assert (np.diff(uq.astype(np.int64)) > 0).all()
    assert (uq[inv] == key).all() and len(uq) == len(set(key.tolist()))
    so, sp = orc.segments(inv, len(uq))
    assert (np.diff(so) == np.bincount(inv, minlength=len(uq))).all()
    assert (sp == np.argsort(inv, kind="stable")).all()


def test_unique_empty_and_single():
    uq, inv = orc.unique(np.zeros(0, np.uint64))
    assert len(uq) == 0 and len(inv) == 0
    uq, inv = orc.unique(np.array([9, 9, 9], np.uint64))
    assert list(uq) == [9] and list(inv) == [0, 0, 0]


# --------------------------------------------------------------------------- forward
def _torch_forward(pr, Wt_f64):
    B = pr["B"]
    outs = []
    for f, (t, pm) in enumerate(pr["fields"]):
        rows = pr["tables"][t][0]
        a, b = pr["offsets"][f * B], pr["offsets"][(f + 1) * B]
        idx = torch.from_numpy((pr["ids"][a:b].astype(np.uint64) % np.uint64(rows)).astype(np.int64))
        off = torch.from_numpy((pr["offsets"][f * B:(f + 1) * B] - a).astype(np.int64))
        outs.append(torch.nn.functional.embedding_bag(idx, Wt_f64[t], off, mode="mean" if pm == 1 else "sum"))
    return torch.cat(outs, dim=1)


@pytest.mark.parametrize("seed", [10, 11])
def test_forward_matches_torch_embedding_bag(seed):
    pr = small_problem(seed, B=12)
    pl = orc.plan(pr["tables"], pr["fields"])
    out, ctx = orc.forward(pl, stack_tables(pl, pr["Wt"]), pr["B"], pr["ids"], pr["offsets"])
    ref = _torch_forward(pr, [torch.from_numpy(w.astype(np.float64)) for w in pr["Wt"]]).numpy()
    np.testing.assert_allclose(out, ref.astype(np.float32), rtol=2e-7, atol=1e-9)
    # the per-field route inside the oracle agrees too
    out2 = orc.direct_forward(pr["tables"], pr["fields"], pr["Wt"], pr["B"], pr["ids"], pr["offsets"])
    assert (out == out2).all()


def test_forward_integer_valued_tables_are_exact():
    # small integers: every partial sum is exact in fp32 and fp64, so sum pooling is exact in any order
    fields = [(0, 0), (1, 0), (2, 0), (0, 0), (3, 0)]
    pr = small_problem(12, B=10, fields=fields, int_valued=True, max_len=9)
    pl = orc.plan(pr["tables"], pr["fields"])
    out, _ = orc.forward(pl, stack_tables(pl, pr["Wt"]), pr["B"], pr["ids"], pr["offsets"])
    B = pr["B"]
    col = 0
    for f, (t, _) in enumerate(fields):
        D = pr["tables"][t][1]
        for b in range(B):
            acc = np.zeros(D, np.int64)
            for i in range(pr["offsets"][f * B + b], pr["offsets"][f * B + b + 1]):
                acc += pr["Wt"][t][pr["ids"][i]].astype(np.int64)
            assert (out[b, col:col + D] == acc).all()
        col += D


def test_forward_closed_forms_repeated_id_and_empty_bag_and_linearity():
    tables = [(6, 4, 0)]
    fields = [(0, 0), (0, 1)]
    B = 3
    # field 0 (sum): bags [2,2,2,2,2], [], [1] ; field 1 (mean): [3,3,3], [0,5], []
    ids = np.array([2, 2, 2, 2, 2, 1, 3, 3, 3, 0, 5], np.int64)
    offsets = np.array([0, 5, 5, 6, 9, 11, 11], np.int32)
    rng = np.random.default_rng(0)
    W1 = rng.standard_normal((6, 4)).astype(np.float32)
    W2 = rng.standard_normal((6, 4)).astype(np.float32)
    pl = orc.plan(tables, fields)
    o1, _ = orc.forward(pl, [W1], B, ids, offsets)
    np.testing.assert_array_equal(o1[0, 0:4], (5.0 * W1[2].astype(np.float64)).astype(np.float32))
    np.testing.assert_array_equal(o1[1, 0:4], 0)
    np.testing.assert_array_equal(o1[2, 0:4], W1[1])
    np.testing.assert_allclose(o1[0, 4:8], W1[3], rtol=1e-7)
    np.testing.assert_allclose(o1[1, 4:8], (W1[0].astype(np.float64) + W1[5]) / 2, rtol=1e-7)
    np.testing.assert_array_equal(o1[2, 4:8], 0)
    # linearity in the table
    o2, _ = orc.forward(pl, [W2], B, ids, offsets)
    o12, _ = orc.forward(pl, [(W1.astype(np.float64) + W2).astype(np.float32)], B, ids, offsets)
    np.testing.assert_allclose(o12, o1.astype(np.float64) + o2, rtol=1e-5, atol=1e-6)


# --------------------------------------------------------------------------- backward + Adagrad
def _torch_two_steps(pr_steps, tables, fields, Wt0, lr, eps):
    params = [torch.nn.Parameter(torch.from_numpy(w.astype(np.float64))) for w in Wt0]
    opt = torch.optim.Adagrad(params, lr=lr, eps=eps, initial_accumulator_value=0.0)
    for pr in pr_steps:
        opt.zero_grad()
        out = _torch_forward(pr, params)
        out.backward(torch.from_numpy(pr["grad"].astype(np.float64)))
        for p_ in params:                      # a table no field reads has no gradient
            if p_.grad is None:
                p_.grad = torch.zeros_like(p_)
        opt.step()
    return [p_.detach().numpy() for p_ in params], [opt.state[p_]["sum"].numpy() for p_ in params]


@pytest.mark.parametrize("seed", [20, 21])
def test_two_steps_match_torch_autograd_and_adagrad(seed):
    lr, eps = 0.05, 1e-8
    steps = [small_problem(seed * 100 + s, B=11) for s in range(2)]
    tables, fields = steps[0]["tables"], steps[0]["fields"]
    Wt0 = [w.copy() for w in steps[0]["Wt"]]
    pl = orc.plan(tables, fields)
    W = stack_tables(pl, Wt0)
    A = [np.zeros_like(w) for w in W]
    Wd = [w.copy() for w in Wt0]
    Ad = [np.zeros_like(w) for w in Wt0]
    for pr in steps:
        out, ctx = orc.forward(pl, W, pr["B"], pr["ids"], pr["offsets"])
        orc.backward_update(pl, W, A, ctx, pr["B"], pr["grad"], lr, eps)
        orc.direct_backward_update(tables, fields, Wd, Ad, pr["B"], pr["ids"], pr["offsets"], pr["grad"], lr, eps)
    Wref, Aref = _torch_two_steps(steps, tables, fields, Wt0, lr, eps)
    for t in range(len(tables)):
        p, base, rows = pl.table_pack[t], pl.table_base[t], tables[t][0]
        # step 2 starts from fp32-rounded state in the oracle, fp64 state in torch: one rounding apart
        np.testing.assert_allclose(W[p][base:base + rows], Wref[t], rtol=3e-7, atol=1e-8)
        np.testing.assert_allclose(A[p][base:base + rows], Aref[t], rtol=3e-7, atol=1e-12)
        assert (W[p][base:base + rows] == Wd[t]).all() and (A[p][base:base + rows] == Ad[t]).all()


def test_backward_closed_forms_duplicates_mean_scale_and_untouched_rows():
    tables = [(8, 2, 0)]
    fields = [(0, 0), (0, 1)]
    B = 2
    # field 0 (sum): [1,1,4], [1] ; field 1 (mean): [6,6,1,3], [3]
    ids = np.array([1, 1, 4, 1, 6, 6, 1, 3, 3], np.int64)
    offsets = np.array([0, 3, 4, 8, 9], np.int32)
    W0 = np.arange(16, dtype=np.float32).reshape(8, 2) / 8
    grad = np.array([[1.0, -2.0, 4.0, 8.0], [0.5, 0.25, -1.0, 3.0]], np.float32)
    lr, eps = 0.1, 1e-8
    pl = orc.plan(tables, fields)
    W = [W0.copy()]; A = [np.zeros_like(W0)]
    _, ctx = orc.forward(pl, W, B, ids, offsets)
    G = orc.scatter_add(pl, 0, B, grad, ctx[0].inverse, ctx[0].packed_offsets, len(ctx[0].unique))
    assert list(ctx[0].unique) == [1, 3, 4, 6]
    # row 1: twice in bag (0,f0), once in (1,f0), once of four in mean bag (0,f1)
    np.testing.assert_array_equal(G[0], [2 * 1.0 + 0.5 + 4.0 / 4, 2 * -2.0 + 0.25 + 8.0 / 4])
    np.testing.assert_array_equal(G[1], [4.0 / 4 + -1.0, 8.0 / 4 + 3.0])       # row 3
    np.testing.assert_array_equal(G[2], [1.0, -2.0])                            # row 4
    np.testing.assert_array_equal(G[3], [2 * 4.0 / 4, 2 * 8.0 / 4])             # row 6 twice in a mean bag
    orc.backward_update(pl, W, A, ctx, B, grad, lr, eps)
    # first step from A = 0: A' = g^2 with g the SUMMED gradient, W' = W - lr*g/(|g|+eps)
    for u, r in enumerate([1, 3, 4, 6]):
        np.testing.assert_allclose(A[0][r], G[u] ** 2, rtol=1e-7)
        with np.errstate(invalid="ignore"):
            step = np.where(G[u] != 0, lr * G[u] / (np.abs(G[u]) + eps), 0.0)
        np.testing.assert_allclose(W[0][r], W0[r] - step, rtol=1e-6)
    for r in [0, 2, 5, 7]:
        assert (W[0][r] == W0[r]).all() and (A[0][r] == 0).all()
    # k identical further steps: A = k * g^2
    for _ in range(2):
        _, ctx = orc.forward(pl, W, B, ids, offsets)
        orc.backward_update(pl, W, A, ctx, B, grad, lr, eps)
    np.testing.assert_allclose(A[0][4], 3 * G[2] ** 2, rtol=1e-6)


def test_integer_valued_gradients_reduce_exactly():
    pr = small_problem(31, B=13, int_valued=True, max_len=6)
    pl = orc.plan(pr["tables"], [(t, 0) for t, _ in pr["fields"]])      # sum pooling everywhere
    B = pr["B"]
    for p in range(pl.n_packs):
        key, po = orc.pack_keys(pl, p, B, pr["ids"], pr["offsets"])
        uq, inv = orc.unique(key)
        G = orc.scatter_add(pl, p, B, pr["grad"], inv, po, len(uq))
        D = int(pl.pack_dim[p])
        ref = np.zeros((len(uq), D), np.int64)
        q = 0
        for f in pl.pack_fields[p]:
            for b in range(B):
                for _ in range(pr["offsets"][f * B + b], pr["offsets"][f * B + b + 1]):
                    c = int(pl.field_col[f])
                    ref[inv[q]] += pr["grad"][b, c:c + D].astype(np.int64)
                    q += 1
        assert (G == ref).all()


# --------------------------------------------------------------------------- bf16
def test_bf16_rounding_closed_forms_and_torch():
    L = orc.lib()
    cases = {1.0: 0x3F80, 1.0 + 2.0 ** -8: 0x3F80, 1.0 + 3 * 2.0 ** -8: 0x3F82, 1.0 + 2.0 ** -8 + 2.0 ** -20: 0x3F81,
             -2.5: 0xC020, 0.0: 0x0000, 3.0e-5: None}
    for v, bits in cases.items():
        got = L.orc_bf16_round(np.float32(v))
        ref = int(torch.tensor([v], dtype=torch.float32).to(torch.bfloat16).view(torch.int16).item()) & 0xFFFF
        assert got == ref
        if bits is not None:
            assert got == bits
        assert abs(L.orc_bf16_widen(got) - v) <= abs(v) * 2.0 ** -8
    rng = np.random.default_rng(5)
    xs = (rng.standard_normal(2000) * 10.0 ** rng.integers(-6, 6, 2000)).astype(np.float32)
    ref = torch.from_numpy(xs).to(torch.bfloat16).view(torch.int16).numpy().astype(np.uint16)
    got = np.array([L.orc_bf16_round(x) for x in xs], np.uint16)
    assert (got == ref).all()


def test_bf16_tables_forward_and_update_within_band():
    tables = [(40, 8, 1), (30, 8, 1)]
    fields = [(0, 0), (1, 1), (0, 0)]
    pr = small_problem(41, B=9, tables=tables, fields=fields)
    pl = orc.plan(tables, fields)
    W = stack_tables(pl, pr["Wt"]); A = [np.zeros(w.shape, np.float32) for w in W]
    out, ctx = orc.forward(pl, W, pr["B"], pr["ids"], pr["offsets"])
    Wf = [torch.from_numpy(synth.bf16_bits_to_f32(w).astype(np.float64)) for w in pr["Wt"]]
    ref = _torch_forward(pr, Wf).numpy()
    np.testing.assert_allclose(out, ref.astype(np.float32), rtol=2e-7, atol=1e-9)   # widening is exact
    W0 = W[0].copy()
    orc.backward_update(pl, W, A, ctx, pr["B"], pr["grad"], 0.01, 1e-8)
    Wref, _ = _torch_two_steps([pr], tables, fields, [synth.bf16_bits_to_f32(w) for w in pr["Wt"]], 0.01, 1e-8)
    got = synth.bf16_bits_to_f32(W[0])
    np.testing.assert_allclose(got, np.concatenate(Wref, axis=0), rtol=2.0 ** -8, atol=1e-30)
    touched = np.zeros(W0.shape[0], bool); touched[ctx[0].unique.astype(np.int64)] = True
    assert (W[0][~touched] == W0[~touched]).all() and (~touched).any()


@pytest.mark.parametrize("n_owners", [1, 2, 3, 8])
def test_partition_matches_a_stable_numpy_sort_by_owner(n_owners):
    # Sec. II-D Partition: distinct keys regrouped by the worker that holds the row (row mod n), order kept
    rng = np.random.default_rng(n_owners)
    uq = np.unique(rng.integers(0, 5000, size=700)).astype(np.uint64)
    keys, idx, off = orc.partition(uq, n_owners)
    order = np.argsort((uq % np.uint64(n_owners)).astype(np.int64), kind="stable")
    assert np.array_equal(keys, uq[order])
    assert np.array_equal(idx, order.astype(np.int32))
    counts = np.bincount((uq % np.uint64(n_owners)).astype(np.int64), minlength=n_owners)
    assert np.array_equal(off, np.concatenate([[0], np.cumsum(counts)]).astype(np.int32))
    assert np.array_equal(uq[idx], keys)                     # Stitch's view: the index leads back to the key
    e_keys, e_idx, e_off = orc.partition(np.zeros(0, np.uint64), n_owners)
    assert len(e_keys) == 0 and list(e_off) == [0] * (n_owners + 1)
