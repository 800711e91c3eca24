"""Parity of the HIP path (through the C ABI) with the CPU oracle, element by
element on the same seeded inputs.

Bar: bit-exact keys / packed offsets / unique / inverse / segment offsets;
pooled outputs, updated rows and updated accumulators within
|gpu - ref| <= 1e-6 + 1e-5*|ref| for fp32 tables and 1e-6 + 2e-2*|ref| for bf16
tables (fp32 accumulation).  Rows the batch does not touch must keep their bits.
"""
import sys

import numpy as np
import pytest
import torch

import synth
from oracle import pk_oracle as orc
from oracle.sparse_tables import SparseOracle
from helpers import pooled_close, small_problem, stack_tables

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def close(got, ref, bf16=False):
    tol = 1e-6 + (2e-2 if bf16 else 1e-5) * np.abs(ref)
    bad = np.abs(got.astype(np.float64) - ref.astype(np.float64)) > tol
    return not bad.any(), int(bad.sum())


def f32_of(arr, dtype):
    return arr if dtype == 0 else synth.bf16_bits_to_f32(arr)


def bits_of(t: torch.Tensor):
    """Device table tensor -> numpy float32, or uint16 bit patterns for bf16."""
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def run_dense_case(name, tables, fields, steps, lr=0.05, eps=1e-8, out_pad=0, grad_pad=0, **plan_opts):
    """steps: list of dicts from small_problem (ids, offsets, grad, B, Wt of the first one)."""
    from paper_2204_04903_amd.layer import PackedEmbedding
    say(f"[case] {name}: tables={len(tables)} fields={len(fields)} steps={len(steps)}")
    pl = orc.plan(tables, fields, **{k: v for k, v in plan_opts.items() if k not in ("interleave_groups", "debug")})
    Wt0 = steps[0]["Wt"]
    W = stack_tables(pl, [w.copy() for w in Wt0])
    A = [np.zeros(w.shape, np.float32) for w in W]
    layer = PackedEmbedding(tables, fields, **plan_opts)
    assert layer.n_packs == pl.n_packs
    try:
        for t, w in enumerate(Wt0):
            layer.load_table(t, w)
        for s, pr in enumerate(steps):
            B = pr["B"]
            ids = torch.from_numpy(pr["ids"]).cuda()
            offsets = torch.from_numpy(pr["offsets"]).cuda()
            out_buf = torch.full((B, layer.out_dim + out_pad), 7.0, dtype=torch.float32, device="cuda")
            grad_buf = torch.zeros((B, layer.out_dim + grad_pad), dtype=torch.float32, device="cuda")
            grad_buf[:, :layer.out_dim] = torch.from_numpy(pr["grad"]).cuda()
            W_before = [bits_of(w).copy() for w in layer.W]
            layer.forward(ids, offsets, B, out=out_buf)
            layer.backward_update(grad_buf, lr, eps)
            torch.cuda.synchronize()
            assert layer.error_word() == 0
            ref_out, ctx = orc.forward(pl, W, B, pr["ids"], pr["offsets"])
            orc.backward_update(pl, W, A, ctx, B, pr["grad"], lr, eps)
            got = out_buf.cpu().numpy()
            ok, nbad = pooled_close(got[:, :layer.out_dim], ref_out, tables, fields)     # band by the field's table dtype
            assert ok, f"{name} step {s}: {nbad} pooled outputs out of tolerance"
            if out_pad:
                assert (got[:, layer.out_dim:] == 7.0).all()
            for p in range(pl.n_packs):
                c = layer.ctx(p)
                assert c["nnz_p"] == len(ctx[p].key) and c["n_unique"] == len(ctx[p].unique)
                assert np.array_equal(c["keys"].astype(np.uint64), ctx[p].key), f"{name}: keys pack {p}"
                assert np.array_equal(c["packed_offsets"], ctx[p].packed_offsets), f"{name}: packed offsets pack {p}"
                assert np.array_equal(c["unique"].astype(np.uint64), ctx[p].unique), f"{name}: unique pack {p}"
                assert np.array_equal(c["inverse"], ctx[p].inverse), f"{name}: inverse pack {p}"
                so, _ = orc.segments(ctx[p].inverse, len(ctx[p].unique))
                assert np.array_equal(c["seg_offsets"], so), f"{name}: segment offsets pack {p}"
                dt = int(pl.pack_dtype[p])
                gw, ga = bits_of(layer.W[p]), layer.A[p].cpu().numpy()
                ok, nbad = close(f32_of(gw, dt), f32_of(W[p], dt), bf16=dt == 1)
                assert ok, f"{name} step {s}: {nbad} table elements out of tolerance (pack {p})"
                ok, nbad = close(ga, A[p])
                assert ok, f"{name} step {s}: {nbad} accumulator elements out of tolerance (pack {p})"
                untouched = np.ones(gw.shape[0], bool)
                untouched[ctx[p].unique.astype(np.int64)] = False
                assert np.array_equal(gw[untouched], W_before[p][untouched]), f"{name}: untouched rows changed"
    finally:
        layer.close()


# --------------------------------------------------------------------------- small, dense tables
@pytest.mark.parametrize("seed", [1, 2])
def test_small_mixed_packs_shared_tables_two_steps(seed):
    steps = [small_problem(seed * 10 + s, B=37, max_len=6) for s in range(2)]
    run_dense_case("mixed", steps[0]["tables"], steps[0]["fields"], steps)


def test_eq1_shard_split_packs_two_steps():
    # the pack above the average volume split into shards (Sec. III-B, Eq. 1): 1 + 1 + 4 packs instead of 3
    rng = np.random.default_rng(77)
    dims = [8] * 4 + [32] * 8 + [16] * 4
    tables = [(int(rng.integers(20, 200)), d, 0) for d in dims]
    fields = [(t, t % 2) for t in range(len(tables))] + [(5, 0), (2, 1)]
    steps = [small_problem(80 + s, B=33, tables=tables, fields=fields, max_len=6) for s in range(2)]
    run_dense_case("shards", tables, fields, steps, max_shards=4)
    vol = [float(v) for v in rng.integers(1, 30, len(fields))]
    run_dense_case("shards+stats", tables, fields, steps, max_shards=3, field_volume=vol)


@pytest.mark.parametrize("groups", [1, 2, 3])
def test_interleaving_groups_do_not_change_results(groups):
    # Sec. III-C K-Interleaving: packs dealt to groups that run side by side on internal streams
    tables = [(60, 4, 0), (80, 8, 0), (50, 16, 0), (40, 32, 0), (30, 4, 0), (70, 8, 0)]
    fields = [(t, t % 2) for t in range(6)] + [(1, 0), (3, 1)]
    steps = [small_problem(90 + s, B=29, tables=tables, fields=fields, max_len=7) for s in range(2)]
    run_dense_case(f"groups={groups}", tables, fields, steps, interleave_groups=groups)


def test_many_packs_and_a_table_nobody_reads():
    # 20 distinct dimensions -> 20 packs (more than share one pooling launch); table 3 has no field, so
    # its pack has rows but no occurrences, and its rows must stay untouched
    dims = [1, 2, 3, 4, 5, 6, 7, 8, 12, 16, 20, 24, 32, 40, 48, 64, 96, 128, 200, 256]
    tables = [(17 + 3 * i, d, 0) for i, d in enumerate(dims)]
    fields = [(t, t % 2) for t in range(len(tables)) if t != 3] + [(0, 1), (19, 0)]
    steps = [small_problem(120 + s, B=11, tables=tables, fields=fields, max_len=4) for s in range(2)]
    run_dense_case("20 packs", tables, fields, steps)


@pytest.mark.parametrize("seed", list(range(300, 312)))
def test_random_small_layers(seed):
    # seeded random layers: table sizes from one row up, dimensions of every lane shape, both dtypes,
    # fields sharing tables, both poolings, empty bags, now and then raw 64-bit IDs
    rng = np.random.default_rng(seed)
    dims_pool = [1, 2, 3, 4, 5, 8, 12, 16, 17, 32, 48, 64, 100, 128, 256]
    n_tables = int(rng.integers(1, 7))
    dims = rng.choice(dims_pool, size=int(rng.integers(1, 4)), replace=False)
    tables = [(int(rng.choice([1, 2, 3, 17, 64, 200, 1000])), int(rng.choice(dims)), int(rng.integers(0, 2)))
              for _ in range(n_tables)]
    fields = [(int(rng.integers(0, n_tables)), int(rng.integers(0, 2))) for _ in range(int(rng.integers(1, 9)))]
    B = int(rng.choice([1, 2, 7, 31, 64, 129]))
    steps = [small_problem(seed * 7 + s, B=B, tables=tables, fields=fields, max_len=int(rng.integers(1, 9)),
                           wild_ids=bool(rng.integers(0, 4) == 0)) for s in range(2)]
    run_dense_case(f"random {seed}", tables, fields, steps, lr=0.01)


@pytest.mark.parametrize("seed,B", [(400, 1500), (401, 4096), (402, 2500), (403, 3333)])
def test_random_medium_layers_hot_keys_and_many_distinct_keys(seed, B):
    # tiny tables make keys with thousands of occurrences (long keys across several backward tiles),
    # large ones make more than 16384 distinct keys in a table (several work items in the sort, chained
    # by look-back); bags of 0..12 IDs
    rng = np.random.default_rng(seed)
    tables = [(5, 8, 0), (300, 64, 0), (40000, 8, 0), (3, 64, int(rng.integers(0, 2))), (50000, 32, 0), (40, 32, 0)]
    fields = [(0, 0), (1, 1), (2, 0), (3, 1), (4, 0), (5, 1), (2, 1), (4, 1), (0, 1)]
    steps = [small_problem(seed * 11 + s, B=B, tables=tables, fields=fields, max_len=12) for s in range(2)]
    run_dense_case(f"medium {seed}", tables, fields, steps, lr=0.01)


@pytest.mark.parametrize("case", ["mixed", "medium", "bf16", "wild", "dims", "empty", "20 packs"])
def test_partitioned_dedup_on_small_inputs(case):
    # debug bit 1: the dedup of large batches (occurrences partitioned by slice, one block per slice, inverse
    # looked up afterwards) on inputs that the one-launch forward pass would otherwise take
    rng = np.random.default_rng(5)
    if case == "mixed":
        steps = [small_problem(610 + s, B=37, max_len=6) for s in range(2)]
        tables, fields = steps[0]["tables"], steps[0]["fields"]
    elif case == "medium":
        tables = [(5, 8, 0), (300, 64, 0), (400000, 8, 0), (3, 64, 1), (50000, 32, 0), (40, 32, 0)]
        fields = [(0, 0), (1, 1), (2, 0), (3, 1), (4, 0), (5, 1), (2, 1), (4, 1), (0, 1)]
        steps = [small_problem(620 + s, B=4096, tables=tables, fields=fields, max_len=12) for s in range(2)]
    elif case == "bf16":
        tables = [(300, 64, 1), (200, 64, 1), (150, 8, 1)]
        fields = [(0, 0), (1, 1), (0, 0), (2, 0)]
        steps = [small_problem(630 + s, B=40, tables=tables, fields=fields, max_len=9) for s in range(2)]
    elif case == "wild":
        steps = [small_problem(640 + s, B=33, wild_ids=True) for s in range(2)]
        tables, fields = steps[0]["tables"], steps[0]["fields"]
    elif case == "dims":
        tables = [(97, d, 0) for d in (3, 100, 200)] + [(50, 100, 1)]
        fields = [(t, t % 2) for t in range(len(tables))] + [(0, 0)]
        steps = [small_problem(650 + s, B=19, tables=tables, fields=fields, max_len=4) for s in range(2)]
    elif case == "empty":
        tables, fields = [(11, 8, 0), (13, 16, 0)], [(0, 0), (1, 1)]
        steps = [small_problem(660, B=5, tables=tables, fields=fields, max_len=0)]
    else:
        dims = [1, 2, 3, 4, 5, 6, 7, 8, 12, 16, 20, 24, 32, 40, 48, 64, 96, 128, 200, 256]
        tables = [(17 + 3 * i, d, 0) for i, d in enumerate(dims)]
        fields = [(t, t % 2) for t in range(len(tables)) if t != 3] + [(0, 1), (19, 0)]
        steps = [small_problem(670 + s, B=11, tables=tables, fields=fields, max_len=4) for s in range(2)]
    run_dense_case(f"partitioned {case}", tables, fields, steps, lr=0.01, debug=2)


def test_wild_64bit_ids_are_folded():
    steps = [small_problem(50 + s, B=33, wild_ids=True) for s in range(2)]
    steps[0]["ids"][:4] = [-1, -2 ** 63, 2 ** 63 - 1, 0]
    run_dense_case("wild ids", steps[0]["tables"], steps[0]["fields"], steps)


def test_bf16_tables():
    tables = [(300, 64, 1), (200, 64, 1), (150, 8, 1)]
    fields = [(0, 0), (1, 1), (0, 0), (2, 0)]
    steps = [small_problem(60 + s, B=40, tables=tables, fields=fields, max_len=9) for s in range(2)]
    run_dense_case("bf16", tables, fields, steps, lr=0.01)


@pytest.mark.parametrize("dims", [(4, 12, 20), (3, 100, 200), (1, 128, 256), (5, 24, 48)])
def test_unusual_dimensions(dims):
    tables = [(97, d, 0) for d in dims] + [(50, dims[1], 1)]
    fields = [(t, t % 2) for t in range(len(tables))] + [(0, 0)]
    steps = [small_problem(70 + s, B=19, tables=tables, fields=fields, max_len=4) for s in range(2)]
    run_dense_case(f"dims {dims}", tables, fields, steps, lr=0.01)


def test_padded_output_and_gradient_strides():
    steps = [small_problem(80 + s, B=21) for s in range(2)]
    run_dense_case("strides", steps[0]["tables"], steps[0]["fields"], steps, out_pad=5, grad_pad=3)


def test_empty_batch_and_single_sample():
    tables = [(11, 8, 0), (13, 16, 0)]
    fields = [(0, 0), (1, 1)]
    pr = small_problem(90, B=1, tables=tables, fields=fields, max_len=3, allow_empty=False)
    run_dense_case("B=1", tables, fields, [pr])
    pr0 = small_problem(91, B=5, tables=tables, fields=fields, max_len=0)
    assert pr0["ids"].shape[0] == 0
    run_dense_case("nnz=0", tables, fields, [pr0])


def test_hot_key_with_integer_gradients_is_exact():
    """One row hit thousands of times (block-per-key pass): with integer-valued
    gradients the reduced gradient is exact, so A' = g^2 must match to the bit."""
    from paper_2204_04903_amd.layer import PackedEmbedding
    tables = [(1000, 32, 0)]
    fields = [(0, 0), (0, 0)]
    B = 2048
    rng = np.random.default_rng(7)
    lens = rng.integers(1, 4, size=2 * B)
    offsets = np.zeros(2 * B + 1, np.int32); offsets[1:] = np.cumsum(lens)
    ids = rng.integers(0, 1000, size=int(offsets[-1])).astype(np.int64)
    ids[rng.random(ids.shape[0]) < 0.7] = 123                       # the hot row
    ids[rng.random(ids.shape[0]) < 0.05] = 77                       # a warm row
    grad = rng.integers(-3, 4, size=(B, 64)).astype(np.float32)
    Wt = [rng.integers(-8, 9, size=(1000, 32)).astype(np.float32)]
    pr = dict(tables=tables, fields=fields, B=B, ids=ids, offsets=offsets, Wt=Wt, grad=grad)
    run_dense_case("hot key", tables, fields, [pr], lr=0.01)
    layer = PackedEmbedding(tables, fields)
    try:
        layer.load_table(0, Wt[0])
        out = layer.forward(torch.from_numpy(ids).cuda(), torch.from_numpy(offsets).cuda(), B)
        layer.backward_update(torch.from_numpy(grad).cuda(), 0.01, 1e-8)
        pl = orc.plan(tables, fields)
        ref_out, ctx = orc.forward(pl, [Wt[0].copy()], B, ids, offsets)
        assert np.array_equal(out.cpu().numpy(), ref_out)            # integer-valued rows: exact sums
        G = orc.scatter_add(pl, 0, B, grad, ctx[0].inverse, ctx[0].packed_offsets, len(ctx[0].unique))
        a = layer.A[0].cpu().numpy()[ctx[0].unique.astype(np.int64)]
        assert np.array_equal(a, (G * G).astype(np.float32))
    finally:
        layer.close()


@pytest.mark.parametrize("debug", [0, 2])                   # the one-launch forward pass, and the large-batch kernels
@pytest.mark.parametrize("kind", ["field boundary", "decreasing inside a field", "past the field's end"])
@pytest.mark.parametrize("tables,fields", [
    ([(11, 8, 0)], [(0, 0), (0, 0)]),                      # one pack
    ([(11, 8, 0), (7, 16, 0)], [(0, 0), (1, 1)]),          # two packs
])
def test_bad_offsets_raise_the_error_word_and_terminate(tables, fields, kind, debug):
    from paper_2204_04903_amd.layer import PackedEmbedding
    pr = small_problem(95, B=8, tables=tables, fields=fields, max_len=3, allow_empty=False)
    layer = PackedEmbedding(tables, fields, debug=debug)
    try:
        for t in range(len(tables)):
            layer.load_table(t, pr["Wt"][t])
        bad = pr["offsets"].copy()
        if kind == "field boundary":
            bad[8] = bad[16] + 3      # the boundary between the two fields runs past the end
        elif kind == "decreasing inside a field":
            bad[3] = bad[5] + 1       # bag 3 of field 0 would begin after bag 4 does
        else:
            bad[5] = bad[8] + 2       # bag 5 of field 0 would begin among the second field's IDs
        out = layer.forward(torch.from_numpy(pr["ids"]).cuda(), torch.from_numpy(bad).cuda(), 8)
        torch.cuda.synchronize()
        assert layer.error_word() & 1
        assert np.isfinite(out.cpu().numpy()).all()       # undefined values, but every read stayed inside the inputs
        # A backward pass after a rejected forward pass leaves the tables and accumulators of the packs whose
        # offsets were rejected alone: every pack for a wrong field boundary, the pack of field 0 for a
        # wrong offset inside that field (the other pack's offsets passed: it is updated).
        say("[bad offsets] backward after the rejected forward")
        layer.backward_update(torch.from_numpy(pr["grad"]).cuda(), 0.05, 1e-8)
        torch.cuda.synchronize()
        W0 = stack_tables(orc.plan(tables, fields), [w.copy() for w in pr["Wt"]])
        rejected = range(layer.n_packs) if kind == "field boundary" else [layer.table_slot[fields[0][0]][0]]
        for p in rejected:
            assert np.array_equal(bits_of(layer.W[p]), W0[p])
            assert (layer.A[p] == 0).all()
        for p in range(layer.n_packs):
            assert torch.isfinite(layer.A[p]).all()
        for t in range(len(tables)):                       # start the check below from the same tables again
            layer.load_table(t, pr["Wt"][t])
        for p in range(layer.n_packs):
            layer.A[p].zero_()
        # and the same workspace works again afterwards
        out = layer.forward(torch.from_numpy(pr["ids"]).cuda(), torch.from_numpy(pr["offsets"]).cuda(), 8)
        torch.cuda.synchronize()
        assert layer.error_word() == 0
        pl = orc.plan(tables, fields)
        ref, _ = orc.forward(pl, stack_tables(pl, [w.copy() for w in pr["Wt"]]), 8, pr["ids"], pr["offsets"])
        assert close(out.cpu().numpy(), ref)[0]
    finally:
        layer.close()


# --------------------------------------------------------------------------- the five configurations
def run_config(idx, steps=2, plan_opts=None, **shrink):
    """Lazily materialised tables: device fill by the generator's kernel, the
    oracle on the generator's host values for the distinct rows only."""
    from paper_2204_04903_amd.layer import PackedEmbedding
    wl = synth.config(idx, **shrink)
    say(f"[config {idx}] {wl.description}; B={wl.batch} fields={wl.n_fields} shrink={shrink}")
    so = SparseOracle(orc, synth, wl)
    pl = so.pl
    layer = PackedEmbedding(so.tables, so.fields, **(plan_opts or {}))
    try:
        stream = torch.cuda.current_stream().cuda_stream
        for t, ts in enumerate(wl.tables):
            synth.fill_device(layer.table_view(t).data_ptr(), ts.rows, ts.dim, ts.dtype, wl.seed, t, stream)
        torch.cuda.synchronize()
        # the device fill writes what the host generator says
        t_probe = len(wl.tables) - 1
        probe = np.array([0, 1, wl.tables[t_probe].rows // 2, wl.tables[t_probe].rows - 1], np.int64)
        got = bits_of(layer.table_view(t_probe)[torch.from_numpy(probe).cuda()])
        assert np.array_equal(got, synth.table_rows(wl, t_probe, rows=probe))
        batches = synth.make_batches(wl, steps)
        bf16 = wl.tables[0].dtype == 1
        for s, batch in enumerate(batches):
            say(f"[config {idx}] step {s}: nnz={batch.nnz}")
            ids = torch.from_numpy(batch.ids).cuda()
            offsets = torch.from_numpy(batch.offsets).cuda()
            grad = torch.from_numpy(batch.grad_out).cuda()
            out = layer.forward(ids, offsets, wl.batch)
            layer.backward_update(grad, wl.lr, wl.eps)
            torch.cuda.synchronize()
            assert layer.error_word() == 0
            ref_out, res = so.step(batch, wl.lr, wl.eps)
            ok, nbad = close(out.cpu().numpy(), ref_out, bf16=bf16)
            assert ok, f"config {idx} step {s}: {nbad} pooled outputs out of tolerance"
            for p in range(pl.n_packs):
                c, r = layer.ctx(p), res[p]
                assert c["nnz_p"] == len(r["keys"]) and c["n_unique"] == len(r["unique"])
                for name in ("keys", "unique"):
                    assert np.array_equal(c[name].astype(np.uint64), r[name]), f"config {idx}: {name} pack {p}"
                for name in ("packed_offsets", "inverse", "seg_offsets"):
                    assert np.array_equal(c[name], r[name]), f"config {idx}: {name} pack {p}"
                dt = int(pl.pack_dtype[p])
                rows = torch.from_numpy(r["unique"].astype(np.int64)).cuda()
                gw = bits_of(layer.W[p][rows]); ga = layer.A[p][rows].cpu().numpy()
                ok, nbad = close(f32_of(gw, dt), f32_of(r["W"], dt), bf16=dt == 1)
                assert ok, f"config {idx} step {s}: {nbad} updated elements out of tolerance (pack {p})"
                ok, nbad = close(ga, r["A"])
                assert ok, f"config {idx} step {s}: {nbad} accumulator elements out of tolerance (pack {p})"
                # rows never touched so far still hold the generator's bits
                R = int(pl.pack_rows[p])
                rng = np.random.default_rng(idx * 100 + p)
                cand = rng.integers(0, R, size=4096).astype(np.uint64)
                cand = np.setdiff1d(cand, so.keys_seen[p])
                gw = bits_of(layer.W[p][torch.from_numpy(cand.astype(np.int64)).cuda()])
                assert np.array_equal(gw, so.init_rows(p, cand)), f"config {idx}: untouched rows changed (pack {p})"
                assert (layer.A[p][torch.from_numpy(cand.astype(np.int64)).cuda()] == 0).all()
    finally:
        layer.close()


def test_config1_full_size():
    run_config(1)


def test_config3_shrunk_spans_tiles_and_ragged_tails():
    run_config(3, batch=333, row_scale=0.02, n_fields=40)


def test_config4_shrunk_interleaved_packs_and_hashed_ids():
    run_config(4, batch=257, row_scale=0.1, n_fields=101)


def test_config5_shrunk_long_sequences_bf16():
    run_config(5, batch=64, row_scale=0.05, n_fields=12)


@pytest.mark.timeout(600)
def test_tables_above_the_fine_slice_limit():
    """Two tables of 140 M rows: the large-batch dedup then cuts slices of 2^17 keys (the wide slice kernels)."""
    free, _ = torch.cuda.mem_get_info()
    if free < 90 * 2**30:
        pytest.skip("needs 90 GiB of free device memory")
    run_config(2, n_fields=2, row_scale=140.0, plan_opts=dict(debug=2))


def test_config2_full_size():
    run_config(2)


@pytest.mark.timeout(900)
def test_config3_full_size():
    # 200 fields, four packs, ~21 M occurrences, ~103 GB of tables and accumulators
    free, _ = torch.cuda.mem_get_info()
    if free < 130 * 2**30:
        pytest.skip("needs about 110 GB of free device memory")
    run_config(3)


@pytest.mark.timeout(900)
def test_config4_full_size():
    # 1000 fields, two packs, ~11 M occurrences of raw 64-bit IDs, ~21 GB of tables and accumulators
    free, _ = torch.cuda.mem_get_info()
    if free < 40 * 2**30:
        pytest.skip("needs about 25 GB of free device memory")
    run_config(4)


@pytest.mark.timeout(900)
def test_config5_full_size():
    # 60 fields of bf16 tables, sequences of 100-1000 IDs, ~5.7 M occurrences, ~46 GB of tables and accumulators
    free, _ = torch.cuda.mem_get_info()
    if free < 70 * 2**30:
        pytest.skip("needs about 50 GB of free device memory")
    run_config(5)
