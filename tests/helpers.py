"""Small random problems for the oracle pins and the parity tests (inputs only)."""
import numpy as np


def small_problem(seed, B=7, tables=None, fields=None, max_len=5, allow_empty=True, wild_ids=False,
                  int_valued=False):
    """tables: list of (rows, dim, dtype); fields: list of (table, pool).
    Returns dict with ids, offsets (field-major bags), per-table dense arrays, grad_out."""
    rng = np.random.default_rng(seed)
    if tables is None:
        tables = [(13, 4, 0), (7, 8, 0), (29, 4, 0), (5, 8, 0)]
    if fields is None:
        fields = [(0, 0), (1, 1), (2, 1), (0, 0), (3, 0), (2, 0)]   # table 0 and 2 shared
    F = len(fields)
    lo = 0 if allow_empty else 1
    lens = rng.integers(lo, max_len + 1, size=(F, B))
    offsets = np.zeros(F * B + 1, np.int32)
    offsets[1:] = np.cumsum(lens.reshape(-1))
    nnz = int(offsets[-1])
    ids = np.zeros(nnz, np.int64)
    for f, (t, _) in enumerate(fields):
        a, b = offsets[f * B], offsets[(f + 1) * B]
        if wild_ids:
            ids[a:b] = rng.integers(-2**63, 2**63 - 1, size=b - a, dtype=np.int64)
        else:
            ids[a:b] = rng.integers(0, tables[t][0], size=b - a)
    Wt = []
    for (rows, dim, dt) in tables:
        if int_valued:
            w = rng.integers(-8, 9, size=(rows, dim)).astype(np.float32)
        else:
            w = (rng.standard_normal((rows, dim)) * 0.1).astype(np.float32)
        if dt == 1:
            w = (w.view(np.uint32) >> np.uint32(16)).astype(np.uint16)   # truncate: exactly bf16
        Wt.append(np.ascontiguousarray(w))
    D_out = sum(tables[t][1] for t, _ in fields)
    if int_valued:
        grad = rng.integers(-4, 5, size=(B, D_out)).astype(np.float32)
    else:
        grad = rng.standard_normal((B, D_out)).astype(np.float32)
    return dict(tables=tables, fields=fields, B=B, ids=ids, offsets=offsets, Wt=Wt, grad=grad, D_out=D_out)


def stack_tables(pl, Wt):
    """Per-table arrays -> per-pack stacked arrays, in the plan's table order."""
    out = []
    for p in range(pl.n_packs):
        ts = [t for t in range(len(Wt)) if pl.table_pack[t] == p]
        assert all(pl.table_base[ts[i]] < pl.table_base[ts[i + 1]] for i in range(len(ts) - 1))
        out.append(np.ascontiguousarray(np.concatenate([Wt[t] for t in ts], axis=0)))
    return out


def pooled_rel_band(tables, fields):
    """Relative tolerance of every pooled output column: 2e-2 where the field's table is bf16
    (fp32 accumulation), 1e-5 where it is fp32.  Fields are concatenated in field order."""
    cols = []
    for t, _ in fields:
        cols.append(np.full(tables[t][1], 2e-2 if tables[t][2] == 1 else 1e-5))
    return np.concatenate(cols)


def pooled_close(got, ref, tables, fields):
    """|got - ref| <= 1e-6 + rel * |ref| with rel chosen per column by the dtype of the field's table."""
    tol = 1e-6 + pooled_rel_band(tables, fields)[None, :] * np.abs(ref)
    bad = np.abs(got.astype(np.float64) - ref.astype(np.float64)) > tol
    return not bad.any(), int(bad.sum())
