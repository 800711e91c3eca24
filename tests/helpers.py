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


# ---------------------------------------------------------------------------
# the oracle's steps on lazily materialised tables (full-size configurations)
# ---------------------------------------------------------------------------
class SparseOracle:
    """Runs the oracle's step functions on tables that exist only as the input
    generator's value function: the rows of the distinct keys are materialised
    on demand (that IS the Gather step's result, by the definition of the
    synthetic table), and rows already updated are remembered per pack."""

    def __init__(self, orc, synth, wl):
        self.orc, self.synth, self.wl = orc, synth, wl
        self.tables = [(t.rows, t.dim, t.dtype) for t in wl.tables]
        self.fields = [(f.table, f.pool) for f in wl.fields]
        self.pl = orc.plan(self.tables, self.fields)
        P = self.pl.n_packs
        self.keys_seen = [np.zeros(0, np.uint64) for _ in range(P)]
        self.W_seen = [None] * P
        self.A_seen = [None] * P

    def init_rows(self, p, uq):
        """Initial values of pack rows `uq` (float32, or bf16 bit patterns)."""
        pl = self.pl
        D = int(pl.pack_dim[p])
        out = np.zeros((len(uq), D), np.float32 if pl.pack_dtype[p] == 0 else np.uint16)
        ts = [t for t in range(len(self.tables)) if pl.table_pack[t] == p]
        bases = np.array([pl.table_base[t] for t in ts], np.int64)
        which = np.searchsorted(bases, uq.astype(np.int64), side="right") - 1
        for n, t in enumerate(ts):
            sel = np.nonzero(which == n)[0]
            if len(sel):
                out[sel] = self.synth.table_rows(self.wl, t, rows=uq[sel].astype(np.int64) - bases[n])
        return out

    def current_rows(self, p, uq):
        W = self.init_rows(p, uq)
        A = np.zeros(W.shape, np.float32)
        seen = self.keys_seen[p]
        if len(seen):
            pos = np.searchsorted(seen, uq)
            pos_c = np.minimum(pos, len(seen) - 1)
            hit = seen[pos_c] == uq
            W[hit] = self.W_seen[p][pos_c[hit]]
            A[hit] = self.A_seen[p][pos_c[hit]]
        return W, A

    def remember(self, p, uq, Wnew, Anew):
        seen = self.keys_seen[p]
        if len(seen) == 0:
            self.keys_seen[p], self.W_seen[p], self.A_seen[p] = uq.copy(), Wnew.copy(), Anew.copy()
            return
        allk = np.union1d(seen, uq)
        W = np.zeros((len(allk), Wnew.shape[1]), Wnew.dtype)
        A = np.zeros((len(allk), Wnew.shape[1]), np.float32)
        i_old = np.searchsorted(allk, seen)
        W[i_old], A[i_old] = self.W_seen[p], self.A_seen[p]
        i_new = np.searchsorted(allk, uq)
        W[i_new], A[i_new] = Wnew, Anew
        self.keys_seen[p], self.W_seen[p], self.A_seen[p] = allk, W, A

    def step(self, batch, lr, eps):
        """One forward + backward + update.  Returns (out, per-pack dict with the
        integer context and the updated rows)."""
        orc, pl, B = self.orc, self.pl, self.wl.batch
        out = np.zeros((B, pl.out_dim), np.float32)
        res = []
        for p in range(pl.n_packs):
            dt = int(pl.pack_dtype[p])
            key, po = orc.pack_keys(pl, p, B, batch.ids, batch.offsets)
            uq, inv = orc.unique(key)
            Wrow, Arow = self.current_rows(p, uq)
            E = orc.widen_rows(Wrow, dt)
            orc.pool(pl, p, B, E, inv, po, out)
            G = orc.scatter_add(pl, p, B, batch.grad_out, inv, po, len(uq))
            Wnew, Anew = orc.adagrad_rows(E, Arow, G, lr, eps, dt)
            self.remember(p, uq, Wnew, Anew)
            so, _ = orc.segments(inv, len(uq))
            res.append(dict(keys=key, packed_offsets=po, unique=uq, inverse=inv, seg_offsets=so, W=Wnew, A=Anew))
        return out, res
