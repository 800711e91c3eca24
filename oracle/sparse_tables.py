"""The oracle's steps driven over tables that are too large to hold on the host.

TEST INFRASTRUCTURE ONLY (tests, smoke check, the benchmark's CPU-baseline leg).
No arithmetic of the method lives here: every step is a call into pk_oracle.
"""
import numpy as np


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

    def step(self, batch, lr, eps, rows=None, B=None):
        """One forward + backward + update.  Returns (out, per-pack dict with the
        integer context and the updated rows).  `rows[p]`, when given, is the
        (W, A) pair current_rows would return for pack p (lets a caller keep the
        input generator out of a timed region).  `B`: samples in `batch` when it
        is not a whole batch of the workload (a micro-batch)."""
        orc, pl = self.orc, self.pl
        B = self.wl.batch if B is None else B
        out = np.zeros((B, pl.out_dim), np.float32)
        res = []
        for p in range(pl.n_packs):
            dt = int(pl.pack_dtype[p])
            key, po = orc.pack_keys(pl, p, B, batch.ids, batch.offsets)
            uq, inv = orc.unique(key)
            Wrow, Arow = rows[p] if rows is not None else self.current_rows(p, uq)
            E = orc.widen_rows(Wrow, dt)
            orc.pool(pl, p, B, E, inv, po, out)
            G = orc.scatter_add(pl, p, B, batch.grad_out, inv, po, len(uq))
            Wnew, Anew = orc.adagrad_rows(E, Arow, G, lr, eps, dt)
            self.remember(p, uq, Wnew, Anew)
            so, _ = orc.segments(inv, len(uq))
            res.append(dict(keys=key, packed_offsets=po, unique=uq, inverse=inv, seg_offsets=so, W=Wnew, A=Anew))
        return out, res
