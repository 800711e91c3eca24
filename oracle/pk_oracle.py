"""ctypes front end of the CPU oracle (pk_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests, the smoke check and the
benchmark's CPU-baseline leg, never by the product path.  All arithmetic of the
method lives in pk_oracle.c; this file marshals numpy arrays and strings the
steps together in the order the paper lists them (Sec. II-D: Unique, Gather,
SegmentReduction, then the mirrored backward pass; Sec. III-B: one packed
operation per group of same-dimension fields).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_lib = None

F32, BF16 = 0, 1
SUM, MEAN = 0, 1


def build(force: bool = False) -> str:
    so = os.path.join(_HERE, "libpk_oracle.so")
    src = os.path.join(_HERE, "pk_oracle.c")
    if force or not os.path.exists(so) or os.path.getmtime(so) < os.path.getmtime(src):
        subprocess.check_call(["gcc", "-O2", "-fPIC", "-shared", "-ffp-contract=off", "-o", so, src, "-lm"])
    return so


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.orc_plan.restype = ctypes.c_int32
        _lib.orc_pack_keys.restype = ctypes.c_int64
        _lib.orc_unique.restype = ctypes.c_int32
        _lib.orc_calc_vparam.restype = ctypes.c_double
        _lib.orc_shard_split.restype = ctypes.c_int32
        _lib.orc_micro_batch_size.restype = ctypes.c_int32
        _lib.orc_field_slots.restype = None
        _lib.orc_bf16_round.restype = ctypes.c_uint16
        _lib.orc_bf16_round.argtypes = [ctypes.c_float]
        _lib.orc_bf16_widen.restype = ctypes.c_float
        _lib.orc_bf16_widen.argtypes = [ctypes.c_uint16]
        _lib.orc_partition.restype = None
        for name in ("orc_segments", "orc_gather", "orc_pool", "orc_scatter_add", "orc_adagrad_rows",
                     "orc_direct_field_forward", "orc_direct_field_grad", "orc_direct_table_adagrad"):
            getattr(_lib, name).restype = None
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else ctypes.c_void_p(a.ctypes.data)


def _c(a, dtype) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=dtype))


i32, i64, f64 = ctypes.c_int32, ctypes.c_int64, ctypes.c_double


@dataclass
class Plan:
    rows: np.ndarray          # int64 [n_tables]
    dim: np.ndarray           # int32 [n_tables]
    dtype: np.ndarray         # int32 [n_tables]
    field_table: np.ndarray   # int32 [n_fields]
    pool: np.ndarray          # int32 [n_fields]
    n_packs: int
    table_pack: np.ndarray
    table_base: np.ndarray
    pack_dim: np.ndarray
    pack_dtype: np.ndarray
    pack_rows: np.ndarray
    field_pack: np.ndarray
    field_slot: np.ndarray
    field_col: np.ndarray
    pack_fields: List[np.ndarray]   # per pack: field indices in slot order
    shards: Optional[np.ndarray] = None   # Eq. 1 split: shards per unsplit pack (None = no split asked for)

    @property
    def out_dim(self) -> int:
        return int(self.dim[self.field_table].sum())


def plan(tables: Sequence[Tuple[int, int, int]], fields: Sequence[Tuple[int, int]],
         max_shards: int = 0, field_volume: Optional[Sequence[float]] = None) -> Plan:
    """tables: (rows, dim, dtype) each; fields: (table, pool) each.  max_shards > 1 applies the Eq. 1 shard
    split; field_volume = occurrences per field from warm-up statistics (uniform when None)."""
    rows = _c([t[0] for t in tables], np.int64)
    dim = _c([t[1] for t in tables], np.int32)
    dtype = _c([t[2] for t in tables], np.int32)
    ft = _c([f[0] for f in fields], np.int32)
    pool = _c([f[1] for f in fields], np.int32)
    nt, nf = len(tables), len(fields)
    table_pack = np.zeros(nt, np.int32); table_base = np.zeros(nt, np.int64)
    pack_dim = np.zeros(nt, np.int32); pack_dtype = np.zeros(nt, np.int32); pack_rows = np.zeros(nt, np.int64)
    field_pack = np.zeros(nf, np.int32); field_slot = np.zeros(nf, np.int32); field_col = np.zeros(nf, np.int64)
    n_packs = lib().orc_plan(i32(nt), _p(rows), _p(dim), _p(dtype), i32(nf), _p(ft),
                             _p(table_pack), _p(table_base), _p(pack_dim), _p(pack_dtype), _p(pack_rows),
                             _p(field_pack), _p(field_slot), _p(field_col))
    shards = None
    if max_shards > 1:
        vol = np.ones(nf, np.float64) if field_volume is None else _c(field_volume, np.float64)
        occ = np.zeros(nt, np.float64)
        for f in range(nf):
            occ[ft[f]] += vol[f]
        base_pack = table_pack.copy()
        shards = np.zeros(n_packs, np.int32)
        n_packs = lib().orc_shard_split(i32(nt), _p(rows), _p(dim), _p(dtype), i32(n_packs), _p(base_pack), _p(occ),
                                        i32(max_shards), _p(shards), _p(table_pack), _p(table_base),
                                        _p(pack_dim), _p(pack_dtype), _p(pack_rows))
        lib().orc_field_slots(i32(nf), _p(ft), _p(table_pack), _p(dim), _p(field_pack), _p(field_slot), _p(field_col))
    pack_fields = []
    for p in range(n_packs):
        fs = np.nonzero(field_pack == p)[0].astype(np.int32)
        assert (field_slot[fs] == np.arange(len(fs))).all()
        pack_fields.append(np.ascontiguousarray(fs))
    pl = Plan(rows, dim, dtype, ft, pool, n_packs, table_pack, table_base, pack_dim[:n_packs].copy(),
              pack_dtype[:n_packs].copy(), pack_rows[:n_packs].copy(), field_pack, field_slot, field_col,
              pack_fields)
    pl.shards = shards
    return pl


def calc_vparam(pl: Plan, occurrences: Sequence[float], pack: int) -> float:
    occ = _c(occurrences, np.float64)
    return float(lib().orc_calc_vparam(i32(len(pl.rows)), _p(pl.table_pack), _p(pl.dim), _p(occ), i32(pack)))


def micro_batch_size(B: int, rbound: Sequence[float], rinstance: Sequence[float]) -> int:
    """Sec. III-C, Eq. 2, then the even cut into micro-batches."""
    rb, ri = _c(rbound, np.float64), _c(rinstance, np.float64)
    return int(lib().orc_micro_batch_size(ctypes.c_int32(B), ctypes.c_int32(len(rb)), _p(rb), _p(ri)))


def pack_keys(pl: Plan, p: int, B: int, ids: np.ndarray, offsets: np.ndarray):
    ids = _c(ids, np.int64); offsets = _c(offsets, np.int32)
    pf = pl.pack_fields[p]
    k = len(pf)
    nnz_p = int(sum(int(offsets[(f + 1) * B]) - int(offsets[f * B]) for f in pf))
    key = np.zeros(nnz_p, np.uint64)
    po = np.zeros(k * B + 1, np.int32)
    n = lib().orc_pack_keys(i32(k), _p(pf), _p(pl.field_table), _p(pl.rows), _p(pl.table_base), i32(B),
                            _p(ids), _p(offsets), _p(key), _p(po))
    assert n == nnz_p
    return key, po


def unique(key: np.ndarray):
    key = _c(key, np.uint64)
    n = key.shape[0]
    uq = np.zeros(n, np.uint64); inv = np.zeros(n, np.int32)
    U = lib().orc_unique(i64(n), _p(key), _p(uq), _p(inv))
    return uq[:U].copy(), inv


def segments(inverse: np.ndarray, U: int):
    inverse = _c(inverse, np.int32)
    so = np.zeros(U + 1, np.int32); sp = np.zeros(inverse.shape[0], np.int32)
    lib().orc_segments(i64(inverse.shape[0]), _p(inverse), i32(U), _p(so), _p(sp))
    return so, sp


def partition(uq: np.ndarray, n_owners: int):
    """Sec. II-D Partition of the distinct keys of a pack: (keys grouped by owner, their indices in `uq`,
    offsets of the owners' groups)."""
    uq = _c(uq, np.uint64)
    U = uq.shape[0]
    keys = np.zeros(U, np.uint64); idx = np.zeros(U, np.int32); off = np.zeros(n_owners + 1, np.int32)
    lib().orc_partition(i32(U), _p(uq), i32(n_owners), _p(keys), _p(idx), _p(off))
    return keys, idx, off


def gather(W: np.ndarray, dtype: int, uq: np.ndarray) -> np.ndarray:
    """W: the pack's stacked table [R, D] (float32, or uint16 bf16 bit patterns)."""
    assert W.flags.c_contiguous and W.dtype == (np.float32 if dtype == F32 else np.uint16)
    D = W.shape[1]
    E = np.zeros((len(uq), D), np.float64)
    lib().orc_gather(_p(W), i32(dtype), i32(D), i32(len(uq)), _p(_c(uq, np.uint64)), _p(E))
    return E


def widen_rows(rows: np.ndarray, dtype: int) -> np.ndarray:
    """Rows already materialised by the input generator -> the double-precision
    array that `gather` would return for them (exact widening)."""
    if dtype == F32:
        return rows.astype(np.float64)
    return (rows.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def pool(pl: Plan, p: int, B: int, E: np.ndarray, inverse: np.ndarray, packed_offsets: np.ndarray,
         out: np.ndarray) -> None:
    assert out.dtype == np.float32 and out.flags.c_contiguous and E.flags.c_contiguous
    pf = pl.pack_fields[p]
    lib().orc_pool(i32(len(pf)), _p(pf), _p(pl.pool), _p(pl.field_col), i32(B), i32(int(pl.pack_dim[p])),
                   _p(E), _p(_c(inverse, np.int32)), _p(_c(packed_offsets, np.int32)), _p(out),
                   i64(out.shape[1]))


def scatter_add(pl: Plan, p: int, B: int, grad_out: np.ndarray, inverse: np.ndarray,
                packed_offsets: np.ndarray, U: int) -> np.ndarray:
    assert grad_out.dtype == np.float32 and grad_out.flags.c_contiguous
    pf = pl.pack_fields[p]
    D = int(pl.pack_dim[p])
    G = np.zeros((U, D), np.float64)
    lib().orc_scatter_add(i32(len(pf)), _p(pf), _p(pl.pool), _p(pl.field_col), i32(B), i32(D), _p(grad_out),
                          i64(grad_out.shape[1]), _p(_c(inverse, np.int32)), _p(_c(packed_offsets, np.int32)),
                          i32(U), _p(G))
    return G


def adagrad_rows(Wrow: np.ndarray, Arow: np.ndarray, G: np.ndarray, lr: float, eps: float, dtype: int):
    U, D = G.shape
    Wrow = _c(Wrow, np.float64); Arow = _c(Arow, np.float32)
    Wnew = np.zeros((U, D), np.float32 if dtype == F32 else np.uint16)
    Anew = np.zeros((U, D), np.float32)
    lib().orc_adagrad_rows(i32(U), i32(D), i32(dtype), _p(Wrow), _p(Arow), _p(_c(G, np.float64)),
                           f64(lr), f64(eps), _p(Wnew), _p(Anew))
    return Wnew, Anew


# ---------------------------------------------------------------------------
# the whole path on dense host tables
# ---------------------------------------------------------------------------
@dataclass
class PackCtx:
    key: np.ndarray
    packed_offsets: np.ndarray
    unique: np.ndarray
    inverse: np.ndarray


def forward(pl: Plan, W: Sequence[np.ndarray], B: int, ids: np.ndarray, offsets: np.ndarray):
    """W[p]: stacked table of pack p.  Returns (out [B, out_dim] float32, per-pack context)."""
    out = np.zeros((B, pl.out_dim), np.float32)
    ctx = []
    for p in range(pl.n_packs):
        key, po = pack_keys(pl, p, B, ids, offsets)
        uq, inv = unique(key)
        E = gather(W[p], int(pl.pack_dtype[p]), uq)
        pool(pl, p, B, E, inv, po, out)
        ctx.append(PackCtx(key, po, uq, inv))
    return out, ctx


def backward_update(pl: Plan, W: Sequence[np.ndarray], A: Sequence[np.ndarray], ctx: Sequence[PackCtx],
                    B: int, grad_out: np.ndarray, lr: float, eps: float) -> None:
    """Updates W[p] and A[p] in place on the rows of the distinct keys only."""
    for p in range(pl.n_packs):
        c = ctx[p]
        dt = int(pl.pack_dtype[p])
        G = scatter_add(pl, p, B, grad_out, c.inverse, c.packed_offsets, len(c.unique))
        r = c.unique.astype(np.int64)
        E = gather(W[p], dt, c.unique)
        Wnew, Anew = adagrad_rows(E, A[p][r], G, lr, eps, dt)
        W[p][r] = Wnew
        A[p][r] = Anew


# ---------------------------------------------------------------------------
# the second route: per field, per table, no packing and no Unique
# ---------------------------------------------------------------------------
def direct_forward(tables, fields, Wt: Sequence[np.ndarray], B: int, ids, offsets) -> np.ndarray:
    ids = _c(ids, np.int64); offsets = _c(offsets, np.int32)
    D_out = sum(tables[t][1] for t, _ in fields)
    out = np.zeros((B, D_out), np.float32)
    col = 0
    for f, (t, pm) in enumerate(fields):
        rows, D, dt = tables[t]
        bo = np.ascontiguousarray(offsets[f * B:(f + 1) * B + 1])
        lib().orc_direct_field_forward(_p(Wt[t]), i32(dt), i64(rows), i32(D), i32(pm), i32(B), _p(ids), _p(bo),
                                       _p(out), i64(D_out), i64(col))
        col += D
    return out


def direct_backward_update(tables, fields, Wt: Sequence[np.ndarray], At: Sequence[np.ndarray], B: int, ids,
                           offsets, grad_out: np.ndarray, lr: float, eps: float) -> None:
    ids = _c(ids, np.int64); offsets = _c(offsets, np.int32)
    dW = [np.zeros((tables[t][0], tables[t][1]), np.float64) for t in range(len(tables))]
    touched = [np.zeros(tables[t][0], np.uint8) for t in range(len(tables))]
    col = 0
    for f, (t, pm) in enumerate(fields):
        rows, D, dt = tables[t]
        bo = np.ascontiguousarray(offsets[f * B:(f + 1) * B + 1])
        lib().orc_direct_field_grad(i64(rows), i32(D), i32(pm), i32(B), _p(ids), _p(bo), _p(grad_out),
                                    i64(grad_out.shape[1]), i64(col), _p(dW[t]), _p(touched[t]))
        col += D
    for t, (rows, D, dt) in enumerate(tables):
        lib().orc_direct_table_adagrad(_p(Wt[t]), _p(At[t]), i32(dt), i64(rows), i32(D), _p(dW[t]),
                                       _p(touched[t]), f64(lr), f64(eps))
