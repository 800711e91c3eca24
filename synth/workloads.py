"""Seeded synthetic workloads for the packed multi-field embedding layer.

Input generation only: nothing here hashes, deduplicates, gathers, pools or
updates.  Both the CPU oracle's tests and the HIP path's tests/bench draw their
inputs from this module so that they see the same bits.

The five configurations mirror the shapes of the recommender workloads the
paper trains on (Sec. IV-A, Tab. "dataset": 26 one-hot fields, ~200 fields of
dims 8-32, ~1000+ small-dim fields, behaviour sequences of 50-100+ IDs) and
the ID skew it reports (Sec. II-B, Fig. 3: a fifth of the IDs covers most of
the occurrences), for which a bounded Zipf law stands in.  None of the paper's
datasets is reproduced.
"""
from __future__ import annotations

import ctypes
import math
import os
import subprocess
from dataclasses import dataclass, field
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
BASE_SEED = 220404903

F32, BF16 = 0, 1
SUM, MEAN = 0, 1

_M64 = (1 << 64) - 1
_GOLD = 0x9E3779B97F4A7C15


def mix64(z: int) -> int:
    """Same 64-bit finaliser as fill.c (python ints)."""
    z &= _M64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _M64
    return z ^ (z >> 31)


def _mix64_np(z: np.ndarray) -> np.ndarray:
    z = z.astype(np.uint64, copy=True)
    z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
    z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
    return z ^ (z >> np.uint64(31))


@dataclass
class TableSpec:
    rows: int
    dim: int
    dtype: int = F32


@dataclass
class FieldSpec:
    table: int
    pool: int = SUM
    len_lo: int = 1          # bag length ~ uniform integer in [len_lo, len_hi]
    len_hi: int = 1


@dataclass
class Workload:
    name: str
    batch: int
    tables: List[TableSpec]
    fields: List[FieldSpec]
    alpha: Optional[float]   # Zipf exponent; None = uniform IDs
    raw_hash_ids: bool = False   # emit full 64-bit hashed IDs (folded by the layer)
    seed: int = BASE_SEED
    lr: float = 0.01
    eps: float = 1e-8
    description: str = ""

    @property
    def n_fields(self) -> int:
        return len(self.fields)

    @property
    def out_dim(self) -> int:
        return sum(self.tables[f.table].dim for f in self.fields)

    def expected_nnz(self) -> float:
        return self.batch * sum((f.len_lo + f.len_hi) / 2 for f in self.fields)


@dataclass
class Batch:
    ids: np.ndarray        # int64 [nnz], field-major bags
    offsets: np.ndarray    # int32 [F*B+1], bag g = f*B + b
    grad_out: np.ndarray   # float32 [B, out_dim]

    @property
    def nnz(self) -> int:
        return int(self.ids.shape[0])


# ---------------------------------------------------------------------------
# the five configurations
# ---------------------------------------------------------------------------
def config(index: int, batch: Optional[int] = None, row_scale: float = 1.0,
           n_fields: Optional[int] = None, len_scale: float = 1.0) -> Workload:
    """Configuration `index` (1..5).  `batch`, `row_scale`, `n_fields` and
    `len_scale` shrink it for parity tests while keeping its structure (dims,
    pooling, skew, length mix, field order)."""
    seed = BASE_SEED + index
    rng = np.random.Generator(np.random.Philox(key=[seed, 0xC0F1]))

    def rows_of(r):
        return max(2, int(r * row_scale))

    def len_of(hi):
        return max(1, int(round(hi * len_scale)))

    if index == 1:
        F = n_fields or 8
        tables = [TableSpec(rows_of(10_000), 16) for _ in range(F)]
        fields = [FieldSpec(t, SUM, 1, 1) for t in range(F)]
        return Workload("cfg1", batch or 512, tables, fields, None, seed=seed,
                        description="8 one-hot fields, 10k x 16 fp32 tables, uniform IDs, sum")
    if index == 2:
        F = n_fields or 26
        tables = [TableSpec(rows_of(1_000_000), 32) for _ in range(F)]
        fields = [FieldSpec(t, SUM, 1, 1) for t in range(F)]
        return Workload("cfg2", batch or 8192, tables, fields, 1.05, seed=seed,
                        description="26 one-hot fields, 1M x 32 fp32 tables, Zipf 1.05, sum, one pack")
    if index == 3:
        F = n_fields or 200
        dims = rng.choice(np.array([8, 16, 32, 64]), size=200)
        rows = np.floor(10.0 ** rng.uniform(5.0, 7.0, size=200)).astype(np.int64)
        tables = [TableSpec(rows_of(int(rows[t])), int(dims[t])) for t in range(F)]
        fields = [FieldSpec(t, MEAN, 1, len_of(50)) for t in range(F)]
        return Workload("cfg3", batch or 4096, tables, fields, 1.2, seed=seed,
                        description="200 multi-hot fields (len 1-50), dims {8,16,32,64}, rows "
                                    "log-uniform 1e5-1e7, Zipf 1.2, mean, packs by dim")
    if index == 4:
        F = n_fields or 1000
        rows = np.floor(10.0 ** rng.uniform(4.0, 6.0, size=1000)).astype(np.int64)
        tables = [TableSpec(rows_of(int(rows[t])), 8 if t % 2 == 0 else 16) for t in range(F)]
        fields = [FieldSpec(t, SUM, 1, len_of(10)) for t in range(F)]
        return Workload("cfg4", batch or 2048, tables, fields, 1.1, raw_hash_ids=True, seed=seed,
                        description="1000 multi-hot fields (len 1-10), dim 8/16 alternating, raw "
                                    "64-bit hashed IDs folded mod rows (1e4-1e6), Zipf 1.1, sum")
    if index == 5:
        n_one = 50 if n_fields is None else max(1, (n_fields * 5) // 6)
        n_seq = 10 if n_fields is None else max(1, n_fields - n_one)
        F = n_one + n_seq
        tables = [TableSpec(rows_of(2_000_000), 64, BF16) for _ in range(F)]
        fields = [FieldSpec(t, SUM, 1, 1) for t in range(n_one)]
        fields += [FieldSpec(n_one + t, SUM, len_of(100), len_of(1000)) for t in range(n_seq)]
        return Workload("cfg5", batch or 1024, tables, fields, 1.1, seed=seed,
                        description="50 one-hot + 10 sequence fields (len 100-1000), dim 64, bf16 "
                                    "tables 2M rows, Zipf 1.1, sum")
    raise ValueError("config index must be 1..5")


# ---------------------------------------------------------------------------
# ID / gradient generation
# ---------------------------------------------------------------------------
def _stream(seed: int, purpose: int, a: int = 0, b: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[seed & _M64, (purpose << 48) | (a << 24) | b]))


def _affine(seed: int, table: int, rows: int):
    """Multiplier/offset of the rank -> row permutation (k*a + c) mod rows."""
    a = int(rows * 0.6180339887498949) | 1
    while math.gcd(a, rows) != 1:
        a += 2
    c = mix64(seed + _GOLD * (table + 17)) % rows
    return a % rows if rows > 1 else 0, c


def _zipf_ranks(rows: int, alpha: Optional[float], u: np.ndarray) -> np.ndarray:
    """Map uniforms in [0,1) to ranks 0..rows-1 with P(rank k) ~ (k+1)^-alpha."""
    if alpha is None:
        return np.minimum((u * rows).astype(np.int64), rows - 1)
    w = np.arange(1, rows + 1, dtype=np.float64)
    np.power(w, -alpha, out=w)
    np.cumsum(w, out=w)
    w /= w[-1]
    k = np.searchsorted(w, u, side="right")
    return np.minimum(k, rows - 1).astype(np.int64)


def make_batches(wl: Workload, n_batches: int, first: int = 0) -> List[Batch]:
    """Batches first..first+n_batches-1 of the workload's stream.  Batch i is
    the same whatever range it is generated in."""
    B, F = wl.batch, wl.n_fields
    lens = np.empty((n_batches, F, B), dtype=np.int64)
    for i in range(n_batches):
        for f, fs in enumerate(wl.fields):
            g = _stream(wl.seed, 1, f, first + i)
            lens[i, f] = g.integers(fs.len_lo, fs.len_hi + 1, size=B)
    ids_parts = [[None] * F for _ in range(n_batches)]
    for f, fs in enumerate(wl.fields):
        rows = wl.tables[fs.table].rows
        n_each = lens[:, f, :].sum(axis=1)
        u = np.concatenate([_stream(wl.seed, 2, f, first + i).random(int(n_each[i]))
                            for i in range(n_batches)])
        k = _zipf_ranks(rows, wl.alpha, u)
        if wl.raw_hash_ids:
            fkey = np.uint64(mix64(wl.seed + _GOLD * (f + 101)))
            raw = _mix64_np(fkey + k.astype(np.uint64) * np.uint64(_GOLD))
            vals = raw.view(np.int64)
        else:
            a, c = _affine(wl.seed, fs.table, rows)
            vals = ((k.astype(np.uint64) * np.uint64(a) + np.uint64(c)) % np.uint64(rows)).astype(np.int64)
        pos = 0
        for i in range(n_batches):
            ids_parts[i][f] = vals[pos:pos + int(n_each[i])]
            pos += int(n_each[i])
    out = []
    D = wl.out_dim
    for i in range(n_batches):
        ids = np.ascontiguousarray(np.concatenate(ids_parts[i]))
        offsets = np.zeros(F * B + 1, dtype=np.int64)
        np.cumsum(lens[i].reshape(-1), out=offsets[1:])
        assert offsets[-1] < 2 ** 31
        grad = _stream(wl.seed, 3, 0, first + i).standard_normal((B, D), dtype=np.float32)
        out.append(Batch(ids, offsets.astype(np.int32), grad))
    return out


def make_batch(wl: Workload, index: int = 0) -> Batch:
    return make_batches(wl, 1, first=index)[0]


def split_batch(batch: Batch, n_fields: int, B: int, n_micro: int) -> List[Batch]:
    """The batch cut into `n_micro` micro-batches of consecutive samples, as even as they come
    (sizes differ by one at most), each in the layer's field-major layout.  Data movement only."""
    M = max(1, min(int(n_micro), B))
    bounds = [(B * m) // M for m in range(M + 1)]
    off = batch.offsets.astype(np.int64)
    out = []
    for m in range(M):
        b0, b1 = bounds[m], bounds[m + 1]
        parts, lens = [], []
        for f in range(n_fields):
            o = off[f * B + b0:f * B + b1 + 1]
            parts.append(batch.ids[o[0]:o[-1]])
            lens.append(np.diff(o))
        offsets = np.zeros(n_fields * (b1 - b0) + 1, dtype=np.int64)
        np.cumsum(np.concatenate(lens), out=offsets[1:])
        out.append(Batch(np.ascontiguousarray(np.concatenate(parts)), offsets.astype(np.int32),
                         np.ascontiguousarray(batch.grad_out[b0:b1])))
    return out


# ---------------------------------------------------------------------------
# table values (host side; the device twin is in fill.hip)
# ---------------------------------------------------------------------------
_cpu_lib = None
_hip_lib = None


def build_cpu(force: bool = False) -> str:
    so = os.path.join(_HERE, "libsynth_cpu.so")
    src = os.path.join(_HERE, "fill.c")
    if force or not os.path.exists(so) or os.path.getmtime(so) < os.path.getmtime(src):
        subprocess.check_call(["gcc", "-O2", "-fPIC", "-shared", "-ffp-contract=off", "-o", so, src])
    return so


def build_hip(force: bool = False) -> str:
    so = os.path.join(_HERE, "libsynth_hip.so")
    src = os.path.join(_HERE, "fill.hip")
    if force or not os.path.exists(so) or os.path.getmtime(so) < os.path.getmtime(src):
        subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-O3", "-fPIC", "-shared",
                               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                               "-o", so, src])
    return so


def _cpu():
    global _cpu_lib
    if _cpu_lib is None:
        lib = ctypes.CDLL(build_cpu())
        for name in ("synth_rows_f32", "synth_rows_bf16"):
            fn = getattr(lib, name)
            fn.restype = None
            fn.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_int64,
                           ctypes.c_int32, ctypes.c_uint64, ctypes.c_int32]
        _cpu_lib = lib
    return _cpu_lib


def table_rows(wl: Workload, table: int, rows: Optional[Sequence[int]] = None,
               row0: int = 0, n: Optional[int] = None) -> np.ndarray:
    """Initial values of some rows of a table: float32 [n, dim] for fp32 tables,
    uint16 bit patterns [n, dim] for bf16 tables.  `rows` = explicit row list,
    else the range [row0, row0+n)."""
    ts = wl.tables[table]
    if rows is not None:
        idx = np.ascontiguousarray(np.asarray(rows, dtype=np.int64))
        n = idx.shape[0]
        ptr = idx.ctypes.data
    else:
        if n is None:
            n = ts.rows - row0
        ptr = None
    out = np.empty((n, ts.dim), dtype=np.float32 if ts.dtype == F32 else np.uint16)
    fn = _cpu().synth_rows_f32 if ts.dtype == F32 else _cpu().synth_rows_bf16
    fn(out.ctypes.data, n, ptr, row0, ts.dim, wl.seed, table)
    return out


def fill_device(ptr: int, rows: int, dim: int, dtype: int, seed: int, table: int, stream: int) -> None:
    """Write a whole table's initial values into device memory at `ptr`."""
    global _hip_lib
    if _hip_lib is None:
        so = os.path.join(_HERE, "libsynth_hip.so")
        if not os.path.exists(so):
            raise RuntimeError("synth/libsynth_hip.so is not built (run __graft_entry__.build())")
        lib = ctypes.CDLL(so)
        lib.synth_fill_device.restype = ctypes.c_int
        lib.synth_fill_device.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32,
                                          ctypes.c_uint64, ctypes.c_int32, ctypes.c_void_p]
        _hip_lib = lib
    rc = _hip_lib.synth_fill_device(ptr, rows, dim, dtype, seed, table, stream)
    if rc != 0:
        raise RuntimeError(f"synth_fill_device failed with code {rc}")


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)
