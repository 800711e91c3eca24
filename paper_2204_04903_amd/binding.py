"""ctypes binding of libpk.so: the same calls as include/pk.h, argument
marshalling only.  Every step of the path runs in the library's HIP kernels;
PyTorch is used by callers for device memory and streams, nothing here computes.

There is no fallback: if the shared library is missing, importing a function
from it raises.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import List, Optional, Sequence, Tuple

_HERE = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_HERE)
LIB_PATH = os.path.join(_HERE, "libpk.so")

PK_OK, PK_EINVAL, PK_ESHAPE, PK_EWORKSPACE, PK_EOVERFLOW, PK_EHIP, PK_ENOMEM = range(7)
PK_F32, PK_BF16 = 0, 1
PK_SUM, PK_MEAN = 0, 1

EXPORTS = [
    "pk_plan_create", "pk_plan_destroy", "pk_plan_num_packs", "pk_plan_pack_info", "pk_plan_pack_fields",
    "pk_plan_table_slot", "pk_plan_field_col", "pk_plan_out_dim", "pk_workspace_bytes", "pk_forward",
    "pk_backward_update", "pk_ctx_pack", "pk_ctx_error", "pk_profile_enable", "pk_profile_read", "pk_last_error",
    "pk_hh_scratch_bytes", "pk_hh_init", "pk_hh_forward", "pk_hh_backward_update", "pk_hh_end_iteration",
    "pk_hh_hot_count", "pk_forward_dedup", "pk_forward_pool", "pk_micro_batch_size", "pk_forward_static",
    "pk_partition_scratch_bytes", "pk_partition_unique",
]


class pk_table_desc(ctypes.Structure):
    _fields_ = [("rows", ctypes.c_int64), ("dim", ctypes.c_int32), ("dtype", ctypes.c_int32)]


class pk_field_desc(ctypes.Structure):
    _fields_ = [("table", ctypes.c_int32), ("pool", ctypes.c_int32)]


class pk_plan_opts(ctypes.Structure):
    _fields_ = [("max_batch", ctypes.c_int32), ("max_nnz", ctypes.c_int64), ("max_shards", ctypes.c_int32),
                ("field_volume", ctypes.POINTER(ctypes.c_double)), ("interleave_groups", ctypes.c_int32),
                ("debug", ctypes.c_int32)]


class pk_hh_pack(ctypes.Structure):
    _fields_ = [("W_cold", ctypes.c_void_p), ("A_cold", ctypes.c_void_p), ("W_hot", ctypes.c_void_p),
                ("A_hot", ctypes.c_void_p), ("slot_of", ctypes.c_void_p), ("hot_row", ctypes.c_void_p),
                ("fcounter", ctypes.c_void_p), ("hot_rows", ctypes.c_int64)]


class PkError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"pk status {status}: {message}")
        self.status = status


def build(force: bool = True) -> str:
    """Compile the library for gfx950 (hipcc cross-compiles without a GPU)."""
    src = [os.path.join(_HERE, "csrc", "pk_plan.cpp"), os.path.join(_HERE, "csrc", "pk_device.hip")]
    deps = src + [os.path.join(_HERE, "csrc", f) for f in sorted(os.listdir(os.path.join(_HERE, "csrc")))
                  if f.endswith(".h")] + [os.path.join(_ROOT, "include", "pk.h")]
    if not force and os.path.exists(LIB_PATH) and all(os.path.getmtime(LIB_PATH) >= os.path.getmtime(d) for d in deps):
        return LIB_PATH
    cmd = ["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-I" + os.path.join(_ROOT, "include"),
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-munsafe-fp-atomics",
           "-o", LIB_PATH] + src
    subprocess.check_call(cmd)
    return LIB_PATH


_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is not built; run __graft_entry__.build() (there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
        L.pk_plan_create.restype = ctypes.c_int
        L.pk_plan_create.argtypes = [ctypes.POINTER(pk_table_desc), i32, ctypes.POINTER(pk_field_desc), i32,
                                     ctypes.POINTER(pk_plan_opts), ctypes.POINTER(vp)]
        L.pk_plan_destroy.restype = None
        L.pk_plan_destroy.argtypes = [vp]
        L.pk_plan_num_packs.restype = i32
        L.pk_plan_num_packs.argtypes = [vp]
        L.pk_plan_pack_info.restype = ctypes.c_int
        L.pk_plan_pack_info.argtypes = [vp, i32] + [ctypes.POINTER(i32)] * 2 + [ctypes.POINTER(i64)] + [ctypes.POINTER(i32)] * 3
        L.pk_plan_pack_fields.restype = ctypes.c_int
        L.pk_plan_pack_fields.argtypes = [vp, i32, ctypes.POINTER(i32)]
        L.pk_plan_table_slot.restype = ctypes.c_int
        L.pk_plan_table_slot.argtypes = [vp, i32, ctypes.POINTER(i32), ctypes.POINTER(i64)]
        L.pk_plan_field_col.restype = ctypes.c_int
        L.pk_plan_field_col.argtypes = [vp, i32, ctypes.POINTER(i64)]
        L.pk_plan_out_dim.restype = i64
        L.pk_plan_out_dim.argtypes = [vp]
        L.pk_workspace_bytes.restype = ctypes.c_size_t
        L.pk_workspace_bytes.argtypes = [vp, i32, i64]
        L.pk_forward.restype = ctypes.c_int
        L.pk_forward.argtypes = [vp, ctypes.POINTER(vp), vp, vp, i32, i64, vp, i64, vp, ctypes.c_size_t, vp]
        L.pk_forward_static.restype = ctypes.c_int
        L.pk_forward_static.argtypes = [vp, ctypes.POINTER(vp), vp, vp, i32, i64, vp, i64, vp]
        L.pk_partition_scratch_bytes.restype = ctypes.c_size_t
        L.pk_partition_scratch_bytes.argtypes = [vp, i64, i32]
        L.pk_partition_unique.restype = ctypes.c_int
        L.pk_partition_unique.argtypes = [vp, vp, ctypes.c_size_t, i32, i64, i32, i32, vp, vp, vp, vp, ctypes.c_size_t, vp]
        L.pk_forward_dedup.restype = ctypes.c_int
        L.pk_forward_dedup.argtypes = [vp, vp, vp, i32, i64, vp, ctypes.c_size_t, vp]
        L.pk_forward_pool.restype = ctypes.c_int
        L.pk_forward_pool.argtypes = [vp, ctypes.POINTER(vp), i32, i64, vp, i64, vp, ctypes.c_size_t, vp]
        L.pk_micro_batch_size.restype = ctypes.c_int32
        L.pk_micro_batch_size.argtypes = [vp, i32, i64, ctypes.c_size_t, ctypes.c_size_t]
        L.pk_backward_update.restype = ctypes.c_int
        L.pk_backward_update.argtypes = [vp, ctypes.POINTER(vp), ctypes.POINTER(vp), vp, i64, i32, i64,
                                         ctypes.c_float, ctypes.c_float, vp, ctypes.c_size_t, vp]
        L.pk_ctx_pack.restype = ctypes.c_int
        L.pk_ctx_pack.argtypes = [vp, vp, i32, i64, i32] + [ctypes.POINTER(vp)] * 5 + [ctypes.POINTER(i64)] * 2
        L.pk_ctx_error.restype = ctypes.c_int
        L.pk_ctx_error.argtypes = [vp, vp, ctypes.POINTER(i32)]
        L.pk_profile_enable.restype = ctypes.c_int
        L.pk_profile_enable.argtypes = [vp, i32]
        L.pk_profile_read.restype = i32
        L.pk_profile_read.argtypes = [vp, ctypes.POINTER(ctypes.c_char_p), ctypes.POINTER(ctypes.c_double),
                                      ctypes.POINTER(i64), i32]
        L.pk_last_error.restype = ctypes.c_char_p
        L.pk_last_error.argtypes = []
        hp = ctypes.POINTER(pk_hh_pack)
        L.pk_hh_scratch_bytes.restype = ctypes.c_size_t
        L.pk_hh_scratch_bytes.argtypes = [vp, hp]
        L.pk_hh_init.restype = ctypes.c_int
        L.pk_hh_init.argtypes = [vp, hp, vp]
        L.pk_hh_forward.restype = ctypes.c_int
        L.pk_hh_forward.argtypes = [vp, hp, vp, vp, i32, i64, vp, i64, vp, ctypes.c_size_t, vp]
        L.pk_hh_backward_update.restype = ctypes.c_int
        L.pk_hh_backward_update.argtypes = [vp, hp, vp, i64, i32, i64, ctypes.c_float, ctypes.c_float, vp,
                                            ctypes.c_size_t, vp]
        L.pk_hh_end_iteration.restype = ctypes.c_int
        L.pk_hh_end_iteration.argtypes = [vp, hp, i64, i32, i32, i32, i64, vp, ctypes.c_size_t, vp, ctypes.c_size_t, vp,
                                          ctypes.POINTER(i64), ctypes.POINTER(i64), ctypes.POINTER(i32)]
        L.pk_hh_hot_count.restype = ctypes.c_int
        L.pk_hh_hot_count.argtypes = [vp, i32, ctypes.POINTER(i64)]
        _lib = L
    return _lib


def pk_last_error() -> str:
    return lib().pk_last_error().decode()


def _check(status: int) -> None:
    if status != PK_OK:
        raise PkError(status, pk_last_error())


def _ptr(x) -> Optional[int]:
    """A device/host address from an int, None, or anything with data_ptr() (torch tensors)."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return x.data_ptr()


def pk_plan_create(tables: Sequence[Tuple[int, int, int]], fields: Sequence[Tuple[int, int]],
                   max_batch: int = 0, max_nnz: int = 0, max_shards: int = 0,
                   field_volume: Optional[Sequence[float]] = None, interleave_groups: int = 0,
                   debug: int = 0) -> int:
    """tables: (rows, dim, dtype) each; fields: (table, pool) each.  Returns the plan handle."""
    T = (pk_table_desc * max(len(tables), 1))(*[pk_table_desc(int(r), int(d), int(t)) for r, d, t in tables])
    Fd = (pk_field_desc * max(len(fields), 1))(*[pk_field_desc(int(t), int(p)) for t, p in fields])
    opts = pk_plan_opts(int(max_batch), int(max_nnz), int(max_shards), None, int(interleave_groups), int(debug))
    if field_volume is not None:
        vol = (ctypes.c_double * len(field_volume))(*[float(v) for v in field_volume])
        opts.field_volume = ctypes.cast(vol, ctypes.POINTER(ctypes.c_double))
    out = ctypes.c_void_p()
    _check(lib().pk_plan_create(T, len(tables), Fd, len(fields), ctypes.byref(opts), ctypes.byref(out)))
    return out.value


def pk_plan_destroy(plan: int) -> None:
    lib().pk_plan_destroy(plan)


def pk_plan_num_packs(plan: int) -> int:
    return int(lib().pk_plan_num_packs(plan))


def pk_plan_pack_info(plan: int, p: int) -> dict:
    dim, dtype, nf, nt, kb = (ctypes.c_int32() for _ in range(5))
    rows = ctypes.c_int64()
    _check(lib().pk_plan_pack_info(plan, p, ctypes.byref(dim), ctypes.byref(dtype), ctypes.byref(rows),
                                   ctypes.byref(nf), ctypes.byref(nt), ctypes.byref(kb)))
    return dict(dim=dim.value, dtype=dtype.value, total_rows=rows.value, n_fields=nf.value, n_tables=nt.value,
                key_bytes=kb.value)


def pk_plan_pack_fields(plan: int, p: int) -> List[int]:
    n = pk_plan_pack_info(plan, p)["n_fields"]
    buf = (ctypes.c_int32 * max(n, 1))()
    _check(lib().pk_plan_pack_fields(plan, p, buf))
    return list(buf[:n])


def pk_plan_table_slot(plan: int, table: int) -> Tuple[int, int]:
    pack, base = ctypes.c_int32(), ctypes.c_int64()
    _check(lib().pk_plan_table_slot(plan, table, ctypes.byref(pack), ctypes.byref(base)))
    return pack.value, base.value


def pk_plan_field_col(plan: int, field: int) -> int:
    col = ctypes.c_int64()
    _check(lib().pk_plan_field_col(plan, field, ctypes.byref(col)))
    return col.value


def pk_plan_out_dim(plan: int) -> int:
    return int(lib().pk_plan_out_dim(plan))


def pk_workspace_bytes(plan: int, B: int, nnz: int) -> int:
    n = int(lib().pk_workspace_bytes(plan, B, nnz))
    if n == 0:
        raise PkError(PK_EINVAL, pk_last_error())
    return n


def _ptr_array(xs):
    arr = (ctypes.c_void_p * max(len(xs), 1))(*[_ptr(x) for x in xs])
    return arr


def pk_forward(plan: int, W: Sequence, ids, offsets, B: int, nnz: int, out, out_row_stride: int,
               workspace, ws_bytes: int, stream: int = 0) -> None:
    _check(lib().pk_forward(plan, _ptr_array(W), _ptr(ids), _ptr(offsets), B, nnz, _ptr(out), out_row_stride,
                            _ptr(workspace), ws_bytes, stream))


def pk_forward_static(plan: int, W: Sequence, ids, offsets, B: int, nnz: int, out, out_row_stride: int,
                      stream: int = 0) -> None:
    _check(lib().pk_forward_static(plan, _ptr_array(W), _ptr(ids), _ptr(offsets), B, nnz, _ptr(out), out_row_stride,
                                   stream))


def pk_partition_scratch_bytes(plan: int, nnz: int, n_owners: int) -> int:
    n = int(lib().pk_partition_scratch_bytes(plan, nnz, n_owners))
    if n == 0:
        raise PkError(PK_EINVAL, lib().pk_last_error().decode())
    return n


def pk_partition_unique(plan: int, workspace, ws_bytes: int, B: int, nnz: int, p: int, n_owners: int, part_keys,
                        part_index, part_offsets, scratch, scratch_bytes: int, stream: int = 0) -> None:
    _check(lib().pk_partition_unique(plan, _ptr(workspace), ws_bytes, B, nnz, p, n_owners, _ptr(part_keys),
                                     _ptr(part_index), _ptr(part_offsets), _ptr(scratch), scratch_bytes, stream))


def pk_forward_dedup(plan: int, ids, offsets, B: int, nnz: int, workspace, ws_bytes: int, stream: int = 0) -> None:
    _check(lib().pk_forward_dedup(plan, _ptr(ids), _ptr(offsets), B, nnz, _ptr(workspace), ws_bytes, stream))


def pk_forward_pool(plan: int, W: Sequence, B: int, nnz: int, out, out_row_stride: int, workspace, ws_bytes: int,
            stream: int = 0) -> None:
    _check(lib().pk_forward_pool(plan, _ptr_array(W), B, nnz, _ptr(out), out_row_stride, _ptr(workspace), ws_bytes, stream))


def pk_micro_batch_size(plan: int, B: int, nnz: int, ws_bound_bytes: int = 0, act_bound_bytes: int = 0) -> int:
    n = int(lib().pk_micro_batch_size(plan, B, nnz, ws_bound_bytes, act_bound_bytes))
    if n < 0:
        raise PkError(PK_EINVAL, pk_last_error())
    return n


def pk_backward_update(plan: int, W: Sequence, A: Sequence, grad_out, grad_row_stride: int, B: int, nnz: int,
                       lr: float, eps: float, workspace, ws_bytes: int, stream: int = 0) -> None:
    _check(lib().pk_backward_update(plan, _ptr_array(W), _ptr_array(A), _ptr(grad_out), grad_row_stride, B, nnz,
                                    lr, eps, _ptr(workspace), ws_bytes, stream))


def _hh_array(packs: Sequence[dict]):
    """packs: per pack a dict with W_cold, A_cold, W_hot, A_hot, slot_of, hot_row, fcounter (tensors or
    addresses) and hot_rows."""
    arr = (pk_hh_pack * max(len(packs), 1))()
    for i, d in enumerate(packs):
        for name in ("W_cold", "A_cold", "W_hot", "A_hot", "slot_of", "hot_row", "fcounter"):
            setattr(arr[i], name, _ptr(d.get(name)))
        arr[i].hot_rows = int(d["hot_rows"])
    return arr


def pk_hh_scratch_bytes(plan: int, packs: Sequence[dict]) -> int:
    n = int(lib().pk_hh_scratch_bytes(plan, _hh_array(packs)))
    if n == 0:
        raise PkError(PK_EINVAL, pk_last_error())
    return n


def pk_hh_init(plan: int, packs: Sequence[dict], stream: int = 0) -> None:
    _check(lib().pk_hh_init(plan, _hh_array(packs), stream))


def pk_hh_forward(plan: int, packs: Sequence[dict], ids, offsets, B: int, nnz: int, out, out_row_stride: int,
                  workspace, ws_bytes: int, stream: int = 0) -> None:
    _check(lib().pk_hh_forward(plan, _hh_array(packs), _ptr(ids), _ptr(offsets), B, nnz, _ptr(out), out_row_stride,
                               _ptr(workspace), ws_bytes, stream))


def pk_hh_backward_update(plan: int, packs: Sequence[dict], grad_out, grad_row_stride: int, B: int, nnz: int,
                          lr: float, eps: float, workspace, ws_bytes: int, stream: int = 0) -> None:
    _check(lib().pk_hh_backward_update(plan, _hh_array(packs), _ptr(grad_out), grad_row_stride, B, nnz, lr, eps,
                                       _ptr(workspace), ws_bytes, stream))


def pk_hh_end_iteration(plan: int, packs: Sequence[dict], itr: int, warmup_iters: int, flush_iters: int, B: int,
                        nnz: int, workspace, ws_bytes: int, scratch, scratch_bytes: int, stream: int = 0,
                        want_counts: bool = True):
    """Returns (queried per pack, hits per pack, flushed)."""
    n = len(packs)
    q = (ctypes.c_int64 * max(n, 1))()
    h = (ctypes.c_int64 * max(n, 1))()
    fl = ctypes.c_int32()
    _check(lib().pk_hh_end_iteration(plan, _hh_array(packs), itr, warmup_iters, flush_iters, B, nnz, _ptr(workspace),
                                     ws_bytes, _ptr(scratch), scratch_bytes, stream, q if want_counts else None,
                                     h if want_counts else None, ctypes.byref(fl)))
    return list(q)[:n], list(h)[:n], bool(fl.value)


def pk_hh_hot_count(plan: int, p: int) -> int:
    n = ctypes.c_int64()
    _check(lib().pk_hh_hot_count(plan, p, ctypes.byref(n)))
    return n.value


def pk_ctx_pack(plan: int, workspace, B: int, nnz: int, p: int) -> dict:
    """Device addresses of pack p's saved context plus nnz_p and n_unique (synchronises)."""
    ptrs = [ctypes.c_void_p() for _ in range(5)]
    nnz_p, n_unique = ctypes.c_int64(), ctypes.c_int64()
    _check(lib().pk_ctx_pack(plan, _ptr(workspace), B, nnz, p, *[ctypes.byref(x) for x in ptrs],
                             ctypes.byref(nnz_p), ctypes.byref(n_unique)))
    names = ("keys", "unique", "inverse", "packed_offsets", "seg_offsets")
    d = {n: (x.value or 0) for n, x in zip(names, ptrs)}
    d["nnz_p"], d["n_unique"] = nnz_p.value, n_unique.value
    return d


def pk_ctx_error(plan: int, workspace) -> int:
    w = ctypes.c_int32()
    _check(lib().pk_ctx_error(plan, _ptr(workspace), ctypes.byref(w)))
    return w.value


def pk_profile_enable(plan: int, enable: bool) -> None:
    _check(lib().pk_profile_enable(plan, 1 if enable else 0))


def pk_profile_read(plan: int, max_entries: int = 64) -> dict:
    names = (ctypes.c_char_p * max_entries)()
    ms = (ctypes.c_double * max_entries)()
    cnt = (ctypes.c_int64 * max_entries)()
    n = lib().pk_profile_read(plan, names, ms, cnt, max_entries)
    return {names[i].decode(): (ms[i], cnt[i]) for i in range(n)}
