"""Buffer management around the C ABI: allocates the packed tables, the Adagrad
accumulators, the output and the workspace as torch device tensors and hands
their addresses to the library.  No arithmetic happens here."""
from __future__ import annotations

from typing import List, Sequence, Tuple

import numpy as np
import torch

from . import binding as pk


class PackedEmbedding:
    def __init__(self, tables: Sequence[Tuple[int, int, int]], fields: Sequence[Tuple[int, int]],
                 device: str = "cuda:0", **plan_opts):
        self.tables, self.fields = list(tables), list(fields)
        self.device = torch.device(device)
        self.plan = pk.pk_plan_create(self.tables, self.fields, **plan_opts)
        self.n_packs = pk.pk_plan_num_packs(self.plan)
        self.packs = [pk.pk_plan_pack_info(self.plan, p) for p in range(self.n_packs)]
        self.pack_fields = [pk.pk_plan_pack_fields(self.plan, p) for p in range(self.n_packs)]
        self.table_slot = [pk.pk_plan_table_slot(self.plan, t) for t in range(len(self.tables))]
        self.field_col = [pk.pk_plan_field_col(self.plan, f) for f in range(len(self.fields))]
        self.out_dim = pk.pk_plan_out_dim(self.plan)
        self.W: List[torch.Tensor] = []
        self.A: List[torch.Tensor] = []
        for info in self.packs:
            dt = torch.float32 if info["dtype"] == pk.PK_F32 else torch.bfloat16
            self.W.append(torch.empty((info["total_rows"], info["dim"]), dtype=dt, device=self.device))
            self.A.append(torch.zeros((info["total_rows"], info["dim"]), dtype=torch.float32, device=self.device))
        self.ws = None
        self.ws_bytes = 0
        self._shape = None

    def close(self):
        if self.plan:
            pk.pk_plan_destroy(self.plan)
            self.plan = None

    def table_view(self, t: int) -> torch.Tensor:
        p, base = self.table_slot[t]
        return self.W[p][base:base + self.tables[t][0]]

    def acc_view(self, t: int) -> torch.Tensor:
        p, base = self.table_slot[t]
        return self.A[p][base:base + self.tables[t][0]]

    def load_table(self, t: int, values: np.ndarray) -> None:
        """values: float32 [rows, dim], or uint16 bf16 bit patterns for a bf16 table."""
        values = np.ascontiguousarray(values)
        if self.tables[t][2] == pk.PK_BF16:
            v = torch.from_numpy(values.view(np.int16)).view(torch.bfloat16)
        else:
            v = torch.from_numpy(values)
        self.table_view(t).copy_(v.to(self.device))

    def _ensure_ws(self, B: int, nnz: int) -> None:
        need = pk.pk_workspace_bytes(self.plan, B, nnz)
        if self.ws is None or self.ws_bytes < need:
            self.ws = torch.empty(need + 256, dtype=torch.uint8, device=self.device)
            self.ws_bytes = need
        self._shape = (B, nnz)

    def forward(self, ids: torch.Tensor, offsets: torch.Tensor, B: int, out: torch.Tensor = None) -> torch.Tensor:
        nnz = int(ids.shape[0])
        self._ensure_ws(B, nnz)
        if out is None:
            out = torch.empty((B, self.out_dim), dtype=torch.float32, device=self.device)
        stream = torch.cuda.current_stream(self.device).cuda_stream
        pk.pk_forward(self.plan, self.W, ids, offsets, B, nnz, out, out.stride(0), self.ws, self.ws_bytes, stream)
        return out

    def backward_update(self, grad_out: torch.Tensor, lr: float, eps: float) -> None:
        B, nnz = self._shape
        stream = torch.cuda.current_stream(self.device).cuda_stream
        pk.pk_backward_update(self.plan, self.W, self.A, grad_out, grad_out.stride(0), B, nnz, lr, eps, self.ws,
                              self.ws_bytes, stream)

    def ctx(self, p: int) -> dict:
        """Pack p's saved context copied to numpy (synchronises)."""
        B, nnz = self._shape
        d = pk.pk_ctx_pack(self.plan, self.ws, B, nnz, p)
        base = self.ws.data_ptr()

        def grab(addr, n, dtype):
            off = addr - base
            return self.ws[off:off + 4 * n].view(dtype).cpu().numpy().copy()

        k = len(self.pack_fields[p])
        return dict(
            nnz_p=d["nnz_p"], n_unique=d["n_unique"],
            keys=grab(d["keys"], d["nnz_p"], torch.int32).view(np.uint32),
            unique=grab(d["unique"], d["n_unique"], torch.int32).view(np.uint32),
            inverse=grab(d["inverse"], d["nnz_p"], torch.int32),
            packed_offsets=grab(d["packed_offsets"], k * B + 1, torch.int32),
            seg_offsets=grab(d["seg_offsets"], d["n_unique"] + 1, torch.int32),
        )

    def error_word(self) -> int:
        return pk.pk_ctx_error(self.plan, self.ws)

    def partition(self, p: int, n_owners: int):
        """Sec. II-D Partition of pack p's distinct keys by owner (row mod n_owners), after a forward pass.
        Returns device tensors (part_keys [nnz] int32 bits of uint32, part_index [nnz] int32, part_offsets
        [n_owners + 1] int32); only the first part_offsets[-1] entries of the first two are meaningful."""
        B, nnz = self._shape
        need = pk.pk_partition_scratch_bytes(self.plan, nnz, n_owners)
        scratch = torch.empty(need, dtype=torch.uint8, device=self.device)
        keys = torch.empty(max(nnz, 1), dtype=torch.int32, device=self.device)
        index = torch.empty(max(nnz, 1), dtype=torch.int32, device=self.device)
        offsets = torch.empty(n_owners + 1, dtype=torch.int32, device=self.device)
        stream = torch.cuda.current_stream(self.device).cuda_stream
        pk.pk_partition_unique(self.plan, self.ws, self.ws_bytes, B, nnz, p, n_owners, keys, index, offsets, scratch,
                               need, stream)
        return keys, index, offsets


class MicroBatchPipeline:
    """D-Interleaving of the layer (Sec. III-C): micro-batches pass through it one after the other, and the
    dedup of the next one (integer work that reads no table) is enqueued on a second stream while the current
    one is pooled and updated on the caller's stream.  Two workspaces, sized for a micro-batch, alternate.
    Scheduling only: every step runs in the library's kernels.

        t = pipe.submit(ids0, offsets0, B0)
        for m in range(M):
            nxt = pipe.submit(ids[m + 1], offsets[m + 1], B[m + 1]) if m + 1 < M else None
            pipe.pool(t, out[m]); ...; pipe.backward_update(t, grad[m], lr, eps)
            t = nxt

    The tensors handed to `submit` must stay alive until the micro-batch has been updated."""

    def __init__(self, layer: PackedEmbedding, max_B: int, max_nnz: int):
        self.layer = layer
        self.ws_bytes = pk.pk_workspace_bytes(layer.plan, max_B, max_nnz)
        self.ws = [torch.empty(self.ws_bytes + 256, dtype=torch.uint8, device=layer.device) for _ in range(2)]
        self.side = torch.cuda.Stream(device=layer.device)
        self.ev_inputs = [torch.cuda.Event() for _ in range(2)]
        self.ev_dedup = [torch.cuda.Event() for _ in range(2)]
        self.count = 0

    def submit(self, ids: torch.Tensor, offsets: torch.Tensor, B: int) -> dict:
        """Enqueue the dedup of a micro-batch.  It starts once everything enqueued so far on the caller's
        stream has run: the inputs are there, and the workspace's previous micro-batch has been updated."""
        layer, slot = self.layer, self.count % 2
        self.count += 1
        nnz = int(ids.shape[0])
        if pk.pk_workspace_bytes(layer.plan, B, nnz) > self.ws_bytes:
            raise ValueError("micro-batch larger than the pipeline was sized for")
        main = torch.cuda.current_stream(layer.device)
        self.ev_inputs[slot].record(main)
        self.side.wait_event(self.ev_inputs[slot])
        pk.pk_forward_dedup(layer.plan, ids, offsets, B, nnz, self.ws[slot], self.ws_bytes, self.side.cuda_stream)
        self.ev_dedup[slot].record(self.side)
        return dict(slot=slot, B=B, nnz=nnz)

    def pool(self, t: dict, out: torch.Tensor) -> torch.Tensor:
        layer = self.layer
        main = torch.cuda.current_stream(layer.device)
        main.wait_event(self.ev_dedup[t["slot"]])
        pk.pk_forward_pool(layer.plan, layer.W, t["B"], t["nnz"], out, out.stride(0), self.ws[t["slot"]],
                           self.ws_bytes, main.cuda_stream)
        return out

    def backward_update(self, t: dict, grad_out: torch.Tensor, lr: float, eps: float) -> None:
        layer = self.layer
        main = torch.cuda.current_stream(layer.device)
        pk.pk_backward_update(layer.plan, layer.W, layer.A, grad_out, grad_out.stride(0), t["B"], t["nnz"], lr, eps,
                              self.ws[t["slot"]], self.ws_bytes, main.cuda_stream)

    def ctx_error(self, t: dict) -> int:
        return pk.pk_ctx_error(self.layer.plan, self.ws[t["slot"]])


class HybridEmbedding(PackedEmbedding):
    """The layer with a Hot-storage in front of its tables (HybridHash): the tables and accumulators are the
    Cold-storage, in pinned host memory when `cold_on_host`, and the `hot_rows[p]` most queried rows of pack p
    live in device memory.  Buffer management only."""

    def __init__(self, tables, fields, hot_rows: Sequence[int], warmup_iters: int, flush_iters: int,
                 cold_on_host: bool = True, device: str = "cuda:0", **plan_opts):
        self.tables, self.fields = list(tables), list(fields)
        self.device = torch.device(device)
        self.plan = pk.pk_plan_create(self.tables, self.fields, **plan_opts)
        self.n_packs = pk.pk_plan_num_packs(self.plan)
        self.packs = [pk.pk_plan_pack_info(self.plan, p) for p in range(self.n_packs)]
        self.pack_fields = [pk.pk_plan_pack_fields(self.plan, p) for p in range(self.n_packs)]
        self.table_slot = [pk.pk_plan_table_slot(self.plan, t) for t in range(len(self.tables))]
        self.field_col = [pk.pk_plan_field_col(self.plan, f) for f in range(len(self.fields))]
        self.out_dim = pk.pk_plan_out_dim(self.plan)
        self.warmup_iters, self.flush_iters, self.itr = int(warmup_iters), int(flush_iters), 0
        self.W, self.A, self.hh = [], [], []
        for p, info in enumerate(self.packs):
            dt = torch.float32 if info["dtype"] == pk.PK_F32 else torch.bfloat16
            R, D, k = info["total_rows"], info["dim"], int(hot_rows[p])
            if cold_on_host:
                Wc = torch.empty((R, D), dtype=dt, pin_memory=True)
                Ac = torch.zeros((R, D), dtype=torch.float32, pin_memory=True)
            else:
                Wc = torch.empty((R, D), dtype=dt, device=self.device)
                Ac = torch.zeros((R, D), dtype=torch.float32, device=self.device)
            self.W.append(Wc)
            self.A.append(Ac)
            self.hh.append(dict(
                W_cold=Wc, A_cold=Ac, hot_rows=k,
                W_hot=torch.empty((max(k, 1), D), dtype=dt, device=self.device),
                A_hot=torch.empty((max(k, 1), D), dtype=torch.float32, device=self.device),
                slot_of=torch.empty(R, dtype=torch.int32, device=self.device),
                hot_row=torch.empty(max(k, 1), dtype=torch.int32, device=self.device),
                fcounter=torch.empty(R, dtype=torch.int32, device=self.device)))
        self.scratch_bytes = pk.pk_hh_scratch_bytes(self.plan, self.hh)
        self.scratch = torch.empty(self.scratch_bytes + 256, dtype=torch.uint8, device=self.device)
        self.ws, self.ws_bytes, self._shape = None, 0, None
        pk.pk_hh_init(self.plan, self.hh, torch.cuda.current_stream(self.device).cuda_stream)

    def load_table(self, t: int, values: np.ndarray) -> None:
        values = np.ascontiguousarray(values)
        if self.tables[t][2] == pk.PK_BF16:
            v = torch.from_numpy(values.view(np.int16)).view(torch.bfloat16)
        else:
            v = torch.from_numpy(values)
        self.table_view(t).copy_(v)

    def forward(self, ids, offsets, B: int, out=None):
        nnz = int(ids.shape[0])
        self._ensure_ws(B, nnz)
        if out is None:
            out = torch.empty((B, self.out_dim), dtype=torch.float32, device=self.device)
        stream = torch.cuda.current_stream(self.device).cuda_stream
        pk.pk_hh_forward(self.plan, self.hh, ids, offsets, B, nnz, out, out.stride(0), self.ws, self.ws_bytes, stream)
        return out

    def backward_update(self, grad_out, lr: float, eps: float) -> None:
        B, nnz = self._shape
        stream = torch.cuda.current_stream(self.device).cuda_stream
        pk.pk_hh_backward_update(self.plan, self.hh, grad_out, grad_out.stride(0), B, nnz, lr, eps, self.ws,
                                 self.ws_bytes, stream)

    def end_iteration(self, want_counts: bool = True):
        """Alg. 1's bookkeeping for the batch just processed; returns (queried, hits, flushed)."""
        B, nnz = self._shape
        stream = torch.cuda.current_stream(self.device).cuda_stream
        r = pk.pk_hh_end_iteration(self.plan, self.hh, self.itr, self.warmup_iters, self.flush_iters, B, nnz, self.ws,
                                   self.ws_bytes, self.scratch, self.scratch_bytes, stream, want_counts)
        self.itr += 1
        return r

    def hot_count(self, p: int) -> int:
        return pk.pk_hh_hot_count(self.plan, p)
