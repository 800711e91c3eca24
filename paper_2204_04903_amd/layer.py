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
