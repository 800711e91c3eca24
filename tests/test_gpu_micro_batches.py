"""D-Interleaving (Sec. III-C): the two stages of the forward pass as separate
calls, and micro-batches pipelined through the layer with the next one's dedup
on a second stream.  Micro-batches are complete steps of the layer taken one
after the other, so the oracle takes the same sequence of smaller steps."""
import numpy as np
import pytest
import torch

import synth
from oracle import pk_oracle as orc
from oracle.sparse_tables import SparseOracle
from test_gpu_parity import bits_of, close, f32_of, say

pytestmark = pytest.mark.gpu


def _filled_layer(wl, so):
    from paper_2204_04903_amd.layer import PackedEmbedding
    layer = PackedEmbedding(so.tables, so.fields)
    stream = torch.cuda.current_stream().cuda_stream
    for t, ts in enumerate(wl.tables):
        synth.fill_device(layer.table_view(t).data_ptr(), ts.rows, ts.dim, ts.dtype, wl.seed, t, stream)
    torch.cuda.synchronize()
    return layer


def test_dedup_then_pool_equals_the_one_call_forward():
    from paper_2204_04903_amd import binding as pk
    wl = synth.config(3, batch=257, row_scale=0.02, n_fields=24)
    so = SparseOracle(orc, synth, wl)
    layer = _filled_layer(wl, so)
    try:
        b = synth.make_batch(wl, 0)
        ids, offsets = torch.from_numpy(b.ids).cuda(), torch.from_numpy(b.offsets).cuda()
        one = layer.forward(ids, offsets, wl.batch)
        ctx_one = [layer.ctx(p) for p in range(layer.n_packs)]
        ws_bytes = pk.pk_workspace_bytes(layer.plan, wl.batch, b.nnz)
        ws = torch.empty(ws_bytes + 256, dtype=torch.uint8, device="cuda")
        two = torch.full_like(one, 3.0)
        stream = torch.cuda.current_stream().cuda_stream
        say("[two stages] dedup, then pool, on a second workspace")
        pk.pk_forward_dedup(layer.plan, ids, offsets, wl.batch, b.nnz, ws, ws_bytes, stream)
        pk.pk_forward_pool(layer.plan, layer.W, wl.batch, b.nnz, two, two.stride(0), ws, ws_bytes, stream)
        torch.cuda.synchronize()
        assert pk.pk_ctx_error(layer.plan, ws) == 0
        assert torch.equal(one, two)
        layer.ws, layer.ws_bytes = ws, ws_bytes          # read the second workspace's context
        for p in range(layer.n_packs):
            c = layer.ctx(p)
            for name in ("keys", "unique", "inverse", "packed_offsets", "seg_offsets"):
                assert np.array_equal(c[name], ctx_one[p][name]), name
        ref, _ = so.step(b, wl.lr, wl.eps)
        assert close(two.cpu().numpy(), ref)[0]
    finally:
        layer.close()


@pytest.mark.parametrize("idx,shrink,n_micro", [
    (3, dict(batch=333, row_scale=0.02, n_fields=40), 4),       # four packs, mean pooling, ragged micro-batches
    (5, dict(batch=64, row_scale=0.05, n_fields=12), 3),        # bf16 tables, long sequences
])
def test_pipelined_micro_batches_match_the_oracle_sequence(idx, shrink, n_micro):
    from paper_2204_04903_amd.layer import MicroBatchPipeline
    wl = synth.config(idx, **shrink)
    so = SparseOracle(orc, synth, wl)
    layer = _filled_layer(wl, so)
    bf16 = wl.tables[0].dtype == 1
    try:
        micro = []
        for b in synth.make_batches(wl, 2):
            micro += synth.split_batch(b, wl.n_fields, wl.batch, n_micro)
        say(f"[micro-batches] config {idx}: {len(micro)} micro-batches of {[m.grad_out.shape[0] for m in micro]} samples")
        dev = [(torch.from_numpy(m.ids).cuda(), torch.from_numpy(m.offsets).cuda(), torch.from_numpy(m.grad_out).cuda(),
                m.grad_out.shape[0]) for m in micro]
        outs = [torch.empty((d[3], layer.out_dim), dtype=torch.float32, device="cuda") for d in dev]
        pipe = MicroBatchPipeline(layer, max(d[3] for d in dev), max(m.nnz for m in micro))
        tickets = []
        t = pipe.submit(dev[0][0], dev[0][1], dev[0][3])
        for m in range(len(dev)):
            nxt = pipe.submit(dev[m + 1][0], dev[m + 1][1], dev[m + 1][3]) if m + 1 < len(dev) else None
            pipe.pool(t, outs[m])
            pipe.backward_update(t, dev[m][2], wl.lr, wl.eps)
            tickets.append(t)
            t = nxt
        torch.cuda.synchronize()
        assert pipe.ctx_error(tickets[-1]) == 0 and pipe.ctx_error(tickets[-2]) == 0
        for m, mb in enumerate(micro):
            ref, _ = so.step(mb, wl.lr, wl.eps, B=dev[m][3])
            ok, nbad = close(outs[m].cpu().numpy(), ref, bf16=bf16)
            assert ok, f"micro-batch {m}: {nbad} pooled outputs out of tolerance"
        for p in range(so.pl.n_packs):
            dt = int(so.pl.pack_dtype[p])
            rows = torch.from_numpy(so.keys_seen[p].astype(np.int64)).cuda()
            ok, nbad = close(f32_of(bits_of(layer.W[p][rows]), dt), f32_of(so.W_seen[p], dt), bf16=dt == 1)
            assert ok, f"pack {p}: {nbad} updated elements out of tolerance"
            ok, nbad = close(layer.A[p][rows].cpu().numpy(), so.A_seen[p])
            assert ok, f"pack {p}: {nbad} accumulator elements out of tolerance"
    finally:
        layer.close()
