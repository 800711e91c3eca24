"""A whole step (pk_forward + pk_backward_update) recorded in a HIP graph and replayed: the calls only
enqueue kernels on the caller's stream and on the library's side streams (forked and joined with events),
clear their scan descriptors in a kernel and allocate nothing after the first call, so a caller may capture
them.  Every replay is checked against the oracle, with eager work and synchronisations in between."""
import numpy as np
import pytest
import torch

from oracle import pk_oracle as orc
from helpers import pooled_close, small_problem, stack_tables
from test_gpu_parity import bits_of, close, f32_of, say

pytestmark = pytest.mark.gpu


FOUR_PACKS = ([(60, 4, 0), (80, 8, 0), (50, 16, 1), (40, 32, 0)], [(0, 0), (1, 1), (2, 0), (3, 1), (1, 0)])


@pytest.mark.parametrize("tables,fields,groups", [
    ([(60, 8, 0), (45, 8, 0)], [(0, 0), (1, 1), (0, 1)], 0),      # one pack
    (*FOUR_PACKS, 0),                                             # four packs on the caller's stream
    (*FOUR_PACKS, 2),                                             # ... and on two side streams, forked and joined
])
def test_a_step_replayed_from_a_graph_matches_the_oracle(tables, fields, groups):
    from paper_2204_04903_amd.layer import PackedEmbedding
    B, lr, eps = 23, 0.01, 1e-8
    pr = small_problem(501, B=B, tables=tables, fields=fields, max_len=5)
    pl = orc.plan(tables, fields)
    W = stack_tables(pl, [w.copy() for w in pr["Wt"]])
    A = [np.zeros(w.shape, np.float32) for w in W]
    layer = PackedEmbedding(tables, fields, interleave_groups=groups)
    try:
        for t, w in enumerate(pr["Wt"]):
            layer.load_table(t, w)
        ids = torch.from_numpy(pr["ids"]).cuda()
        offsets = torch.from_numpy(pr["offsets"]).cuda()
        grad = torch.from_numpy(pr["grad"]).cuda()
        out = torch.zeros((B, layer.out_dim), dtype=torch.float32, device="cuda")

        def step():
            layer.forward(ids, offsets, B, out=out)
            layer.backward_update(grad, lr, eps)

        def check(tag):
            ref_out, ctx = orc.forward(pl, W, B, pr["ids"], pr["offsets"])
            orc.backward_update(pl, W, A, ctx, B, pr["grad"], lr, eps)
            assert pooled_close(out.cpu().numpy(), ref_out, tables, fields)[0], tag
            for p in range(pl.n_packs):
                dt = int(pl.pack_dtype[p])
                assert close(f32_of(bits_of(layer.W[p]), dt), f32_of(W[p], dt), bf16=dt == 1)[0], tag
                assert close(layer.A[p].cpu().numpy(), A[p])[0], tag

        say("[graph] one eager step (the library sets up its device state on the first call)")
        step()
        torch.cuda.synchronize()
        check("eager")
        say("[graph] capture")
        side = torch.cuda.Stream()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            step()
        torch.cuda.synchronize()
        for r in range(3):
            say(f"[graph] replay {r}")
            g.replay()
            torch.cuda.synchronize()
            check(f"replay {r}")
            scratch = torch.randn(1 << 16, device="cuda").sum()       # eager work between the replays
            torch.cuda.synchronize()
            assert torch.isfinite(scratch)
    finally:
        layer.close()
