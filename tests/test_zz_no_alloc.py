"""pk_forward_static, the forward pass for callers that cannot allocate, against pk_forward: the same
kernels with the workspace in the library's static device array.  Two calls in a row, the second with a
smaller input (the array keeps the first call's contents), on the one-launch path and on the partitioned
one; then a call the array cannot hold, which must be refused."""
import numpy as np
import pytest
import torch

from helpers import small_problem

pytestmark = pytest.mark.gpu


def _run_pair(layer, pr, B):
    from paper_2204_04903_amd import binding as pk
    ids = torch.from_numpy(pr["ids"]).cuda()
    offsets = torch.from_numpy(pr["offsets"]).cuda()
    nnz = int(ids.shape[0])
    ref = layer.forward(ids, offsets, B).clone()
    got = torch.full((B, layer.out_dim), 3.0, dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    pk.pk_forward_static(layer.plan, layer.W, ids, offsets, B, nnz, got, got.stride(0), stream)
    torch.cuda.synchronize()
    assert layer.error_word() == 0
    return ref.cpu().numpy(), got.cpu().numpy()


@pytest.mark.parametrize("debug", [0, 2])          # 0: one launch; 2: occurrences partitioned by slice
def test_static_forward_equals_forward_twice_the_second_call_smaller(debug):
    from paper_2204_04903_amd.layer import PackedEmbedding
    tables = [(5, 8, 0), (300, 64, 0), (40000, 8, 0), (3, 64, 1), (50000, 32, 0), (40, 32, 0)]
    fields = [(0, 0), (1, 1), (2, 0), (3, 1), (4, 0), (5, 1), (2, 1), (4, 1), (0, 1)]
    big = small_problem(900, B=1500, tables=tables, fields=fields, max_len=12)
    small = small_problem(901, B=200, tables=tables, fields=fields, max_len=5)
    layer = PackedEmbedding(tables, fields, debug=debug)
    try:
        for t, w in enumerate(big["Wt"]):
            layer.load_table(t, w)
        for name, pr in (("first", big), ("second, smaller", small)):
            print(f"[static] {name}: B={pr['B']} nnz={len(pr['ids'])} debug={debug}", flush=True)
            ref, got = _run_pair(layer, pr, pr["B"])
            assert np.array_equal(ref.view(np.uint32), got.view(np.uint32)), name      # the same kernels: the same bits
    finally:
        layer.close()


def test_static_forward_refuses_what_the_static_array_cannot_hold():
    from paper_2204_04903_amd import binding as pk
    from paper_2204_04903_amd.layer import PackedEmbedding
    tables, fields = [(1000, 8, 0)], [(0, 0)]
    layer = PackedEmbedding(tables, fields)
    try:
        B = 1 << 21                                   # 2 M one-hot bags: the workspace alone exceeds 32 MiB
        assert pk.pk_workspace_bytes(layer.plan, B, B) > (32 << 20)
        ids = torch.zeros(B, dtype=torch.int64, device="cuda")
        offsets = torch.arange(B + 1, dtype=torch.int32, device="cuda")
        out = torch.zeros((B, 8), dtype=torch.float32, device="cuda")
        with pytest.raises(pk.PkError) as e:
            pk.pk_forward_static(layer.plan, layer.W, ids, offsets, B, B, out, 8, torch.cuda.current_stream().cuda_stream)
        assert e.value.status == pk.PK_EWORKSPACE
    finally:
        layer.close()
