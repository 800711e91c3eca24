"""Partition (Sec. II-D; Sec. III-B fuses it with Unique) on one GPU: the distinct keys of every pack,
regrouped by owner through the C ABI, against the oracle's plain loop -- bit for bit."""
from __future__ import annotations

import numpy as np
import pytest
import torch

import synth
from oracle import pk_oracle as orc
from helpers import small_problem

pytestmark = pytest.mark.gpu


def check_partition(layer, pl, uniques, owners):
    for p in range(pl.n_packs):
        uq = uniques[p]
        for n in owners:
            k, i, o = layer.partition(p, n)
            torch.cuda.synchronize()
            rk, ri, ro = orc.partition(uq, n)
            U = len(uq)
            o = o.cpu().numpy()
            assert np.array_equal(o, ro), f"pack {p}, {n} owners: offsets"
            assert np.array_equal(k.cpu().numpy().view(np.uint32)[:U].astype(np.uint64), rk), f"pack {p}, {n} owners: keys"
            assert np.array_equal(i.cpu().numpy()[:U], ri), f"pack {p}, {n} owners: index"


@pytest.mark.parametrize("case", ["small", "medium", "medium, dedup by slices in several launches", "empty"])
def test_partition_matches_the_oracle(case):
    from paper_2204_04903_amd.layer import PackedEmbedding
    if case == "small":
        tables = [(50, 8, 0), (1000, 16, 0), (300, 8, 1)]
        fields = [(0, 0), (1, 1), (1, 0), (2, 0)]
        B, max_len = 37, 5
    elif case.startswith("medium"):        # several chunks of 2048 distinct keys and a ragged last one
        tables = [(200_000, 8, 0), (70_001, 8, 0), (90, 4, 0)]
        fields = [(0, 0), (0, 1), (1, 0), (2, 0)]
        B, max_len = 3000, 9
    else:
        tables = [(64, 4, 0)]
        fields = [(0, 0)]
        B, max_len = 4, 0
    pr = small_problem(11, B=B, tables=tables, fields=fields, max_len=max_len)
    pl = orc.plan(tables, fields)
    layer = PackedEmbedding(tables, fields, debug=2 if "launches" in case else 0)
    try:
        ids = torch.from_numpy(pr["ids"]).cuda()
        offsets = torch.from_numpy(pr["offsets"]).cuda()
        layer.forward(ids, offsets, B)
        torch.cuda.synchronize()
        uniques = []
        for p in range(pl.n_packs):
            key, _ = orc.pack_keys(pl, p, B, pr["ids"], pr["offsets"])
            uniques.append(orc.unique(key)[0])
        check_partition(layer, pl, uniques, (1, 2, 3, 8, 64))
    finally:
        layer.close()


def test_partition_rejects_bad_arguments():
    from paper_2204_04903_amd import binding as pk
    from paper_2204_04903_amd.layer import PackedEmbedding
    layer = PackedEmbedding([(64, 4, 0)], [(0, 0)])
    try:
        pr = small_problem(3, B=8, tables=[(64, 4, 0)], fields=[(0, 0)], max_len=3)
        layer.forward(torch.from_numpy(pr["ids"]).cuda(), torch.from_numpy(pr["offsets"]).cuda(), 8)
        with pytest.raises(pk.PkError):
            layer.partition(0, 65)
        with pytest.raises(pk.PkError):
            layer.partition(1, 8)
    finally:
        layer.close()
