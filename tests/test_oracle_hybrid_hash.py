"""Pins of the HybridHash oracle (Sec. III-D, Alg. 1) against things other than itself."""
import numpy as np

from oracle.hybrid_hash import HybridHashOracle


def test_warm_up_serves_everything_from_cold_storage_and_counts():
    h = HybridHashOracle(n_rows=10, k=3, warmup_iters=2, flush_iters=1)
    for itr in range(2):
        hit, flushed = h.iteration([1, 5, 7], itr)
        assert not hit.any() and not flushed
    assert h.fcounter.tolist() == [0, 2, 0, 0, 0, 2, 0, 2, 0, 0]
    assert len(h.hot) == 0


def test_hand_worked_sequence():
    # k = 2, warm-up 1 iteration, reload every 2nd iteration; worked by hand from Alg. 1
    h = HybridHashOracle(n_rows=8, k=2, warmup_iters=1, flush_iters=2)
    assert h.iteration([0, 3, 4], 0)[1] is False            # warm-up: counts 0:1 3:1 4:1
    hit, fl = h.iteration([3, 4, 6], 1)                       # 1 % 2 != 0: no reload, Hot-storage still empty
    assert hit.tolist() == [False, False, False] and not fl   # counts 0:1 3:2 4:2 6:1
    hit, fl = h.iteration([3, 6], 2)                          # counts 3:3 4:2 6:2 0:1 -> reload: {3, then 4 (tie 4 < 6)}
    assert hit.tolist() == [False, False] and fl
    assert h.hot.tolist() == [3, 4]
    hit, fl = h.iteration([4, 6, 7], 3)                       # served: 4 hot, 6 and 7 cold; no reload
    assert hit.tolist() == [True, False, False] and not fl    # counts 3:3 4:3 6:3 7:1 0:1
    hit, fl = h.iteration([6], 4)                             # 6 still cold when queried; counts 6:4 -> reload {6, 3 (tie 3 < 4)}
    assert hit.tolist() == [False] and fl
    assert h.hot.tolist() == [3, 6]


def test_top_k_against_plain_sorting_and_edge_cases():
    rng = np.random.default_rng(3)
    h = HybridHashOracle(n_rows=500, k=40, warmup_iters=0, flush_iters=1)
    h.fcounter[:] = rng.integers(0, 6, size=500)              # many ties, many zeros
    exp = sorted(sorted((r for r in range(500) if h.fcounter[r] > 0), key=lambda r: (-h.fcounter[r], r))[:40])
    assert h.top_k().tolist() == exp
    h.k = 10_000                                              # more room than queried rows: all of them, none of the others
    assert h.top_k().tolist() == [r for r in range(500) if h.fcounter[r] > 0]
    h.fcounter[:] = 1
    h.k = 7                                                   # all equal: the smallest rows
    assert h.top_k().tolist() == list(range(7))


def test_hit_ratio_grows_with_hot_storage_on_skewed_queries():
    # the shape of Tab. "cache": a larger Hot-storage hits more of a batch's distinct IDs, with shrinking gains
    rng = np.random.default_rng(11)
    ratios = []
    for k in (50, 200, 800, 3200):
        h = HybridHashOracle(n_rows=20000, k=k, warmup_iters=20, flush_iters=10)
        hits = tot = 0
        for itr in range(60):
            ids = np.unique((rng.zipf(1.2, size=2000) - 1) % 20000)
            hit, _ = h.iteration(ids, itr)
            if itr >= 30:
                hits += int(hit.sum()); tot += len(ids)
        ratios.append(hits / tot)
    assert ratios == sorted(ratios) and ratios[0] > 0.05 and ratios[-1] < 1.0
    gains = np.diff(ratios)
    assert gains[-1] < gains[0] * 4 and ratios[-1] - ratios[0] > 0.2


def test_selection_compares_counts_up_to_the_cap():
    # counts of 65535 and more are equally hot in the selection; the smaller row wins among them
    o = HybridHashOracle(n_rows=10, k=3, warmup_iters=0, flush_iters=1)
    o.fcounter[:] = [5, 70000, 65535, 65534, 0, 900000, 65535, 1, 2, 3]
    assert list(o.top_k()) == [1, 2, 5]            # rows 1, 2, 5, 6 sit at the cap: rows 1, 2, 5 are the smallest
    o.k = 5
    assert list(o.top_k()) == [1, 2, 3, 5, 6]      # then the cap's last row, then 65534
    o.fcounter[1] = 65534                          # below the cap the true count decides again
    o.k = 3
    assert list(o.top_k()) == [2, 5, 6]
