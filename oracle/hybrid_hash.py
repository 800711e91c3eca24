"""CPU oracle of HybridHash (Sec. III-D, Alg. 1): which embedding rows live in the
Hot-storage, which queries hit it, and when it is refreshed.

TEST INFRASTRUCTURE ONLY (like everything under oracle/).  Plain Python / numpy,
one pack of rows at a time; it follows the algorithm's steps in the paper's order:

  warm-up (itr < warmup_iters): every queried ID bumps FCounter and is served by the
      Cold-storage;
  afterwards: an ID found in the Hot-storage is served from there, the others from
      the Cold-storage; every queried ID bumps FCounter; when itr is a multiple of
      flush_iters the Hot-storage is reloaded with the top-k IDs of FCounter.

Readings where the paper is silent:
  - "IDs" are the IDs that reach the store, i.e. the distinct IDs of the batch (Gather
    runs after Unique, Sec. II-D; the paper's hit ratio is that of the unique IDs of a
    batch, Sec. IV-C): FCounter counts iterations in which a row was queried.
  - top-k: by count, larger first; equal counts by row, smaller first; rows never
    queried do not enter, so fewer than k rows may be hot.
  - the selection compares counts up to COUNT_CAP = 65535: rows queried in that many
    iterations or more count as equally hot (and are told apart by row).  FCounter
    itself keeps counting.
  - the Hot-storage is where a hot row is read AND updated, so before a reload the
    rows it holds are written back to the Cold-storage.
The cache is transparent: it never changes a value the layer computes.
"""
from __future__ import annotations

import numpy as np


COUNT_CAP = 65535


class HybridHashOracle:
    def __init__(self, n_rows: int, k: int, warmup_iters: int, flush_iters: int):
        self.n_rows, self.k = int(n_rows), int(k)
        self.warmup_iters, self.flush_iters = int(warmup_iters), int(flush_iters)
        self.fcounter = np.zeros(self.n_rows, np.int64)
        self.hot = np.zeros(0, np.int64)          # rows in the Hot-storage, ascending

    def top_k(self) -> np.ndarray:
        """Rows of the k largest positive counts; ties go to the smaller row.  Ascending rows."""
        rows = np.nonzero(self.fcounter)[0]
        order = sorted(rows.tolist(), key=lambda r: (-min(int(self.fcounter[r]), COUNT_CAP), r))
        return np.array(sorted(order[:self.k]), np.int64)

    def iteration(self, ids, itr: int):
        """One call of Alg. 1 with the distinct row IDs of a batch.  Returns (hit mask per ID,
        whether the Hot-storage was reloaded)."""
        ids = np.asarray(ids, np.int64)
        assert len(np.unique(ids)) == len(ids)
        if itr < self.warmup_iters:
            self.fcounter[ids] += 1
            return np.zeros(len(ids), bool), False
        hit = np.isin(ids, self.hot)
        self.fcounter[ids] += 1
        flushed = False
        if itr % self.flush_iters == 0:
            self.hot = self.top_k()
            flushed = True
        return hit, flushed
