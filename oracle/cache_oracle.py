"""CPU oracle of the activation cache (test infrastructure only: tests, smoke()
and bench.py's cpu_baseline may import it; the product never does).

Follows Section 4.3 of the paper ("Caching frozen layers' activations",
Figure 6): a table keyed by sample id whose value is the activation tensor of
the last frozen layer for that sample; the activations of future mini-batches
are put in ahead of time, the forward pass reads them back by sample id, and
only the most recent mini-batches are kept (five in the paper).

Written as the description reads: one dictionary per mini-batch put in, the
mini-batches in a queue of bounded length, a lookup that goes through the
queue from the newest mini-batch to the oldest.

Readings taken where the text is silent:
  * A sample id put in again by a newer mini-batch is served from the newer
    one, and stays as long as that newer mini-batch stays.
  * A sample id that occurs twice in one mini-batch keeps its last row.
  * Negative ids are not samples: never stored, never found.
  * A lookup reports per sample whether it was found; the rows of samples that
    were not found are left as they were (the caller computes them).
"""
from __future__ import annotations

from collections import deque

import numpy as np


class CacheOracle:
    def __init__(self, window: int = 5):
        assert window >= 1
        self.batches = deque(maxlen=window)     # oldest ... newest, one dict per mini-batch

    def put(self, ids, rows):
        """ids: [n] integers; rows: [n, D] array.  The mini-batch becomes the newest one."""
        ids = np.asarray(ids).astype(np.int64)
        rows = np.asarray(rows)
        assert rows.shape[0] == ids.shape[0]
        batch = {}
        for i in range(ids.shape[0]):
            if ids[i] >= 0:
                batch[int(ids[i])] = rows[i].copy()   # a repeated id keeps its last row
        self.batches.append(batch)                    # a full queue drops its oldest mini-batch

    def get(self, ids, out):
        """Copies the cached row of every found id into out (in place); returns the hit mask [n] uint8."""
        ids = np.asarray(ids).astype(np.int64)
        hit = np.zeros(ids.shape[0], np.uint8)
        for i in range(ids.shape[0]):
            for batch in reversed(self.batches):      # newest first
                row = batch.get(int(ids[i]))
                if row is not None:
                    out[i] = row
                    hit[i] = 1
                    break
        return hit
