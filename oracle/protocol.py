"""One training run of the embedding side, on the CPU oracle (test
infrastructure only).

Order of one iteration (Algorithm 1 of the paper: warm up, snapshot, compare
consecutive snapshots against T, drop the inputs that only reach stale
entries, train on the rest):

    filter_batch -> forward -> (gradients of the kept samples) ->
    backward_update -> every K iterations: first time capture the snapshot
    (the first period is the warm-up, section 3.1.1), afterwards detect_stale
    with a snapshot refresh.

The dense part of the model is not built; the gradient w.r.t. each pooled
vector is an input.
"""
from __future__ import annotations

from typing import List, Optional

import numpy as np

from . import detect_stale, embbag_backward_update, embbag_forward, filter_batch


class OracleRun:
    def __init__(self, weights: List[np.ndarray], hot_ids: np.ndarray,
                 lr: float, threshold: float, snapshot_every: int,
                 alpha: Optional[int] = None):
        self.W = weights                      # updated in place
        self.T = len(weights)
        self.R, self.D = weights[0].shape
        self.hot_ids = [np.ascontiguousarray(h, dtype=np.int32)
                        for h in hot_ids]
        self.lr = float(lr)
        self.threshold = float(threshold)
        self.K = int(snapshot_every)
        self.alpha = alpha                    # None -> every lookup stale
        words = (self.R + 31) // 32
        self.bits = [np.zeros(words, dtype=np.uint32) for _ in range(self.T)]
        self.snapshot: Optional[List[np.ndarray]] = None
        self.it = 0
        self.last_detect = None               # (stale_hot, drift, count)

    def step(self, idx: np.ndarray, grads: np.ndarray) -> dict:
        """idx int32 [T, B, L]; grads fp32 [T, B, D] for all B samples."""
        T, B, L = idx.shape
        alpha = T * L if self.alpha is None else self.alpha
        skip, kept, idx_c = filter_batch(self.R, self.bits, idx, alpha)
        n_kept = kept.shape[0]
        pooled = embbag_forward(self.W, idx_c, n_kept)
        g_c = np.zeros_like(grads)
        g_c[:, :n_kept] = grads[:, kept]
        embbag_backward_update(self.W, self.bits, idx_c, g_c, self.lr, n_kept)
        detected = False
        if (self.it + 1) % self.K == 0:
            if self.snapshot is None:
                self.snapshot = [np.ascontiguousarray(self.W[t][self.hot_ids[t]])
                                 for t in range(self.T)]
            else:
                self.last_detect = detect_stale(
                    self.W, self.bits, self.hot_ids, self.snapshot,
                    self.threshold, refresh=True)
                detected = True
        self.it += 1
        return dict(skip=skip, kept=kept, idx_c=idx_c, pooled=pooled,
                    n_kept=n_kept, detected=detected)
