"""One training iteration of the embedding side, enqueued on the GPU.

Order (Algorithm 1 of the paper): filter_batch -> forward -> (gradients of the
kept samples arrive from the dense part of the model) -> backward_update ->
every K iterations: the first time capture the snapshot (the first period is
the warm-up of section 3.1.1), afterwards detect_stale with a snapshot refresh.

This class only owns buffers and issues the library calls in order; nothing
here synchronises with the host.  With overlap=True the grouping half of the
backward pass (which needs only the indices) is issued on a second stream
right after the filter, so that it runs next to the forward pass.
"""
from __future__ import annotations

from typing import Optional, Sequence

import torch

from . import binding as B


class EmbeddingStep:
    def __init__(self, weights: Sequence[torch.Tensor],
                 hot_ids: Sequence[torch.Tensor], batch: int, bag: int,
                 lr: float, threshold: float, snapshot_every: int,
                 alpha: Optional[int] = None, diagnostics: bool = True,
                 overlap: bool = False, grouped_forward: bool = False):
        self.tables = B.Tables(weights)
        self.bits = self.tables.new_bits()
        self.hot = B.HotState(self.tables, hot_ids, diagnostics=diagnostics)
        T, D = self.tables.num_tables, self.tables.dim
        dev = self.tables.device
        self.batch, self.bag = batch, bag
        self.lr, self.threshold, self.K = float(lr), float(threshold), int(snapshot_every)
        self.alpha = T * bag if alpha is None else int(alpha)
        self.skip_mask = torch.zeros(batch, dtype=torch.uint8, device=dev)
        self.kept_ids = torch.zeros(batch, dtype=torch.int32, device=dev)
        self.n_kept = torch.zeros(1, dtype=torch.int32, device=dev)
        self.idx_c = torch.zeros(T, batch, bag, dtype=torch.int32, device=dev)
        self.pooled = torch.zeros(T, batch, D, dtype=torch.float32, device=dev)
        self.ws_filter = torch.empty(
            max(256, B.ss_filter_batch_workspace_bytes(T, batch, bag)),
            dtype=torch.uint8, device=dev)
        self.ws_backward = torch.empty(
            B.ss_backward_workspace_bytes(T, batch, bag, D),
            dtype=torch.uint8, device=dev)
        self.it = 0
        self.have_snapshot = False
        self.overlap = overlap
        # forward and the grouping half of the backward pass in one call
        self.grouped_forward = grouped_forward and not overlap
        if overlap:
            self.side = torch.cuda.Stream(device=dev)      # default priority
            self.ev_filtered = torch.cuda.Event()
            self.ev_grouped = torch.cuda.Event()

    def filter_forward(self, idx: torch.Tensor) -> None:
        """Classify and compact the batch, then pool the kept samples."""
        B.ss_filter_batch(self.tables, idx, self.alpha, self.skip_mask,
                          self.kept_ids, self.n_kept, self.idx_c, self.ws_filter)
        if self.overlap:
            main = torch.cuda.current_stream()
            self.ev_filtered.record(main)
            self.side.wait_event(self.ev_filtered)
            B.ss_embbag_backward_prepare(self.tables, self.idx_c, self.n_kept,
                                         self.ws_backward, stream=self.side)
            self.ev_grouped.record(self.side)
        if self.grouped_forward:
            B.ss_embbag_forward_grouped(self.tables, self.idx_c, self.n_kept,
                                        self.pooled, self.ws_backward)
        else:
            B.ss_embbag_forward(self.tables, self.idx_c, self.n_kept, self.pooled)

    def backward(self, grad_c: torch.Tensor) -> bool:
        """grad_c: fp32 [T, B, D], row j = gradient of the j-th kept sample.
        Returns True if this iteration ended with a detect pass."""
        if self.overlap or self.grouped_forward:
            if self.overlap:
                torch.cuda.current_stream().wait_event(self.ev_grouped)
            B.ss_embbag_backward_apply(self.tables, self.batch, self.bag, grad_c,
                                       self.lr, self.ws_backward)
        else:
            B.ss_embbag_backward_update(self.tables, self.idx_c, self.n_kept, grad_c,
                                        self.lr, self.ws_backward)
        detected = False
        if (self.it + 1) % self.K == 0:
            if not self.have_snapshot:
                B.ss_detect_stale(self.tables, self.hot, 0.0, True)
                self.have_snapshot = True
            else:
                B.ss_detect_stale(self.tables, self.hot, self.threshold, True)
                detected = True
        self.it += 1
        return detected


class SnapshotRing:
    """N temporal snapshots of the hot rows (section 3.1.2 keeps N of them; the
    comparison itself is always between two, Eq. 1 / Eq. 5).

    The library compares the current rows with whichever stored snapshot it is
    handed, so a ring needs no kernel of its own: it is N snapshot buffers and a
    head.  `detect(threshold, lag)` measures the drift against the snapshot taken
    `lag` pushes ago; with lag == depth that snapshot is the oldest one, which
    the same launch then overwrites with the current rows (compare and refresh
    read the hot rows once).  depth = 1, lag = 1 is the two-snapshot scheme of
    Eq. 5 that EmbeddingStep uses.
    """

    def __init__(self, tables: B.Tables, hot_ids: Sequence[torch.Tensor], depth: int,
                 diagnostics: bool = True):
        if depth < 1:
            raise ValueError("depth >= 1")
        self.tables, self.depth = tables, depth
        self.slots = [B.HotState(tables, hot_ids, diagnostics=diagnostics)
                      for _ in range(depth)]
        self.pushed = 0                       # snapshots taken so far

    def _slot(self, lag: int) -> B.HotState:
        """The snapshot taken `lag` pushes ago (lag = 1: the newest)."""
        if not 1 <= lag <= min(self.depth, self.pushed):
            raise ValueError(f"lag {lag}: {min(self.depth, self.pushed)} snapshots are held")
        return self.slots[(self.pushed - lag) % self.depth]

    def push(self) -> None:
        """Store the current hot rows as the newest snapshot (drops the oldest)."""
        B.ss_detect_stale(self.tables, self.slots[self.pushed % self.depth], 0.0, True)
        self.pushed += 1

    def detect(self, threshold: float, lag: int = 1, push: bool = True) -> B.HotState:
        """Flag rows whose drift since `lag` snapshots ago is within the threshold;
        returns the slot whose drift / verdict buffers this call filled."""
        ref = self._slot(lag)
        fused = push and lag == self.depth    # the reference is the slot to overwrite
        B.ss_detect_stale(self.tables, ref, threshold, fused)
        if fused:
            self.pushed += 1
        elif push:
            self.push()
        return ref
