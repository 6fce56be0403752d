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


class PipelinedStep:
    """The same iteration with the index work of the coming batches taken off the
    critical path: a thin front of the library's ss_step (csrc/step.hip), which
    owns the index streams, the events and the issue threads and decides what is
    enqueued where and when.  This class allocates the ring of buffer sets and the
    pooled output, and marshals arguments.

    Classifying a batch and grouping its lookups by row (ss_filter_batch,
    ss_embbag_backward_prepare) need the indices and the stale bitmaps only, not
    the weights: they run on index streams while earlier batches are still in their
    lookup and update kernels.  submit() hands over the indices of a coming batch,
    as far ahead as room() allows; forward() and backward() run on the stream that
    was current when the object was built.  Results are those of EmbeddingStep bit
    for bit.
    """

    class _Set:
        def __init__(self, T, batch, bag, D, dev):
            self.skip_mask = torch.zeros(batch, dtype=torch.uint8, device=dev)
            self.kept_ids = torch.zeros(batch, dtype=torch.int32, device=dev)
            self.n_kept = torch.zeros(1, dtype=torch.int32, device=dev)
            self.idx_c = torch.zeros(T, batch, bag, dtype=torch.int32, device=dev)
            self.ws_filter = torch.empty(
                max(256, B.ss_filter_batch_workspace_bytes(T, batch, bag)),
                dtype=torch.uint8, device=dev)
            self.ws_backward = torch.empty(
                B.ss_backward_workspace_bytes(T, batch, bag, D), dtype=torch.uint8, device=dev)
            self.idx = None                        # keeps the index tensor alive
            self.ready = None                      # ... and the event it was handed over with

    @staticmethod
    def auto_every(T: int, batch: int, bag: int, n_side: int) -> int:
        """Batches between two cross-stream events, as the library chooses them."""
        return B.ss_step_plan_for(T, batch, bag, 0, n_side, 0).every

    @staticmethod
    def auto_streams(batch: int, bag: int, num_tables: int = 8, dim: int = 0) -> int:
        """Index streams, as the library chooses them for the shape."""
        return B.ss_step_plan_for(num_tables, batch, bag, 1, 0, 0, dim=dim).index_streams

    def __init__(self, weights: Sequence[torch.Tensor],
                 hot_ids: Sequence[torch.Tensor], batch: int, bag: int,
                 lr: float, threshold: float, snapshot_every: int,
                 alpha: Optional[int] = None, diagnostics: bool = True,
                 every: Optional[int] = None, index_streams: Optional[int] = None,
                 issue_thread=None, host_wait_us: Optional[int] = None):
        """every: batches between two cross-stream events; index_streams; issue_thread:
        False / 0 = the calling thread enqueues everything, True = the library's issue
        threads (one, or one per index stream from three streams on), an int = that
        many threads (at most one per index stream); host_wait_us: how long forward()
        may keep the calling thread polling for a batch's index work (0: never).  None
        leaves a choice to the library (ss_step_plan_for)."""
        self.tables = B.Tables(weights)
        self.bits = self.tables.new_bits()
        self.hot = B.HotState(self.tables, hot_ids, diagnostics=diagnostics)
        T, D = self.tables.num_tables, self.tables.dim
        dev = self.tables.device
        self.batch, self.bag = batch, bag
        self.lr, self.threshold, self.K = float(lr), float(threshold), int(snapshot_every)
        self.alpha = T * bag if alpha is None else int(alpha)
        self.pooled = torch.zeros(T, batch, D, dtype=torch.float32, device=dev)
        streams = B.ss_step_plan_for(T, batch, bag, 1, int(index_streams or 0), 0,
                                     dim=D).index_streams
        if issue_thread is None:
            threads = -1
        elif issue_thread is True:
            threads = streams if streams >= 3 else 1
        else:
            threads = min(int(issue_thread), streams)
        plan = B.ss_step_plan_for(T, batch, bag, int(every or 0), streams, threads,
                                  -1 if host_wait_us is None else int(host_wait_us), dim=D)
        self.plan = plan
        self.every = plan.every
        self.sets = [self._Set(T, batch, bag, D, dev) for _ in range(plan.num_sets)]
        self.sides = [None] * plan.index_streams        # the library's own streams
        self.queues = [None] * plan.issue_threads       # ... and issue threads
        # the training stream is the one current now
        self.main = torch.cuda.current_stream(dev)
        self._step = B.ss_step_create(self.tables, batch, bag, self.alpha, self.lr,
                                      self.threshold, self.K, self.hot, plan, self.sets,
                                      self.pooled, stream=self.main)
        self._cur_set = 0
        self.submitted = 0        # batches handed to submit()
        self.forwarded = 0        # batches whose forward() was enqueued
        self.it = 0               # batches whose backward() was enqueued

    def flush(self) -> None:
        """Returns once every submitted batch whose index work was handed to an issue
        thread has been enqueued on its stream, so that a device synchronisation after
        it covers that work.  A no-op without issue threads."""
        B.ss_step_flush(self._step)

    def close(self) -> None:
        """Ends the issue threads, waits for the index streams and releases the
        library's streams and events; the object must not be used afterwards."""
        if self._step is not None:
            B.ss_step_destroy(self._step)
            self._step = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # what the batch in flight produced
    def _cur(self) -> "PipelinedStep._Set":
        return self.sets[self._cur_set]

    skip_mask = property(lambda self: self._cur().skip_mask)
    kept_ids = property(lambda self: self._cur().kept_ids)
    n_kept = property(lambda self: self._cur().n_kept)
    idx_c = property(lambda self: self._cur().idx_c)

    def counters(self) -> dict:
        """Diagnosis: lookups, wait commands of the training stream, host polls."""
        return B.ss_step_counters(self._step)

    def room(self) -> int:
        """How many more batches submit() takes right now."""
        return B.ss_step_room(self._step)

    def submit(self, idx: torch.Tensor, ready: Optional[torch.cuda.Event] = None) -> None:
        """Index work of the next batch.

        idx (int32 [T, B, L], contiguous, on the device) must stay untouched until the
        batch's backward() has run.  If idx is still being produced on some stream,
        pass the event recorded after its producer; without one it is taken to be
        complete already.
        """
        if self.room() <= 0:
            raise RuntimeError("PipelinedStep: too far ahead (see room())")
        B.ss_step_submit(self._step, idx, ready)
        # the wait for `ready` may be enqueued later than this call (issue thread, or a
        # batch held back behind a detect pass): the event lives as long as the set
        # holds this batch
        st = self.sets[self.submitted % len(self.sets)]
        st.idx, st.ready = idx, ready
        self.submitted += 1

    def forward(self) -> torch.Tensor:
        """Pooled lookup of the oldest submitted batch; returns the pooled tensor."""
        if self.forwarded != self.it or self.forwarded >= self.submitted:
            raise RuntimeError("PipelinedStep: forward() needs a submitted batch and the "
                               "previous batch finished")
        self._cur_set = B.ss_step_forward(self._step)
        self.forwarded += 1
        return self.pooled

    def backward(self, grad_c: torch.Tensor) -> bool:
        """Update with the gradients of the kept samples; True after a detect pass."""
        if self.forwarded != self.it + 1:
            raise RuntimeError("PipelinedStep: backward() follows forward()")
        detected = B.ss_step_backward(self._step, grad_c)
        self.it += 1
        return detected
