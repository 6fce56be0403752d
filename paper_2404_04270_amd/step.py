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

import ctypes as C
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
    critical path.

    Classifying a batch and grouping its lookups by row (ss_filter_batch,
    ss_embbag_backward_prepare) need the indices and the stale bitmaps only, not
    the weights: they can run while earlier batches are still in their forward
    and update kernels, which are bound by memory traffic and leave room on the
    compute units for these latency-bound kernels.  submit() enqueues them on a
    second stream (default priority) into a ring of buffer sets; forward() and
    backward() run on the stream that was current when the object was built.

    An event recorded on one stream and waited for on the other costs about ten
    microseconds of GPU time on this platform, a sixth of a whole step, so the
    two streams do not meet once per batch: each records an event only every
    `every` batches ("everything up to batch k is done"), and a stream waits only
    when the batch it needs is not yet covered by an event it has waited for.
    The ring holds 3 * every sets (times the number of index streams) and the
    index work may run two thirds of the ring ahead; callers that submit less far ahead still get correct results, only with
    more events (one is recorded on demand).

    Results are those of EmbeddingStep bit for bit: the only reordering is that
    index work of later batches runs before the update of earlier ones, which it
    does not read.  It does read the stale bitmaps, so batches after one that ends
    with a detect pass are held back until that pass is enqueued.
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

    class _Marks:
        """Events of one stream, each with the last batch it covers, and what each
        stream that waits on them already knows.  The events are the library's
        (device-scope release), recorded and waited for by the calling thread."""

        POOL = 66                 # 64 marks are kept, one is being recorded, one spare

        def __init__(self):
            self.recorded = []        # (covers_up_to_batch, event), ascending
            # every event this object will ever use, created before the first batch
            self.spare = [B.ss_event_create() for _ in range(self.POOL)]
            self.known = {}           # waiting stream (by position) -> batches <= this are done

        def record(self, stream, handle, covers: int) -> None:
            ev = self.spare.pop() if self.spare else B.ss_event_create()
            B.IssueQueue.record_now(ev, handle)
            self.recorded.append((covers, ev))
            if len(self.recorded) > 64:
                self.spare.append(self.recorded.pop(0)[1])

        def cover(self, waiter: int, waiting_stream, waiting_handle, batch: int) -> bool:
            """Makes waiting_stream wait until `batch` is done, if it does not know yet.
            False if no recorded event covers the batch."""
            if batch <= self.known.get(waiter, -1):
                return True
            for covers, ev in self.recorded:
                if covers >= batch:
                    B.IssueQueue.wait_now(waiting_handle, ev)
                    self.known[waiter] = covers
                    return True
            return False

        def close(self) -> None:
            for _, ev in self.recorded:
                B.ss_event_destroy(ev)
            for ev in self.spare:
                B.ss_event_destroy(ev)
            self.recorded, self.spare = [], []

    class _QueueMarks:
        """The same when the index streams are fed by the library's issue thread.

        Everything that concerns an index stream goes through the queue, so that it
        stays in order with the index work queued for that stream: the marks of an
        index stream (by_queue) are recorded by the queue and waited for by the
        training stream at once, after the host has made sure that the record has
        been issued; the marks of the training stream are recorded at once and
        waited for through the queue."""

        def __init__(self, queues, by_queue: bool, own: int = 0):
            # queues[j % len(queues)] feeds index stream j; `own` is the index stream
            # whose marks these are (by_queue), unused for the training stream's
            self.queues, self.by_queue = queues, by_queue
            self.queue = queues[own % len(queues)]
            self.recorded = []        # (covers_up_to_batch, event, ticket), ascending
            # every event this object will ever use, created before the first batch
            self.spare = [self.queue.new_event() for _ in range(PipelinedStep._Marks.POOL)]
            self.known = {}

        def record(self, stream, handle, covers: int) -> None:
            ev = self.spare.pop() if self.spare else self.queue.new_event()
            ticket = None
            if self.by_queue:
                ticket = self.queue.record_event(ev, handle)
            else:
                self.queue.record_now(ev, handle)
            self.recorded.append((covers, ev, ticket))
            if len(self.recorded) > 64:
                # 64 marks back: issued and waited for long ago
                self.spare.append(self.recorded.pop(0)[1])

        def cover(self, waiter: int, waiting_stream, waiting_handle, batch: int) -> bool:
            if batch <= self.known.get(waiter, -1):
                return True
            for covers, ev, ticket in self.recorded:
                if covers >= batch:
                    if self.by_queue:
                        self.queue.wait_issued(ticket)     # a wait for an unrecorded event is a no-op
                        self.queue.wait_now(waiting_handle, ev)
                    else:         # the waiter is index stream `waiter`: through its queue
                        self.queues[waiter % len(self.queues)].wait_event(ev, waiting_handle)
                    self.known[waiter] = covers
                    return True
            return False

    RING_BYTES = 96 << 20     # what the grouped lists of the whole ring may take

    @classmethod
    def auto_every(cls, T: int, batch: int, bag: int, n_side: int) -> int:
        """Batches between two cross-stream events: 8 (an event pair costs about
        10 us of GPU time), or fewer when a ring of 3 * every * n_side sets would not
        fit the 256 MB memory-side cache next to the step's own traffic: a grouped
        list written by the index stream should still be there when the update
        kernel reads it (measured at 8 tables x 81920 lookups: 99.9 / 102.1 / 104.0
        us per step for every = 2 / 4 / 8)."""
        # keys and payloads, two buffers each, padded to 2048 lookups per table
        per_set = 16 * T * ((batch * bag + 2047) // 2048) * 2048
        every = 8
        while every > 2 and 3 * every * n_side * per_set > cls.RING_BYTES:
            every //= 2
        return every

    @staticmethod
    def auto_streams(batch: int, bag: int, num_tables: int = 8) -> int:
        """Index streams.  One while a table has at most 16384 lookups per batch (a
        second one costs 1-2 us there).  Beyond that the grouping is a global radix
        sort, a chain of six small launches per batch that lasts about as long as
        the training kernels: two such chains side by side keep the index work ahead
        (8 tables x 81920 lookups: 88 against 104 us per step once the hot rows are
        frozen, 101 either way before).  Three when those launches are tiny (fewer
        than 128 workgroups over all tables): the chain then lasts almost three
        times as long as the training kernels (one table x 65536 lookups: 77 / 44 /
        38 us per step with one / two / three streams, 35 us with three and the
        issue thread; four are slower again)."""
        lookups = batch * bag
        if lookups <= 16384:
            return 1
        return 3 if num_tables * ((lookups + 2047) // 2048) < 128 else 2

    @staticmethod
    def auto_issue_thread(T: int, batch: int, bag: int, n_side: int) -> bool:
        """Whether the index work is enqueued by the library's issue thread: where a
        batch is a string of launches at their latency floor, so that the host, not
        the GPU, sets the pace.  That is the three-stream case above, and batches of
        at most 65536 lookups over all tables (26 tables x 2048 lookups: 21 against
        28 us per step).  Larger shapes gain nothing from it (26 x 8192: 49.8 us
        either way).  With three index streams or more each stream gets a thread of
        its own (one table x 65536 lookups: 29.7 us per step either way while nothing
        is stale, 23.5 against 29.7 us once 76 % of the samples are skipped and the
        training kernels are short)."""
        return n_side >= 3 or T * batch * bag <= 65536

    def __init__(self, weights: Sequence[torch.Tensor],
                 hot_ids: Sequence[torch.Tensor], batch: int, bag: int,
                 lr: float, threshold: float, snapshot_every: int,
                 alpha: Optional[int] = None, diagnostics: bool = True,
                 every: Optional[int] = None, index_streams: Optional[int] = None,
                 issue_thread=None):
        """every: batches between two cross-stream events (None: auto_every);
        index_streams: None = auto_streams; issue_thread: None = auto_issue_thread,
        False / 0 = the calling thread enqueues everything, True = the library's issue
        threads (one, or one per index stream from three streams on), an int = that
        many threads (at most one per index stream)."""
        self.tables = B.Tables(weights)
        self.bits = self.tables.new_bits()
        self.hot = B.HotState(self.tables, hot_ids, diagnostics=diagnostics)
        T, D = self.tables.num_tables, self.tables.dim
        dev = self.tables.device
        self.batch, self.bag = batch, bag
        self.lr, self.threshold, self.K = float(lr), float(threshold), int(snapshot_every)
        self.alpha = T * bag if alpha is None else int(alpha)
        self.pooled = torch.zeros(T, batch, D, dtype=torch.float32, device=dev)
        if index_streams is None:
            index_streams = self.auto_streams(batch, bag, T)
        n_side = max(1, int(index_streams))
        if every is None:
            every = self.auto_every(T, batch, bag, n_side)
        self.every = max(1, int(every))
        # Three groups of `every` sets, of which two may be in use ahead of the batch
        # being trained on: the set a new batch takes over was then last used at least
        # `every` batches ago, which an event recorded by the training stream already
        # covers, and the training stream finds an event of the index stream that
        # covers the batch it starts.  With less slack each stream would have to
        # record an extra event for almost every batch.
        self.sets = [self._Set(T, batch, bag, D, dev) for _ in range(3 * self.every * n_side)]
        for s in self.sets:       # arguments marshalled once (the bitmaps are attached)
            s.filter = B.prepared_filter_batch(self.tables, batch, bag, self.alpha, s.skip_mask,
                                               s.kept_ids, s.n_kept, s.idx_c, s.ws_filter)
            s.group = B.prepared_backward_prepare(self.tables, s.idx_c, s.n_kept, s.ws_backward)
            s.lookup = B.prepared_forward(self.tables, s.idx_c, s.n_kept, self.pooled)
            s.update = B.prepared_backward_apply(self.tables, batch, bag, self.lr,
                                                 s.ws_backward)
        # Index streams (default priority); batch k goes to stream k mod n.  More than
        # one pays when the index work of a batch takes longer than its training
        # kernels (one huge table: the grouping is a chain of small launches).
        self.sides = [torch.cuda.Stream(device=dev) for _ in range(max(1, int(index_streams)))]
        self.side_handles = [B.stream_handle(st) for st in self.sides]
        # the training stream is the one current now (asking torch for it on every
        # call costs more host time than the launch it is needed for)
        self.main = torch.cuda.current_stream(dev)
        self.main_handle = B.stream_handle(self.main)
        # With issue_thread the index work is enqueued by a host thread of the library
        # (ss_issue_queue): a kernel launch costs the host about 3 us, and where the
        # kernels of a batch are short (one huge table; hot rows frozen) one host thread
        # cannot enqueue eleven of them as fast as the GPU finishes them.
        if issue_thread is None:
            issue_thread = self.auto_issue_thread(T, batch, bag, n_side)
        # One issue thread per index stream when there are three or more of them (the
        # launches of a batch are then so short that a single thread enqueueing the
        # index work of all streams sets the pace); an int asks for that many.
        n_threads = int(issue_thread) if issue_thread else 0
        if issue_thread is True:
            n_threads = n_side if n_side >= 3 else 1
        n_threads = min(n_threads, n_side)
        self.queues = [B.IssueQueue() for _ in range(n_threads)]
        self.queue = self.queues[0] if self.queues else None
        self._last_tickets = [0] * n_threads
        if self.queue is not None:
            for i, s in enumerate(self.sets):     # set i always serves index stream i % n_side
                s.index = self.queues[(i % n_side) % n_threads].prepared_index_batch(
                    self.tables, batch, bag, self.alpha, s.skip_mask, s.kept_ids, s.n_kept,
                    s.idx_c, s.ws_filter, s.ws_backward)
            self.indexed = [self._QueueMarks(self.queues, True, j) for j in range(n_side)]
            self.trained = self._QueueMarks(self.queues, False)
        else:
            # index work of this stream's batches done up to batch ... (one per index stream)
            self.indexed = [self._Marks() for _ in self.sides]
            self.trained = self._Marks()      # main stream: update done up to batch ...
        self.submitted = 0        # batches handed to submit()
        self.issued = 0           # ... whose index work is enqueued
        self.forwarded = 0        # batches whose forward() was enqueued
        self.it = 0               # batches whose backward() was enqueued
        self.held_back = []       # batches waiting for a detect pass before them
        self.last_detect = -1     # last batch that ended with a detect pass
        self.have_snapshot = False

    def flush(self) -> None:
        """With issue_thread: returns once every submitted batch whose index work was
        handed to the issue thread has been enqueued on its stream, so that a device
        synchronisation after it covers that work.  A no-op otherwise."""
        for q, ticket in zip(self.queues, self._last_tickets):
            if ticket:
                q.wait_issued(ticket)

    def close(self) -> None:
        """Stops the issue threads (if any); the object must not be used afterwards."""
        if self.queues:
            for q in self.queues:       # every queued job issued, every thread ended ...
                q.stop()
            for q in self.queues:       # ... before the events those jobs name go
                q.close()
            self.queues, self.queue = [], None
        else:
            for m in self.indexed + [self.trained]:
                m.close()

    # what the batch in flight produced
    def _cur(self) -> "PipelinedStep._Set":
        return self.sets[(self.forwarded - 1) % len(self.sets)]

    skip_mask = property(lambda self: self._cur().skip_mask)
    kept_ids = property(lambda self: self._cur().kept_ids)
    n_kept = property(lambda self: self._cur().n_kept)
    idx_c = property(lambda self: self._cur().idx_c)

    def _boundary(self, k: int) -> bool:
        return (k + 1) % self.K == 0

    def _boundary_in(self, lo: int, hi: int) -> bool:
        """Does a batch in [lo, hi) end with a snapshot / detect pass?"""
        first = (lo // self.K + 1) * self.K - 1          # first such batch at or after lo
        return first < hi

    def room(self) -> int:
        """How many more batches submit() takes right now."""
        return 2 * self.every * len(self.sides) - (self.submitted - self.it)

    def submit(self, idx: torch.Tensor, ready: Optional[torch.cuda.Event] = None) -> None:
        """Index work of the next batch.

        idx must stay untouched until the batch's backward() has run.  If idx is
        still being produced on some stream, pass the event recorded after its
        producer; without one it is taken to be complete already.
        """
        if self.room() <= 0:
            raise RuntimeError("PipelinedStep: too far ahead (see room())")
        k = self.submitted
        self.submitted += 1
        # a boundary batch before this one that has not had its backward() yet?
        if self.held_back or self._boundary_in(self.it, k):
            self.held_back.append((idx, ready))
            self._drain(2)
            return
        self._issue(k, idx, ready)

    def _drain(self, limit: int) -> None:
        """Enqueues the index work of up to `limit` batches that were held back, as
        far as no detect pass is still due before them.  A few at a time: enqueueing
        all sixteen at once after a detect pass kept the calling thread busy for
        180 us, during which the training stream ran dry."""
        while limit > 0 and self.held_back and not self._boundary_in(self.it, self.issued):
            idx, ready = self.held_back.pop(0)
            self._issue(self.issued, idx, ready)
            limit -= 1

    def _issue(self, k: int, idx: torch.Tensor, ready: Optional[torch.cuda.Event]) -> None:
        assert k == self.issued
        s = self.sets[k % len(self.sets)]
        j = k % len(self.sides)
        side, handle = self.sides[j], self.side_handles[j]
        if ready is not None:
            if self.queue is not None:
                self.queues[j % len(self.queues)].wait_event(C.c_void_p(ready.cuda_event), handle)
            else:
                side.wait_event(ready)
        # the set's previous batch must be over, and so must the last detect pass
        need = max(k - len(self.sets), self.last_detect)
        if need >= 0 and not self.trained.cover(j, side, handle, need):
            self.trained.record(self.main, self.main_handle, self.it - 1)
            assert self.trained.cover(j, side, handle, need)
        s.idx = idx
        if self.queue is not None:
            self._last_tickets[j % len(self.queues)] = s.index(idx, handle)
        else:
            s.filter(idx, handle)
            s.group(handle)
        self.issued += 1
        # every `every`-th batch of this stream, and a batch the training stream is about
        # to ask for (right after a detect pass, or a caller that submits just in time):
        # an event recorded later, on demand, would also cover, and so wait for, whatever
        # index work has been enqueued behind this batch by then (measured after a detect
        # pass at 26 tables: the next step took 155 us instead of 50)
        if (k // len(self.sides) + 1) % self.every == 0 or k - self.it < self.every * len(self.sides):
            self.indexed[j].record(side, handle, k)

    def forward(self) -> torch.Tensor:
        """Pooled lookup of the oldest submitted batch; returns the pooled tensor."""
        k = self.forwarded
        if k == self.it and k >= self.issued:
            self._drain(1)                 # the batch may be waiting among the held ones
        if k != self.it or k >= self.issued:
            raise RuntimeError("PipelinedStep: forward() needs a submitted batch and the "
                               "previous batch finished")
        s = self.sets[k % len(self.sets)]
        j = k % len(self.sides)
        if not self.indexed[j].cover(0, self.main, self.main_handle, k):
            # on demand: this stream's last issued batch is the last one congruent to j
            last = self.issued - 1 - (self.issued - 1 - j) % len(self.sides)
            self.indexed[j].record(self.sides[j], self.side_handles[j], last)
            assert self.indexed[j].cover(0, self.main, self.main_handle, k)
        self.forwarded += 1
        s.lookup(self.main_handle)
        return self.pooled

    def backward(self, grad_c: torch.Tensor) -> bool:
        """Update with the gradients of the kept samples; True after a detect pass."""
        if self.forwarded != self.it + 1:
            raise RuntimeError("PipelinedStep: backward() follows forward()")
        s = self._cur()
        main = self.main
        s.update(grad_c, self.main_handle)
        detected = False
        k = self.it
        if self._boundary(k):
            if not self.have_snapshot:
                B.ss_detect_stale(self.tables, self.hot, 0.0, True, stream=main)
                self.have_snapshot = True
            else:
                B.ss_detect_stale(self.tables, self.hot, self.threshold, True, stream=main)
                detected = True
            self.last_detect = k
        self.it += 1
        if self.it % self.every == 0:
            self.trained.record(main, self.main_handle, k)
        # batches that waited for a detect pass (this one's, or an earlier one's)
        self._drain(2)
        return detected
