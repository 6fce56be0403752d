"""Host logic of PipelinedStep, checked on the CPU against a model of streams.

PipelinedStep spreads the calls of a batch over several streams and lets them meet
through events as rarely as it can.  A missing wait there would not fail loudly on
the GPU: it would be a race that the parity tests only catch when the timing
happens to be bad.  Here the library binding and the stream / event objects are
replaced by recorders, PipelinedStep is driven through a few hundred batches, and
the recorded program (per stream: kernels, event records, event waits) is then
executed by a scheduler that picks runnable streams at random.  Whatever order it
picks, every kernel must find its inputs complete:

  filter(k)   after update(k - ring) (the buffer set's previous batch) and after the
              detect pass of the last boundary batch before k (it reads the bitmaps);
  group(k)    after filter(k);
  lookup(k)   after filter(k) and update(k - 1);
  update(k)   after group(k) and lookup(k);
  detect(b)   after update(b);

and the program must run to its end (no wait for an event nobody records).  A wait
takes the event's most recent record at the moment the wait is ENQUEUED, as HIP
does; with issue threads, jobs reach their stream late and in bursts, which is what
ss_issue_wait() is for.  Two planted mistakes (a cover() that claims everything is
known; an ss_issue_wait() that does not wait) show that the checker sees such races.
"""
import random
import types

import pytest
import torch

from paper_2404_04270_amd import step as step_mod


class Recorder:
    """Streams as lists of enqueued operations, events as versioned marks."""

    def __init__(self, rng, lazy):
        self.rng, self.lazy = rng, lazy
        self.streams = {}            # handle -> list of ops
        self.latest = {}             # event id -> (stream handle, position) of its last record
        self.n_events = 0
        self.queues = []
        self.counts = dict(filter=0, lookup=0, update=0)

    def stream(self, handle):
        return self.streams.setdefault(handle, [])

    # enqueue-time actions (called at once, or when a queue job is issued)
    def kernel(self, handle, kind, batch):
        self.stream(handle).append(("kernel", kind, batch))

    def record(self, handle, ev):
        ops = self.stream(handle)
        ops.append(("record", ev))
        self.latest[ev] = (handle, len(ops) - 1)

    def wait(self, handle, ev):
        # binds to the last record enqueued so far; none: the wait is a no-op
        self.stream(handle).append(("wait", self.latest.get(ev)))

    def pump_some(self):
        """Issue threads make progress at moments of their own choosing."""
        for q in self.queues:
            if self.rng.random() < 0.5:
                q.pump(self.rng.randint(0, 4))


class FakeStream:
    n = 0

    def __init__(self, device=None):
        FakeStream.n += 1
        self.handle = FakeStream.n


def make_binding(rec, honour_wait_issued=True):
    B = types.SimpleNamespace()

    class Tables:
        def __init__(self, weights):
            self.num_tables, self.dim = len(weights), weights[0].shape[1]
            self.device, self.c = weights[0].device, None

        def new_bits(self):
            return [torch.zeros(1, dtype=torch.int32) for _ in range(self.num_tables)]

    class HotState:
        def __init__(self, tables, hot_ids, diagnostics=True):
            pass

    class IssueQueue:
        def __init__(self):
            self.jobs, self.submitted, self.issued = [], 0, 0
            rec.queues.append(self)

        def _push(self, job):
            self.jobs.append(job)
            self.submitted += 1
            if not rec.lazy:
                self.pump(len(self.jobs))
            else:
                rec.pump_some()
            return self.submitted

        def pump(self, n):
            while n > 0 and self.jobs:
                self.jobs.pop(0)()
                self.issued += 1
                n -= 1

        def new_event(self):
            rec.n_events += 1
            return rec.n_events

        @staticmethod
        def record_now(ev, handle):
            rec.record(handle, ev)
            rec.pump_some()

        @staticmethod
        def wait_now(handle, ev):
            rec.wait(handle, ev)
            rec.pump_some()

        def wait_event(self, ev, handle):
            return self._push(lambda: rec.wait(handle, ev))

        def record_event(self, ev, handle):
            return self._push(lambda: rec.record(handle, ev))

        def wait_issued(self, ticket):
            assert ticket <= self.submitted
            if honour_wait_issued:
                self.pump(ticket - self.issued)

        def prepared_index_batch(self, *a):
            def call(idx, handle):
                k = rec.counts["filter"]
                rec.counts["filter"] += 1

                def job():
                    rec.kernel(handle, "filter", k)
                    rec.kernel(handle, "group", k)
                return self._push(job)
            return call

        def stop(self):
            self.pump(len(self.jobs))

        def close(self):
            self.stop()

    def prepared_filter_batch(*a):
        def call(idx, handle):
            k = rec.counts["filter"]
            rec.counts["filter"] += 1
            rec.kernel(handle, "filter", k)
            rec.last_filtered = k
        return call

    def prepared_backward_prepare(*a):
        return lambda handle: rec.kernel(handle, "group", rec.last_filtered)

    def prepared_forward(*a):
        def call(handle):
            rec.kernel(handle, "lookup", rec.counts["lookup"])
            rec.counts["lookup"] += 1
            rec.pump_some()
        return call

    def prepared_backward_apply(*a):
        def call(grad, handle):
            rec.kernel(handle, "update", rec.counts["update"])
            rec.counts["update"] += 1
            rec.pump_some()
        return call

    def ss_detect_stale(tables, hot, thr, refresh, stream=None):
        rec.kernel(stream.handle, "detect", rec.counts["update"] - 1)

    def ss_event_create():
        rec.n_events += 1
        return rec.n_events

    B.Tables, B.HotState, B.IssueQueue = Tables, HotState, IssueQueue
    B.prepared_filter_batch = prepared_filter_batch
    B.prepared_backward_prepare = prepared_backward_prepare
    B.prepared_forward = prepared_forward
    B.prepared_backward_apply = prepared_backward_apply
    B.ss_detect_stale = ss_detect_stale
    B.ss_event_create = ss_event_create
    B.ss_event_destroy = lambda ev: None
    B.ss_filter_batch_workspace_bytes = lambda T, b, L: 256
    B.ss_backward_workspace_bytes = lambda T, b, L, D: 256
    B.stream_handle = lambda st: st.handle
    return B


def drive(monkeypatch, rng, n_batches, K, every, streams, threads, lazy, greedy,
          honour_wait_issued=True):
    rec = Recorder(rng, lazy)
    monkeypatch.setattr(step_mod, "B", make_binding(rec, honour_wait_issued))
    monkeypatch.setattr(torch.cuda, "Stream", FakeStream)
    main = FakeStream()
    monkeypatch.setattr(torch.cuda, "current_stream", lambda dev=None: main)
    W = [torch.zeros(4, 4) for _ in range(2)]
    st = step_mod.PipelinedStep(W, [torch.zeros(1, dtype=torch.int32)] * 2, 8, 1, 0.01, 1e-3, K,
                                every=every, index_streams=streams, issue_thread=threads)
    idx, grad = torch.zeros(2, 8, 1, dtype=torch.int32), torch.zeros(2, 8, 4)
    ahead = 0
    for it in range(n_batches):
        want = st.room() if greedy else rng.randint(0, st.room())
        while ahead < n_batches and st.room() > 0 and (want > 0 or ahead <= it):
            st.submit(idx)
            ahead += 1
            want -= 1
        st.forward()
        st.backward(grad)
    st.flush()
    st.close()
    for q in rec.queues:              # (only a broken wait_issued leaves any)
        q.pump(len(q.jobs))
    return rec, len(st.sets) if hasattr(st, "sets") else None


def execute(rec, ring, K, rng):
    """Runs the recorded program with a random scheduler; returns the violations."""
    streams = {h: ops for h, ops in rec.streams.items() if ops}
    pos = {h: 0 for h in streams}
    done_records = set()              # (handle, position) of executed record ops
    done = set()                      # (kind, batch) of executed kernels
    bad = []

    def need(kind, k, what):
        if what not in done:
            bad.append((kind, k, "before", what))

    def runnable(h):
        if pos[h] >= len(streams[h]):
            return False
        op = streams[h][pos[h]]
        return not (op[0] == "wait" and op[1] is not None and op[1] not in done_records)

    while True:
        ready = [h for h in streams if runnable(h)]
        if not ready:
            break
        h = rng.choice(ready)
        # a burst from one stream, as a GPU that runs one queue ahead of the others
        for _ in range(rng.randint(1, 6)):
            if not runnable(h):
                break
            op = streams[h][pos[h]]
            if op[0] == "record":
                done_records.add((h, pos[h]))
            elif op[0] == "kernel":
                _, kind, k = op
                if kind == "filter":
                    if k >= ring:
                        need(kind, k, ("update", k - ring))
                    b = (k // K) * K - 1          # last boundary batch before k
                    if b >= 0:
                        need(kind, k, ("detect", b))
                elif kind == "group":
                    need(kind, k, ("filter", k))
                elif kind == "lookup":
                    need(kind, k, ("filter", k))
                    if k > 0:
                        need(kind, k, ("update", k - 1))
                elif kind == "update":
                    need(kind, k, ("group", k))
                    need(kind, k, ("lookup", k))
                elif kind == "detect":
                    need(kind, k, ("update", k))
                done.add((kind, k))
            pos[h] += 1
    stuck = {h: streams[h][pos[h]] for h in streams if pos[h] < len(streams[h])}
    return bad, stuck, done


CASES = [
    # K, every, streams, issue threads (0: none), lazy queues, greedy submit
    (7, 1, 1, 0, False, True), (7, 4, 1, 0, False, True), (5, 2, 2, 0, False, False),
    (100, 8, 1, 0, False, True), (3, 2, 3, 0, False, False), (11, 4, 2, 0, False, False),
    (7, 1, 1, 1, True, True), (7, 4, 1, 1, True, False), (5, 2, 2, 1, True, False),
    (5, 2, 3, 3, True, False), (9, 1, 3, True, True, True), (4, 2, 4, True, True, False),
    (13, 4, 3, 2, True, False), (100, 8, 2, 2, True, True), (2, 1, 2, 2, True, False),
    (1, 1, 1, 1, True, True), (1, 2, 3, 3, True, False),
]


@pytest.mark.parametrize("K,every,streams,threads,lazy,greedy", CASES)
def test_every_kernel_finds_its_inputs_complete(monkeypatch, K, every, streams, threads, lazy,
                                                greedy):
    for seed in range(4):
        rng = random.Random(1000 * seed + 17 * K + every + streams)
        n = 150
        rec, ring = drive(monkeypatch, rng, n, K, every, streams, threads, lazy, greedy)
        assert ring == 3 * every * streams
        for _ in range(6):
            bad, stuck, done = execute(rec, ring, K, rng)
            assert not stuck, stuck
            assert not bad, bad[:5]
            for kind in ("filter", "group", "lookup", "update"):
                assert sum(1 for d in done if d[0] == kind) == n
            assert sum(1 for d in done if d[0] == "detect") == n // K


@pytest.mark.parametrize("issue_threads", [0, 2])
def test_the_checker_sees_a_missing_wait(monkeypatch, issue_threads):
    """Planted mistake: marks that claim every batch is already known to the waiter."""
    marks = step_mod.PipelinedStep._QueueMarks if issue_threads else step_mod.PipelinedStep._Marks
    monkeypatch.setattr(marks, "cover", lambda self, *a: True)
    rng = random.Random(5)
    rec, ring = drive(monkeypatch, rng, 120, 7, 2, 2, issue_threads, bool(issue_threads), False)
    found = False
    for _ in range(20):
        bad, stuck, _ = execute(rec, ring, 7, rng)
        found = found or bool(bad)
    assert found


def test_the_checker_sees_a_wait_for_an_event_not_yet_recorded(monkeypatch):
    """Planted mistake: ss_issue_wait() returns at once, so the training stream is made
    to wait for events whose record is still sitting in an issue queue - a no-op."""
    rng = random.Random(6)
    rec, ring = drive(monkeypatch, rng, 120, 7, 2, 2, 2, True, False, honour_wait_issued=False)
    found = False
    for _ in range(20):
        bad, stuck, _ = execute(rec, ring, 7, rng)
        found = found or bool(bad)
    assert found
