"""Host logic of the step scheduler (ss_step, csrc/step.hip), checked on the CPU
against a model of streams.

The scheduler spreads the calls of a batch over several streams and lets them meet
through events as rarely as it can.  A missing wait there would not fail loudly on
the GPU: it would be a race that the parity tests only catch when the timing
happens to be bad.  Here the scheduler is built with ss_step_create_traced, which
hands every operation it would enqueue to a callback instead; it is driven through
a few hundred batches, and the recorded program (per stream: kernels, event
records, event waits) is then executed by a scheduler that picks runnable streams
at random.  Whatever order it picks, every kernel must find its inputs complete:

  filter(k)   after update(k - ring) (the buffer set's previous batch) and after the
              detect pass of the last boundary batch before k (it reads the bitmaps);
  group(k)    after filter(k);
  lookup(k)   after filter(k) and update(k - 1);
  update(k)   after group(k) and lookup(k);
  detect(b)   after update(b);

and the program must run to its end (no wait for an event nobody records).  A wait
takes the event's most recent record at the moment the wait is ENQUEUED, as HIP
does; with issue threads, jobs reach their stream late and in bursts (here: when the
model's queues are pumped, at random moments), which is what waiting for a job to
have been issued is for.  Two planted mistakes (in the model, not in the library: a
stream that drops the waits it is given; a "wait until issued" that does not wait)
show that the checker sees such races.
"""
import ctypes as C
import random

import pytest

from paper_2404_04270_amd import binding as B

MAIN = -1


class Recorder:
    """Streams as lists of enqueued operations, events as versioned marks, issue
    queues as lists of jobs that are issued when the model chooses."""

    def __init__(self, rng, lazy, n_queues, honour_wait_issued=True, drop_waits=False):
        self.rng, self.lazy = rng, lazy
        self.honour_wait_issued, self.drop_waits = honour_wait_issued, drop_waits
        self.streams = {}            # stream number -> list of ops
        self.latest = {}             # event id -> (stream, position) of its last record
        self.queues = [dict(jobs=[], submitted=0, issued=0) for _ in range(n_queues)]
        self.counts = dict(filter=0, lookup=0, update=0)

    def stream(self, s):
        return self.streams.setdefault(s, [])

    # enqueue-time actions (called at once, or when a queue job is issued)
    def kernel(self, s, kind, batch):
        self.stream(s).append(("kernel", kind, batch))

    def record(self, s, ev):
        ops = self.stream(s)
        ops.append(("record", ev))
        self.latest[ev] = (s, len(ops) - 1)

    def wait(self, s, ev):
        if self.drop_waits:
            return
        # binds to the last record enqueued so far; none: the wait is a no-op
        self.stream(s).append(("wait", self.latest.get(ev)))

    def index(self, s):
        k = self.counts["filter"]
        self.counts["filter"] += 1
        return k

    # issue queues
    def push(self, q, job):
        queue = self.queues[q]
        queue["jobs"].append(job)
        queue["submitted"] += 1
        if not self.lazy:
            self.pump(q, len(queue["jobs"]))
        else:
            self.pump_some()
        return queue["submitted"]

    def pump(self, q, n):
        queue = self.queues[q]
        while n > 0 and queue["jobs"]:
            queue["jobs"].pop(0)()
            queue["issued"] += 1
            n -= 1

    def pump_some(self):
        """Issue threads make progress at moments of their own choosing."""
        for q in range(len(self.queues)):
            if self.rng.random() < 0.5:
                self.pump(q, self.rng.randint(0, 4))

    def callbacks(self):
        """The table of operations ss_step_create_traced takes."""
        T = B.StepTraceOps

        def index_now(_, s, st):
            k = self.index(s)
            self.kernel(s, "filter", k)
            self.kernel(s, "group", k)
            return 0

        def q_index(_, q, s, st, ticket):
            k = self.index(s)

            def job():
                self.kernel(s, "filter", k)
                self.kernel(s, "group", k)
            ticket[0] = self.push(q, job)
            return 0

        def lookup(_, st):
            self.kernel(MAIN, "lookup", self.counts["lookup"])
            self.counts["lookup"] += 1
            self.pump_some()
            return 0

        def update(_, st):
            self.kernel(MAIN, "update", self.counts["update"])
            self.counts["update"] += 1
            self.pump_some()
            return 0

        def detect(_, with_threshold):          # the capture is a launch of the same kernel
            self.kernel(MAIN, "detect", self.counts["update"] - 1)
            return 0

        def record_now(_, ev, s):
            self.record(s, ev)
            self.pump_some()
            return 0

        def wait_now(_, s, ev):
            self.wait(s, ev)
            self.pump_some()
            return 0

        def q_record(_, q, ev, s, ticket):
            ticket[0] = self.push(q, lambda: self.record(s, ev))
            return 0

        def q_wait(_, q, ev, s, ticket):
            ticket[0] = self.push(q, lambda: self.wait(s, ev))
            return 0

        def q_wait_issued(_, q, ticket):
            queue = self.queues[q]
            assert ticket <= queue["submitted"]
            if self.honour_wait_issued:
                self.pump(q, ticket - queue["issued"])
            return 0

        self._keep = T(None, T.INDEX_NOW(index_now), T.Q_INDEX(q_index), T.ON_SET(lookup),
                       T.ON_SET(update), T.ON_SET(detect), T.EVENT_NOW(record_now),
                       T.EVENT_NOW(wait_now), T.Q_EVENT(q_record), T.Q_EVENT(q_wait),
                       T.Q_WAIT_ISSUED(q_wait_issued))
        return self._keep


def drive(rng, n_batches, K, every, streams, threads, lazy, greedy, honour_wait_issued=True,
          drop_waits=False):
    if threads is True:              # a thread per stream from three streams on, else one
        threads = streams if streams >= 3 else 1
    plan = B.ss_step_plan_for(1, 1, 1, every, streams, int(threads))
    assert (plan.every, plan.index_streams, plan.issue_threads) == (every, streams, min(int(threads), streams))
    rec = Recorder(rng, lazy, plan.issue_threads, honour_wait_issued, drop_waits)
    step = B.ss_step_create_traced(plan, K, rec.callbacks())
    idx = C.c_int32(0)               # never read: the traced scheduler only passes it on

    class _Idx:                      # what ss_step_submit's binding asks of a tensor
        @staticmethod
        def data_ptr():
            return C.addressof(idx)
    ahead = 0
    for it in range(n_batches):
        room = B.ss_step_room(step)
        want = room if greedy else rng.randint(0, room)
        while ahead < n_batches and B.ss_step_room(step) > 0 and (want > 0 or ahead <= it):
            B.ss_step_submit(step, _Idx)
            ahead += 1
            want -= 1
        B.ss_step_forward(step)
        B.ss_step_backward(step, _Idx)
    B.ss_step_flush(step)
    B.ss_step_destroy(step)
    for q in range(len(rec.queues)):   # (only a broken "wait until issued" leaves any)
        rec.pump(q, len(rec.queues[q]["jobs"]))
    return rec, plan.num_sets


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
def test_every_kernel_finds_its_inputs_complete(K, every, streams, threads, lazy, greedy):
    for seed in range(4):
        rng = random.Random(1000 * seed + 17 * K + every + streams)
        n = 150
        rec, ring = drive(rng, n, K, every, streams, threads, lazy, greedy)
        assert ring == 3 * every * streams
        for _ in range(6):
            bad, stuck, done = execute(rec, ring, K, rng)
            assert not stuck, stuck
            assert not bad, bad[:5]
            for kind in ("filter", "group", "lookup", "update"):
                assert sum(1 for d in done if d[0] == kind) == n
            assert sum(1 for d in done if d[0] == "detect") == n // K


@pytest.mark.parametrize("issue_threads", [0, 2])
def test_the_checker_sees_a_missing_wait(issue_threads):
    """Planted mistake (in the model): streams that drop the waits they are given."""
    rng = random.Random(5)
    rec, ring = drive(rng, 120, 7, 2, 2, issue_threads, bool(issue_threads), False,
                      drop_waits=True)
    found = False
    for _ in range(20):
        bad, stuck, _ = execute(rec, ring, 7, rng)
        found = found or bool(bad)
    assert found


def test_the_checker_sees_a_wait_for_an_event_not_yet_recorded():
    """Planted mistake (in the model): "wait until that job has been issued" returns at
    once, so the training stream is made to wait for events whose record is still
    sitting in an issue queue - a no-op."""
    rng = random.Random(6)
    rec, ring = drive(rng, 120, 7, 2, 2, 2, True, False, honour_wait_issued=False)
    found = False
    for _ in range(20):
        bad, stuck, _ = execute(rec, ring, 7, rng)
        found = found or bool(bad)
    assert found


def test_calls_out_of_order_are_refused_and_enqueue_nothing():
    rng = random.Random(7)
    plan = B.ss_step_plan_for(1, 1, 1, 1, 1, 0)            # ring of 3: two batches ahead at most
    rec = Recorder(rng, False, 0)
    step = B.ss_step_create_traced(plan, 4, rec.callbacks())
    word = C.c_int32(0)

    class _Idx:
        @staticmethod
        def data_ptr():
            return C.addressof(word)
    with pytest.raises(B.SlipstreamError):
        B.ss_step_forward(step)                            # nothing submitted
    B.ss_step_submit(step, _Idx)
    with pytest.raises(B.SlipstreamError):
        B.ss_step_backward(step, _Idx)                     # no forward yet
    B.ss_step_forward(step)
    B.ss_step_submit(step, _Idx)
    assert B.ss_step_room(step) == 0
    with pytest.raises(B.SlipstreamError):
        B.ss_step_submit(step, _Idx)                       # too far ahead
    with pytest.raises(B.SlipstreamError):
        B.ss_step_forward(step)                            # previous batch not finished
    before = {s: len(ops) for s, ops in rec.streams.items()}
    with pytest.raises(B.SlipstreamError):
        B.ss_step_forward(step)
    assert before == {s: len(ops) for s, ops in rec.streams.items()}
    B.ss_step_backward(step, _Idx)
    B.ss_step_forward(step)
    B.ss_step_backward(step, _Idx)
    B.ss_step_destroy(step)
    kinds = [op[1] for ops in rec.streams.values() for op in ops if op[0] == "kernel"]
    assert kinds.count("lookup") == 2 and kinds.count("update") == 2 and kinds.count("filter") == 2
