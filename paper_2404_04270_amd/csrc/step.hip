// ss_step: one training iteration after the other (Algorithm 1 of the paper: drop
// the inputs that only reach stale entries, train on the rest, every K iterations
// compare the hot rows with their last snapshot), with the index work of the coming
// batches taken off the critical path.
//
// Classifying a batch and grouping its lookups by row (ss_filter_batch,
// ss_embbag_backward_prepare) need the indices and the stale bitmaps only, not the
// weights: they run for the coming batches on index streams of their own, into a
// ring of buffer sets, while the current batch is in its lookup and update kernels
// on the training stream.  An event recorded on a stream, or a wait for one, as a
// command of its own between two dependent kernels costs that stream several
// microseconds on this platform, so there are as few such commands as possible.
// Events ride on launches that happen anyway (the dispatch's own completion signal):
// every batch's index work carries one on its last launch, and every `every`-th
// update of the training stream carries one ("everything up to batch k is done").
// A stream is made to wait only for a batch that is not covered by an event it has
// waited for already, the training stream only if the calling thread cannot see that
// the event has happened, and then for as many further batches as the index streams
// can be expected to be ahead (cover_indexed).  The ring holds
// 3 * every sets per index stream, of which two thirds may be in use ahead of the
// batch being trained on: the set a new batch takes over was then last used at
// least `every` batches ago, which an event of the training stream already covers.
// The index work reads the stale bitmaps, so batches after one that ends with a
// detect pass are held back until that pass has been enqueued.
//
// The scheduling logic talks to the GPU through a small table of operations
// (StepOps).  The real table enqueues the library's kernels and HIP events, where
// asked through ss_issue_queue threads; a second one hands every operation to
// callbacks, which lets a test execute the recorded program of streams, events and
// waits under a random scheduler on the CPU and check that every kernel finds its
// inputs complete.
#include <algorithm>
#include <chrono>
#include <deque>
#include <memory>
#include <new>
#include <string>
#include <vector>

#include "ss_common.h"

namespace ss {

namespace {

constexpr int kMainStream = -1;
constexpr size_t kMarksKept = 64;     // recorded marks kept per stream
constexpr int kEventPool = 66;        // ... one being recorded, one spare
constexpr size_t kRingBytes = 96u << 20;

struct StepOps {
    virtual ~StepOps() {}
    // ss_filter_batch + ss_embbag_backward_prepare of a batch into buffer set `set`,
    // on index stream `stream`: at once, or as a job of issue queue `queue`; then
    // event `done` is recorded on that stream as record_now / q_record would
    // (*ticket: the job after which the record has been issued)
    virtual int32_t index_now(int stream, int set, const int32_t *idx, void *done) = 0;
    virtual int32_t q_index(int queue, int stream, int set, const int32_t *idx, void *done,
                            uint64_t *ticket) = 0;
    // on the training stream
    virtual int32_t lookup(int set) = 0;
    // record_after (may be null): an event of the training stream to record once the
    // update is complete, as record_now would right after it
    virtual int32_t update(int set, const float *grad, void *record_after) = 0;
    virtual int32_t detect(float threshold) = 0;
    // events; stream kMainStream is the training stream
    virtual int32_t new_event(void **ev) = 0;
    virtual int32_t record_now(void *ev, int stream) = 0;
    virtual int32_t wait_now(int stream, void *ev) = 0;
    // has the event, recorded (issued) earlier, happened already?  "no" is always a safe answer
    virtual bool done_now(void *ev) = 0;
    virtual bool polls() const = 0;    // can done_now ever say yes?
    virtual int32_t q_record(int queue, void *ev, int stream, uint64_t *ticket) = 0;
    virtual int32_t q_wait(int queue, void *ev, int stream, uint64_t *ticket) = 0;
    virtual int32_t q_wait_issued(int queue, uint64_t ticket) = 0;
    virtual int32_t shutdown() = 0;    // queues drained and ended, then events destroyed
};

}  // namespace

}  // namespace ss

using ss::StepOps;

struct ss_step {
    std::unique_ptr<StepOps> ops;
    int every = 1, n_side = 1, n_sets = 3, n_queues = 0, K = 1;
    float threshold = 0.f;

    // Events of one stream, each with the last batch it covers, and what each
    // waiting stream already knows to be done.
    struct Mark {
        int64_t covers;
        void *ev;
        uint64_t ticket;
    };
    struct Marks {
        std::deque<Mark> recorded;        // ascending in `covers`
        std::vector<void *> spare;
        std::vector<int64_t> known;       // by waiter: batches <= this are done
        int stream = ss::kMainStream;     // the stream whose progress these marks tell
        bool by_queue = false;            // recorded through that stream's issue queue
        int queue = 0;
    };
    std::vector<Marks> indexed;           // one per index stream
    Marks trained;                        // training stream: update done up to batch ...

    int64_t submitted = 0, issued = 0, forwarded = 0, it = 0, last_detect = -1;
    int64_t lead_lost = -1;               // last batch before which the index streams had no lead
    int host_wait_us = 0;                 // longest the calling thread polls for index work
    int64_t n_wait_cmds = 0, n_polls = 0, n_polls_done = 0;      // ss_step_counters
    static constexpr int kProgress = 8;
    void *progress[kProgress] = {};       // by batch % kProgress: the event that says its update is done
    std::vector<void *> progress_pool;    // ... those of them that are not also in `trained`
    bool have_snapshot = false;
    struct Held {
        const int32_t *idx;
        void *ready;
    };
    std::deque<Held> held_back;           // batches waiting for a detect pass before them
    std::vector<uint64_t> last_ticket;    // per queue

    int queue_of(int stream) const { return n_queues ? stream % n_queues : 0; }
    bool boundary(int64_t k) const { return (k + 1) % K == 0; }
    // does a batch in [lo, hi) end with a snapshot / detect pass?
    bool boundary_in(int64_t lo, int64_t hi) const { return (lo / K + 1) * K - 1 < hi; }
    int room() const { return (int)(2 * (int64_t)every * n_side - (submitted - it)); }

    void keep(Marks &m, int64_t covers, void *ev, uint64_t ticket)
    {
        m.recorded.push_back(Mark{covers, ev, ticket});
        if (m.recorded.size() > ss::kMarksKept) {     // that far back: issued and waited for long ago
            m.spare.push_back(m.recorded.front().ev);
            m.recorded.pop_front();
        }
    }

    int32_t record(Marks &m, int64_t covers)
    {
        if (m.spare.empty())
            return ss::fail(SS_ERR_HIP, "ss_step: event pool exhausted");
        void *ev = m.spare.back();
        m.spare.pop_back();
        uint64_t ticket = 0;
        const int32_t rc = (n_queues && m.by_queue) ? ops->q_record(m.queue, ev, m.stream, &ticket)
                                                    : ops->record_now(ev, m.stream);
        if (rc) return rc;
        keep(m, covers, ev, ticket);
        return SS_OK;
    }

    // Makes `waiting_stream` wait until `batch` is done on the marks' stream, if it
    // does not know yet.  *covered = false if no recorded event covers the batch.
    int32_t cover(Marks &m, int waiter, int waiting_stream, int64_t batch, bool *covered)
    {
        *covered = true;
        if (batch <= m.known[waiter]) return SS_OK;
        for (const Mark &mk : m.recorded) {
            if (mk.covers < batch) continue;
            int32_t rc;
            if (!n_queues) {
                rc = ops->wait_now(waiting_stream, mk.ev);
            } else if (m.by_queue) {
                // a wait for an event whose record has not been issued yet is a no-op
                rc = ops->q_wait_issued(m.queue, mk.ticket);
                if (!rc) rc = ops->wait_now(waiting_stream, mk.ev);
            } else {      // the waiter is an index stream: through its queue, in order with its work
                uint64_t t = 0;
                rc = ops->q_wait(queue_of(waiting_stream), mk.ev, waiting_stream, &t);
            }
            if (rc) return rc;
            m.known[waiter] = mk.covers;
            return SS_OK;
        }
        *covered = false;
        return SS_OK;
    }

    // Is the update of the batch before the last one still unfinished?  Then the training
    // stream has more than one batch of work left.
    bool backlog()
    {
        if (it < 2 || !progress[(it - 2) % kProgress]) return false;
        return !ops->done_now(progress[(it - 2) % kProgress]);
    }

    // The calling thread is ahead of the GPU: the index work of the batch it is about to
    // enqueue the lookup of has not finished.  While the training stream still has more
    // than a batch of work queued, nothing is lost by keeping the thread here until that
    // index work is done, and the stream is spared a wait command, which takes it 8 us
    // between two kernels even when the event has long happened by the time the stream
    // gets there.  With less work queued (a start from an empty pipeline, the batches
    // behind a detect pass) the thread would be late with the lookup: the wait command is
    // better there (20 steps from an empty pipeline at 26 tables x 8192 lookups: 56-58 us
    // each when always polled for, 48.5 so).  Measured, 2000 steps: 94.5-94.9 instead of
    // 96.6 us per step at 8 tables x 81920 lookups, where 37 % of the batches got a wait
    // command; 44.8 either way at 26 x 8192 (19 %); 27.5 against 27.4 at one table x
    // 65536.  Regions of 20 steps take 1 us per step longer with it (the thread submits
    // the index work of later batches later), which is why ss_step_plan_for turns it on
    // for bags of several lookups only.
    int32_t poll_indexed(const Marks &m, const Mark *mine)
    {
        if (n_queues) {      // the event's record must have been issued before a query means anything
            const int32_t rc = ops->q_wait_issued(m.queue, mine->ticket);
            if (rc) return rc;
        }
        const auto t0 = std::chrono::steady_clock::now();
        const auto limit = std::chrono::microseconds(host_wait_us);
        ++n_polls;
        while (!ops->done_now(mine->ev) && backlog() &&
               std::chrono::steady_clock::now() - t0 < limit)
            __builtin_ia32_pause();
        if (ops->done_now(mine->ev)) ++n_polls_done;
        return SS_OK;
    }

    // The training stream is about to look up batch k, whose index work ran on index
    // stream j.  Every batch has an event of its own there.  If the calling thread can see
    // that the index stream is past k already, nothing is enqueued, and all batches up to
    // the newest finished one count as known.  Otherwise the training stream gets a wait
    // command, which costs it a few microseconds between two kernels whether it has to wait
    // or not: it is made to cover `ahead` further batches of that stream, as many as the
    // index streams can be expected to have regained of their lead since the last detect
    // pass (behind which they start with none and gain only the difference between the
    // two paces per batch; an event that covered a whole ring there kept the training
    // stream waiting 130-180 us once per pass).
    int32_t cover_indexed(int j, int64_t k)
    {
        Marks &m = indexed[j];
        if (k <= m.known[0]) return SS_OK;
        const auto at = [&](int64_t batch) -> const Mark * {
            for (const Mark &mk : m.recorded)
                if (mk.covers == batch) return &mk;
            return nullptr;
        };
        const int64_t last = issued - 1 - (issued - 1 - j) % n_side;     // newest batch of stream j
        const Mark *mine = at(k);
        if (!mine) return ss::fail(SS_ERR_HIP, "ss_step: internal: batch %lld has no event", (long long)k);
        if (host_wait_us > 0 && ops->polls() && !ops->done_now(mine->ev)) {
            const int32_t rc = poll_indexed(m, mine);
            if (rc) return rc;
            if (n_queues && ops->done_now(mine->ev)) {
                m.known[0] = k;       // (later events of the stream may not have been recorded yet)
                return SS_OK;
            }
        }
        if (!n_queues) {
            // events of a stream happen in order: the newest finished one, by bisection
            if (ops->done_now(mine->ev)) {
                int64_t lo = k, hi = last;           // lo is done
                while (lo < hi) {
                    const int64_t mid = lo + ((hi - lo) / n_side + 1) / 2 * n_side;
                    const Mark *mk = at(mid);
                    if (mk && ops->done_now(mk->ev)) lo = mid;
                    else hi = mid - n_side;
                }
                m.known[0] = lo;
                return SS_OK;
            }
        }
        // A caller that submits just in time (at the start, or when it starts again after
        // a synchronisation) has no lead either: that moment counts like a detect pass.
        if (issued - 1 - k <= 1) lead_lost = k - 1;
        const int64_t since = k - std::max(last_detect, lead_lost) - 1;
        const int64_t ahead = std::min<int64_t>(
            {(int64_t)every - 1, since / (8 * n_side), (last - k) / n_side});
        const Mark *target = at(std::min(last, k + ahead * n_side));
        if (!target) target = mine;
        int32_t rc = SS_OK;
        if (n_queues) {
            // a wait for an event whose record has not been issued yet is a no-op
            rc = ops->q_wait_issued(m.queue, target->ticket);
            if (rc) return rc;
        }
        ++n_wait_cmds;
        rc = ops->wait_now(ss::kMainStream, target->ev);
        if (rc) return rc;
        m.known[0] = target->covers;
        return SS_OK;
    }

    int32_t issue(int64_t k, const int32_t *idx, void *ready)
    {
        const int set = (int)(k % n_sets), j = (int)(k % n_side);
        int32_t rc = SS_OK;
        if (ready) {
            uint64_t t = 0;
            rc = n_queues ? ops->q_wait(queue_of(j), ready, j, &t) : ops->wait_now(j, ready);
            if (rc) return rc;
        }
        // the set's previous batch must be over, and so must the last detect pass
        const int64_t need = std::max<int64_t>(k - n_sets, last_detect);
        if (need >= 0) {
            bool ok = false;
            rc = cover(trained, j, j, need, &ok);
            if (rc) return rc;
            if (!ok) {
                rc = record(trained, it - 1);
                if (rc) return rc;
                rc = cover(trained, j, j, need, &ok);
                if (rc) return rc;
                if (!ok) return ss::fail(SS_ERR_HIP, "ss_step: internal: batch %lld not covered",
                                         (long long)need);
            }
        }
        // Every batch's index work carries an event of its own, on its last launch.  The
        // training stream then never waits for more index work than the batch it is about
        // to look up needs (an event that covered several batches kept it waiting 130-180 us
        // once behind every detect pass, while the index streams had not regained their
        // lead), and as long as the index streams are ahead it does not wait at all.
        Marks &m = indexed[j];
        if (m.spare.empty()) return ss::fail(SS_ERR_HIP, "ss_step: event pool exhausted");
        void *ev = m.spare.back();
        m.spare.pop_back();
        uint64_t ticket = 0;
        if (n_queues) {
            rc = ops->q_index(queue_of(j), j, set, idx, ev, &ticket);
            last_ticket[queue_of(j)] = ticket;
        } else {
            rc = ops->index_now(j, set, idx, ev);
        }
        if (rc) {
            m.spare.push_back(ev);
            return rc;
        }
        ++issued;
        keep(m, k, ev, ticket);
        return rc;
    }

    // Index work of up to `limit` held-back batches, as far as no detect pass is still
    // due before them.  A few at a time: enqueueing a whole ring at once after a detect
    // pass keeps the calling thread busy while the training stream runs dry.
    int32_t drain(int limit)
    {
        while (limit > 0 && !held_back.empty() && !boundary_in(it, issued)) {
            const Held h = held_back.front();
            held_back.pop_front();
            const int32_t rc = issue(issued, h.idx, h.ready);
            if (rc) return rc;
            --limit;
        }
        return SS_OK;
    }
};

namespace ss {

namespace {

// Batches between two cross-stream events: 8, or fewer when the grouped lists of a
// ring of 3 * every * streams sets would not fit the memory-side cache next to the
// step's own traffic (a list written by an index stream should still be there when
// the update kernel reads it).
int auto_every(int T, int B, int L, int n_side)
{
    const size_t per_set = (size_t)16 * T * (((size_t)B * L + 2047) / 2048) * 2048;
    int every = 8;
    while (every > 2 && (size_t)3 * every * n_side * per_set > kRingBytes) every /= 2;
    return every;
}

// Index streams: one while a table has at most 16384 lookups per batch; beyond that
// the grouping is a chain of three launches per batch behind the two of the classifier
// that lasts 50-70 us beside the training kernels, longer than those do at most shapes,
// and two chains side by side keep the index work ahead (52.7 against 63.7 us per step
// at 8 tables x 32768 lookups of 64 floats, 38.9 against 52.8 at 2 x 80000 x 64); three
// when those launches are tiny (fewer than 128 workgroups over all tables: 24.4 / 28.4 /
// 50.1 us with 3 / 2 / 1 at one table x 65536).  Where the training kernels of a batch
// move so much that they outlast the chain (more than 256 MB of looked-up rows: 335 MB
// and 85 us at 8 tables x 81920 lookups of 128 floats), one stream is enough and a second
// only puts more index kernels beside them (84.7 against 87.4 us per step).
int auto_streams(int T, int B, int L, int dim)
{
    const int64_t lookups = (int64_t)B * L;
    if (lookups <= 16384) return 1;
    if (T * ((lookups + 2047) / 2048) < 128) return 3;
    return (int64_t)T * lookups * dim * 4 > (256LL << 20) ? 1 : 2;
}

// Issue threads: where a batch is a string of launches at their latency floor, so
// that one host thread cannot enqueue them as fast as the GPU finishes them.
int auto_threads(int T, int B, int L, int n_side)
{
    if (!(n_side >= 3 || (int64_t)T * B * L <= 65536)) return 0;
    return n_side >= 3 ? n_side : 1;
}

// ---- the real operations: library kernels, HIP events, issue queues --------
struct GpuOps final : StepOps {
    ss_tables tables;
    int B, L, alpha, H;
    float lr;
    std::vector<ss_step_set> sets;
    int32_t *const *hot_ids;
    float **snapshot;
    uint8_t **stale_hot;
    double **drift;
    uint32_t *stale_count;
    float *pooled;
    hipStream_t main;
    std::vector<hipStream_t> sides;
    std::vector<ss_issue_queue *> queues;
    std::vector<void *> events;

    hipStream_t stream(int s) const { return s == kMainStream ? main : sides[s]; }

    // the event rides on the last launch of the index work: no command of its own
    int32_t index_now(int s, int set, const int32_t *idx, void *done) override
    {
        const ss_step_set &b = sets[set];
        int32_t rc = launch_filter(&tables, idx, B, L, alpha, b.skip_mask, b.kept_ids, b.n_kept,
                                   b.idx_c, b.ws_filter, stream(s));
        if (rc) return rc;
        return launch_backward_prepare(&tables, b.idx_c, B, L, b.n_kept, b.ws_backward, stream(s),
                                       static_cast<hipEvent_t>(done));
    }
    int32_t q_index(int q, int s, int set, const int32_t *idx, void *done,
                    uint64_t *ticket) override
    {
        const ss_step_set &b = sets[set];
        return issue_index_batch(queues[q], &tables, idx, B, L, alpha, b.skip_mask, b.kept_ids,
                                 b.n_kept, b.idx_c, b.ws_filter, b.ws_filter_bytes, b.ws_backward,
                                 b.ws_backward_bytes, stream(s), done, ticket);
    }
    int32_t lookup(int set) override
    {
        const ss_step_set &b = sets[set];
        return launch_forward(&tables, b.idx_c, B, L, b.n_kept, pooled, main);
    }
    int32_t update(int set, const float *grad, void *record_after) override
    {
        // the event rides on the update's last launch: no command of its own on the stream
        return launch_backward_apply(&tables, B, L, grad, lr, sets[set].ws_backward, main,
                                     static_cast<hipEvent_t>(record_after));
    }
    int32_t detect(float threshold) override
    {
        return launch_detect(&tables, hot_ids, H, snapshot, threshold, 1, stale_hot, drift,
                             stale_count, main);
    }
    int32_t new_event(void **ev) override
    {
        const int32_t rc = ss_event_create(ev);
        if (!rc) events.push_back(*ev);
        return rc;
    }
    int32_t record_now(void *ev, int s) override { return ss_event_record(ev, stream(s)); }
    bool done_now(void *ev) override
    {
        if (hipEventQuery(static_cast<hipEvent_t>(ev)) == hipSuccess) return true;
        (void)hipGetLastError();        // "not ready" is not an error to keep
        return false;
    }
    bool polls() const override { return true; }
    int32_t wait_now(int s, void *ev) override
    {
        // An event that has already happened needs no wait command on the stream (a
        // command that the stream would spend microseconds on between two kernels).
        // Every event that comes here has been recorded before: ss_step records its
        // own before it waits for them, through an issue queue only after the record
        // has been issued, and a caller's ready event is recorded before ss_step_submit.
        if (done_now(ev)) return SS_OK;
        return ss_stream_wait_event(stream(s), ev);
    }
    int32_t q_record(int q, void *ev, int s, uint64_t *t) override
    {
        return ss_issue_record_event(queues[q], ev, stream(s), t);
    }
    int32_t q_wait(int q, void *ev, int s, uint64_t *t) override
    {
        return ss_issue_wait_event(queues[q], ev, stream(s), t);
    }
    int32_t q_wait_issued(int q, uint64_t t) override { return ss_issue_wait(queues[q], t); }
    int32_t shutdown() override
    {
        int32_t rc = SS_OK;
        // every queued job issued and every thread ended before any event goes: a job
        // of one queue may name an event that another queue's marks own
        for (ss_issue_queue *q : queues) {
            const int32_t r = ss_issue_queue_destroy(q);
            if (r && !rc) rc = r;
        }
        queues.clear();
        for (hipStream_t s : sides) (void)hipStreamSynchronize(s);
        for (void *e : events) (void)ss_event_destroy(e);
        events.clear();
        for (hipStream_t s : sides) (void)hipStreamDestroy(s);
        sides.clear();
        return rc;
    }
    ~GpuOps() override { (void)shutdown(); }
};

// ---- operations handed to callbacks (the CPU model check) ------------------
struct TracedOps final : StepOps {
    ss_step_trace_ops cb;
    int next_event = 0;
    int32_t index_now(int s, int set, const int32_t *, void *done) override
    {
        const int32_t rc = cb.index_now(cb.user, s, set);
        if (rc || !done) return rc;
        return cb.record_now(cb.user, id(done), s);
    }
    int32_t q_index(int q, int s, int set, const int32_t *, void *done, uint64_t *t) override
    {
        const int32_t rc = cb.q_index(cb.user, q, s, set, t);
        if (rc || !done) return rc;
        return cb.q_record(cb.user, q, id(done), s, t);
    }
    int32_t lookup(int set) override { return cb.lookup(cb.user, set); }
    int32_t update(int set, const float *, void *record_after) override
    {
        const int32_t rc = cb.update(cb.user, set);
        if (rc || !record_after) return rc;
        return cb.record_now(cb.user, id(record_after), kMainStream);
    }
    int32_t detect(float thr) override { return cb.detect(cb.user, thr > 0.f ? 1 : 0); }
    int32_t new_event(void **ev) override
    {
        *ev = reinterpret_cast<void *>(static_cast<uintptr_t>(++next_event));
        return SS_OK;
    }
    static int id(void *ev) { return (int)reinterpret_cast<uintptr_t>(ev); }
    int32_t record_now(void *ev, int s) override { return cb.record_now(cb.user, id(ev), s); }
    int32_t wait_now(int s, void *ev) override { return cb.wait_now(cb.user, s, id(ev)); }
    bool done_now(void *) override { return false; }
    bool polls() const override { return false; }
    int32_t q_record(int q, void *ev, int s, uint64_t *t) override
    {
        return cb.q_record(cb.user, q, id(ev), s, t);
    }
    int32_t q_wait(int q, void *ev, int s, uint64_t *t) override
    {
        return cb.q_wait(cb.user, q, id(ev), s, t);
    }
    int32_t q_wait_issued(int q, uint64_t t) override { return cb.q_wait_issued(cb.user, q, t); }
    int32_t shutdown() override { return SS_OK; }
};

int32_t check_plan(const char *who, int32_t T, int32_t B, int32_t L, const ss_step_plan *p)
{
    if (!p) return fail(SS_ERR_INVALID_ARG, "%s: plan is NULL", who);
    if (T < 1 || T > 65535 || B < 1 || L < 1)
        return fail(SS_ERR_INVALID_ARG, "%s: T = %d, B = %d, L = %d", who, T, B, L);
    if (p->every < 1 || p->index_streams < 1 || p->index_streams > 16 || p->issue_threads < 0 ||
        p->issue_threads > p->index_streams || p->host_wait_us < 0)
        return fail(SS_ERR_INVALID_ARG,
                    "%s: every = %d, index_streams = %d, issue_threads = %d, host_wait_us = %d "
                    "(need every >= 1, 1 <= streams <= 16, 0 <= threads <= streams, "
                    "host_wait_us >= 0)",
                    who, p->every, p->index_streams, p->issue_threads, p->host_wait_us);
    if (p->num_sets != 3 * p->every * p->index_streams)
        return fail(SS_ERR_INVALID_ARG, "%s: num_sets = %d, need 3 * every * index_streams = %d",
                    who, p->num_sets, 3 * p->every * p->index_streams);
    return SS_OK;
}

// Builds the scheduler state around a table of operations.
int32_t make_step(std::unique_ptr<StepOps> ops, const ss_step_plan *plan, int32_t K,
                  float threshold, ss_step **out)
{
    std::unique_ptr<ss_step> st(new (std::nothrow) ss_step);
    if (!st) return fail(SS_ERR_HIP, "ss_step: out of host memory");
    st->ops = std::move(ops);
    st->every = plan->every;
    st->n_side = plan->index_streams;
    st->n_sets = plan->num_sets;
    st->n_queues = plan->issue_threads;
    st->host_wait_us = plan->host_wait_us;
    st->K = K;
    st->threshold = threshold;
    st->last_ticket.assign(std::max(1, st->n_queues), 0);
    st->indexed.resize(st->n_side);
    auto fill = [&](ss_step::Marks &m, int stream, bool by_queue, int waiters) -> int32_t {
        m.stream = stream;
        m.by_queue = by_queue;
        m.queue = st->queue_of(stream == kMainStream ? 0 : stream);
        m.known.assign(waiters, -1);
        for (int i = 0; i < kEventPool; ++i) {       // every event it will ever use, up front
            void *ev = nullptr;
            const int32_t rc = st->ops->new_event(&ev);
            if (rc) return rc;
            m.spare.push_back(ev);
        }
        return SS_OK;
    };
    for (int j = 0; j < st->n_side; ++j) {
        const int32_t rc = fill(st->indexed[j], j, true, 1);        // waited for by the training stream
        if (rc) return rc;
    }
    const int32_t rc = fill(st->trained, kMainStream, false, st->n_side);
    if (rc) return rc;
    if (st->host_wait_us > 0 && st->ops->polls())
        for (int i = 0; i < ss_step::kProgress; ++i) {
            void *ev = nullptr;
            const int32_t rc2 = st->ops->new_event(&ev);
            if (rc2) return rc2;
            st->progress_pool.push_back(ev);
        }
    *out = st.release();
    return SS_OK;
}

}  // namespace

}  // namespace ss

using namespace ss;

extern "C" {

int32_t ss_step_plan_for(int32_t T, int32_t B, int32_t L, ss_step_plan *plan)
{
    const char *who = "ss_step_plan_for";
    if (!plan) return fail(SS_ERR_INVALID_ARG, "%s: plan is NULL", who);
    if (T < 1 || T > 65535 || B < 1 || L < 1 || (int64_t)B * L >= (1LL << 31))
        return fail(SS_ERR_INVALID_ARG, "%s: T = %d, B = %d, L = %d", who, T, B, L);
    if (plan->dim < 0) return fail(SS_ERR_INVALID_ARG, "%s: dim = %d", who, plan->dim);
    if (plan->index_streams <= 0) plan->index_streams = auto_streams(T, B, L, plan->dim);
    if (plan->index_streams > 16)
        return fail(SS_ERR_INVALID_ARG, "%s: index_streams = %d (at most 16)", who,
                    plan->index_streams);
    if (plan->every <= 0) plan->every = auto_every(T, B, L, plan->index_streams);
    if (plan->issue_threads < 0) plan->issue_threads = auto_threads(T, B, L, plan->index_streams);
    if (plan->issue_threads > plan->index_streams) plan->issue_threads = plan->index_streams;
    if (plan->host_wait_us < 0) plan->host_wait_us = L > 1 ? 2000 : 0;
    plan->num_sets = 3 * plan->every * plan->index_streams;
    return SS_OK;
}

int32_t ss_step_create(const ss_tables *tables, int32_t B, int32_t L, int32_t alpha, float lr,
                       float threshold, int32_t snapshot_every, int32_t *const *hot_ids,
                       int32_t H, float **snapshot, uint8_t **stale_hot, double **drift,
                       uint32_t *stale_count, const ss_step_plan *plan, const ss_step_set *sets,
                       float *pooled, void *train_stream, ss_step **out)
{
    const char *who = "ss_step_create";
    if (!out) return fail(SS_ERR_INVALID_ARG, "%s: out is NULL", who);
    int32_t rc = check_tables(tables, who);
    if (rc) return rc;
    rc = check_plan(who, tables->num_tables, B, L, plan);
    if (rc) return rc;
    if (!tables->stale_bits)
        return fail(SS_ERR_INVALID_ARG, "%s: tables->stale_bits is NULL", who);
    if (!hot_ids || !snapshot || H < 1)
        return fail(SS_ERR_INVALID_ARG, "%s: hot_ids or snapshot is NULL, or H = %d", who, H);
    if (snapshot_every < 1)
        return fail(SS_ERR_INVALID_ARG, "%s: snapshot_every = %d", who, snapshot_every);
    if (threshold != threshold) return fail(SS_ERR_INVALID_ARG, "%s: threshold is NaN", who);
    if (!sets || !pooled) return fail(SS_ERR_INVALID_ARG, "%s: sets or pooled is NULL", who);
    if (reinterpret_cast<uintptr_t>(pooled) % 16 != 0)
        return fail(SS_ERR_INVALID_ARG, "%s: pooled is not 16-byte aligned", who);
    for (int i = 0; i < plan->num_sets; ++i) {
        const ss_step_set &b = sets[i];
        // (the index tensor comes with each batch: any other non-NULL address stands in)
        rc = check_filter(who, tables, reinterpret_cast<const int32_t *>(pooled), B, L,
                          b.skip_mask, b.kept_ids, b.n_kept, b.idx_c, b.ws_filter,
                          b.ws_filter_bytes);
        if (rc) return rc;
        rc = check_backward(who, tables, B, L, b.ws_backward, b.ws_backward_bytes);
        if (rc) return rc;
    }
    std::unique_ptr<GpuOps> ops(new (std::nothrow) GpuOps);
    if (!ops) return fail(SS_ERR_HIP, "%s: out of host memory", who);
    ops->tables = *tables;
    ops->B = B;
    ops->L = L;
    ops->alpha = alpha;
    ops->H = H;
    ops->lr = lr;
    ops->sets.assign(sets, sets + plan->num_sets);
    ops->hot_ids = hot_ids;
    ops->snapshot = snapshot;
    ops->stale_hot = stale_hot;
    ops->drift = drift;
    ops->stale_count = stale_count;
    ops->pooled = pooled;
    ops->main = static_cast<hipStream_t>(train_stream);
    for (int j = 0; j < plan->index_streams; ++j) {
        hipStream_t s = nullptr;
        // default priority; non-blocking, so that it never orders itself against the
        // legacy default stream
        if (hipStreamCreateWithFlags(&s, hipStreamNonBlocking) != hipSuccess)
            return fail(SS_ERR_HIP, "%s: hipStreamCreateWithFlags failed", who);
        ops->sides.push_back(s);
    }
    for (int q = 0; q < plan->issue_threads; ++q) {
        ss_issue_queue *iq = nullptr;
        rc = ss_issue_queue_create(&iq);
        if (rc) return rc;
        ops->queues.push_back(iq);
    }
    return make_step(std::move(ops), plan, snapshot_every, threshold, out);
}

int32_t ss_step_create_traced(const ss_step_plan *plan, int32_t snapshot_every,
                              const ss_step_trace_ops *callbacks, ss_step **out)
{
    const char *who = "ss_step_create_traced";
    if (!out || !callbacks) return fail(SS_ERR_INVALID_ARG, "%s: out or callbacks is NULL", who);
    int32_t rc = check_plan(who, 1, 1, 1, plan);
    if (rc) return rc;
    if (snapshot_every < 1)
        return fail(SS_ERR_INVALID_ARG, "%s: snapshot_every = %d", who, snapshot_every);
    std::unique_ptr<TracedOps> ops(new (std::nothrow) TracedOps);
    if (!ops) return fail(SS_ERR_HIP, "%s: out of host memory", who);
    ops->cb = *callbacks;
    return make_step(std::move(ops), plan, snapshot_every, 1.0f, out);
}

int32_t ss_step_destroy(ss_step *st)
{
    if (!st) return SS_OK;
    const int32_t rc = st->ops->shutdown();
    delete st;
    return rc;
}

int32_t ss_step_room(const ss_step *st) { return st ? st->room() : 0; }

int32_t ss_step_submit(ss_step *st, const int32_t *idx, void *ready_event)
{
    const char *who = "ss_step_submit";
    if (!st) return fail(SS_ERR_INVALID_ARG, "%s: step is NULL", who);
    if (!idx) return fail(SS_ERR_INVALID_ARG, "%s: idx is NULL", who);
    if (st->room() <= 0)
        return fail(SS_ERR_INVALID_ARG, "%s: too far ahead (see ss_step_room)", who);
    const int64_t k = st->submitted++;
    // a boundary batch before this one that has not had its update yet?
    if (!st->held_back.empty() || st->boundary_in(st->it, k)) {
        st->held_back.push_back(ss_step::Held{idx, ready_event});
        return st->drain(2);
    }
    return st->issue(k, idx, ready_event);
}

int32_t ss_step_forward(ss_step *st, int32_t *set_used)
{
    const char *who = "ss_step_forward";
    if (!st) return fail(SS_ERR_INVALID_ARG, "%s: step is NULL", who);
    const int64_t k = st->forwarded;
    if (k == st->it && k >= st->issued) {       // the batch may be waiting among the held ones
        const int32_t rc = st->drain(1);
        if (rc) return rc;
    }
    if (k != st->it || k >= st->issued)
        return fail(SS_ERR_INVALID_ARG,
                    "%s: needs a submitted batch and the previous batch finished", who);
    const int set = (int)(k % st->n_sets), j = (int)(k % st->n_side);
    int32_t rc = st->cover_indexed(j, k);
    if (rc) return rc;
    ++st->forwarded;
    if (set_used) *set_used = set;
    return st->ops->lookup(set);
}

int32_t ss_step_backward(ss_step *st, const float *grad, int32_t *detected)
{
    const char *who = "ss_step_backward";
    if (!st) return fail(SS_ERR_INVALID_ARG, "%s: step is NULL", who);
    if (st->forwarded != st->it + 1)
        return fail(SS_ERR_INVALID_ARG, "%s: follows ss_step_forward", who);
    if (!grad) return fail(SS_ERR_INVALID_ARG, "%s: grad is NULL", who);
    if (reinterpret_cast<uintptr_t>(grad) % 16 != 0)
        return fail(SS_ERR_INVALID_ARG, "%s: grad is not 16-byte aligned", who);
    const int64_t k = st->it;
    // Every `every`-th batch the training stream leaves an event for the index streams
    // (a buffer set is free again once its batch has been trained on).  Without a
    // detect pass behind it the update's last launch carries the event.
    const bool mark = (k + 1) % st->every == 0;
    void *rides = nullptr;
    if (mark && !st->boundary(k) && !st->trained.spare.empty()) {
        rides = st->trained.spare.back();
        st->trained.spare.pop_back();
    }
    // every other update carries an event that only tells the calling thread how far
    // the training stream has got (poll_indexed)
    void *tells = rides;
    if (!tells && !st->progress_pool.empty()) tells = st->progress_pool[k % ss_step::kProgress];
    int32_t rc = st->ops->update((int)(k % st->n_sets), grad, tells);
    if (rc) {
        if (rides) st->trained.spare.push_back(rides);
        return rc;
    }
    st->progress[k % ss_step::kProgress] = tells;
    if (rides) st->keep(st->trained, k, rides, 0);
    int32_t det = 0;
    if (st->boundary(k)) {
        // the first period is the warm-up: its end captures the first snapshot
        rc = st->ops->detect(st->have_snapshot ? st->threshold : 0.0f);
        if (rc) return rc;
        det = st->have_snapshot ? 1 : 0;
        st->have_snapshot = true;
        st->last_detect = k;
    }
    ++st->it;
    if (mark && !rides) {
        rc = st->record(st->trained, k);
        if (rc) return rc;
    }
    if (detected) *detected = det;
    // batches that waited for a detect pass (this one's, or an earlier one's)
    return st->drain(2);
}

int32_t ss_step_counters(const ss_step *st, int64_t *out)
{
    if (!st || !out) return fail(SS_ERR_INVALID_ARG, "ss_step_counters: step or out is NULL");
    out[0] = st->forwarded;
    out[1] = st->n_wait_cmds;
    out[2] = st->n_polls;
    out[3] = st->n_polls_done;
    return SS_OK;
}

int32_t ss_step_flush(ss_step *st)
{
    if (!st) return fail(SS_ERR_INVALID_ARG, "ss_step_flush: step is NULL");
    for (int q = 0; q < st->n_queues; ++q)
        if (st->last_ticket[q]) {
            const int32_t rc = st->ops->q_wait_issued(q, st->last_ticket[q]);
            if (rc) return rc;
        }
    return SS_OK;
}

}  // extern "C"
