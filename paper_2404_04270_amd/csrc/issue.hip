// ss_issue_queue: a host thread that enqueues library work on HIP streams.
//
// Enqueueing a kernel costs the calling host thread about 3 us on this
// platform, whatever the kernel does.  The index work of a batch (section 3.4 of
// the paper: the input classifier, plus the grouping half of the update) is up
// to eight launches, the training kernels three: at shapes whose kernels are
// short (one huge table; any shape once most hot rows are frozen) one host
// thread cannot enqueue a batch as fast as the GPU finishes it.  Two host
// threads enqueue on two streams at full rate each (measured: 2.8 us per launch
// alone, 1.5 us per launch overall with two threads), so the index work gets a
// thread of its own.
//
// The queue holds three kinds of job, issued in the order they were submitted:
// the index work of a batch, "make this stream wait for that event", and "record
// this event on that stream".  Nothing here touches device memory or waits for
// the GPU; ss_issue_wait() waits for the host thread to have ISSUED a job, which
// is what a caller needs before it makes another stream wait for an event that
// the queue records.
#include <condition_variable>
#include <deque>
#include <mutex>
#include <new>
#include <string>
#include <thread>

#include "ss_common.h"

namespace ss {

namespace {

enum JobKind { kIndexBatch, kWaitEvent, kRecordEvent };

struct Job {
    JobKind kind;
    hipStream_t stream;
    hipEvent_t event;
    // index batch
    ss_tables tables;
    const int32_t *idx;
    int32_t B, L, alpha;
    uint8_t *skip_mask;
    int32_t *kept_ids, *n_kept, *idx_c;
    void *ws_filter, *ws_backward;
};

}  // namespace

}  // namespace ss

struct ss_issue_queue {
    std::thread thread;
    std::mutex mu;
    std::condition_variable have_job, job_issued;
    std::deque<ss::Job> jobs;
    uint64_t submitted = 0, issued = 0;     // tickets are 1-based job numbers
    int32_t first_error = 0;
    std::string first_error_text;
    bool stop = false;
    int device = 0;
};

namespace ss {

namespace {

void run_job(ss_issue_queue *q, const Job &j)
{
    int32_t rc = SS_OK;
    const char *who = "ss_issue_queue";
    switch (j.kind) {
    case kWaitEvent:
        if (hipStreamWaitEvent(j.stream, j.event, 0) != hipSuccess)
            rc = fail(SS_ERR_HIP, "%s: hipStreamWaitEvent failed", who);
        else
            after_stream_wait(j.stream);
        break;
    case kRecordEvent:
        if (hipEventRecord(j.event, j.stream) != hipSuccess)
            rc = fail(SS_ERR_HIP, "%s: hipEventRecord failed", who);
        break;
    case kIndexBatch:
        rc = checked_indices(who, j.tables.num_tables, j.tables.rows, j.idx, j.B, j.L, nullptr,
                             j.stream);
        if (rc != SS_OK) break;
        rc = launch_filter(&j.tables, j.idx, j.B, j.L, j.alpha, j.skip_mask, j.kept_ids,
                           j.n_kept, j.idx_c, j.ws_filter, j.stream);
        if (rc == SS_OK)
            rc = launch_backward_prepare(&j.tables, j.idx_c, j.B, j.L, j.n_kept,
                                         j.ws_backward, j.stream, j.event);
        break;
    }
    std::lock_guard<std::mutex> lk(q->mu);
    if (rc != SS_OK && q->first_error == SS_OK) {
        q->first_error = rc;
        q->first_error_text = ss_last_error();    // this thread's text
    }
    ++q->issued;
}

void worker(ss_issue_queue *q)
{
    (void)hipSetDevice(q->device);
    for (;;) {
        Job j;
        {
            std::unique_lock<std::mutex> lk(q->mu);
            q->have_job.wait(lk, [q] { return q->stop || !q->jobs.empty(); });
            if (q->jobs.empty()) return;          // stop, and nothing left to issue
            j = q->jobs.front();
            q->jobs.pop_front();
        }
        run_job(q, j);
        q->job_issued.notify_all();
    }
}

int32_t push(ss_issue_queue *q, const Job &j, uint64_t *ticket)
{
    {
        std::lock_guard<std::mutex> lk(q->mu);
        if (q->stop) return fail(SS_ERR_INVALID_ARG, "ss_issue_queue: queue is shut down");
        q->jobs.push_back(j);
        ++q->submitted;
        if (ticket) *ticket = q->submitted;
    }
    q->have_job.notify_one();
    return SS_OK;
}

}  // namespace

}  // namespace ss

using namespace ss;

extern "C" {

int32_t ss_issue_queue_create(ss_issue_queue **out)
{
    if (!out) return fail(SS_ERR_INVALID_ARG, "ss_issue_queue_create: out is NULL");
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess)
        return fail(SS_ERR_HIP, "ss_issue_queue_create: no current device");
    ss_issue_queue *q = new (std::nothrow) ss_issue_queue;
    if (!q) return fail(SS_ERR_HIP, "ss_issue_queue_create: out of host memory");
    q->device = dev;
    q->thread = std::thread(worker, q);
    *out = q;
    return SS_OK;
}

int32_t ss_issue_queue_destroy(ss_issue_queue *q)
{
    if (!q) return SS_OK;
    {
        std::lock_guard<std::mutex> lk(q->mu);
        q->stop = true;
    }
    q->have_job.notify_all();
    if (q->thread.joinable()) q->thread.join();      // issues what is still queued
    delete q;
    return SS_OK;
}

int32_t ss_issue_index_batch(ss_issue_queue *q, const ss_tables *tables,
                             const int32_t *idx, int32_t B, int32_t L, int32_t alpha,
                             uint8_t *skip_mask, int32_t *kept_ids, int32_t *n_kept,
                             int32_t *idx_c, void *ws_filter, size_t ws_filter_bytes,
                             void *ws_backward, size_t ws_backward_bytes, void *stream,
                             uint64_t *ticket)
{
    return ss::issue_index_batch(q, tables, idx, B, L, alpha, skip_mask, kept_ids, n_kept, idx_c,
                                 ws_filter, ws_filter_bytes, ws_backward, ws_backward_bytes,
                                 stream, nullptr, ticket);
}

}  // extern "C"

int32_t ss::issue_index_batch(ss_issue_queue *q, const ss_tables *tables, const int32_t *idx,
                              int32_t B, int32_t L, int32_t alpha, uint8_t *skip_mask,
                              int32_t *kept_ids, int32_t *n_kept, int32_t *idx_c,
                              void *ws_filter, size_t ws_filter_bytes, void *ws_backward,
                              size_t ws_backward_bytes, void *stream, void *record_after,
                              uint64_t *ticket)
{
    const char *who = "ss_issue_index_batch";
    if (!q) return fail(SS_ERR_INVALID_ARG, "%s: queue is NULL", who);
    int32_t rc = check_filter(who, tables, idx, B, L, skip_mask, kept_ids, n_kept, idx_c,
                              ws_filter, ws_filter_bytes);
    if (rc) return rc;
    rc = check_backward(who, tables, B, L, ws_backward, ws_backward_bytes);
    if (rc) return rc;
    Job j{};
    j.kind = kIndexBatch;
    j.stream = static_cast<hipStream_t>(stream);
    j.tables = *tables;
    j.idx = idx;
    j.B = B;
    j.L = L;
    j.alpha = alpha;
    j.skip_mask = skip_mask;
    j.kept_ids = kept_ids;
    j.n_kept = n_kept;
    j.idx_c = idx_c;
    j.ws_filter = ws_filter;
    j.ws_backward = ws_backward;
    j.event = static_cast<hipEvent_t>(record_after);
    return push(q, j, ticket);
}

extern "C" {

int32_t ss_issue_wait_event(ss_issue_queue *q, void *event, void *stream, uint64_t *ticket)
{
    if (!q || !event)
        return fail(SS_ERR_INVALID_ARG, "ss_issue_wait_event: queue or event is NULL");
    Job j{};
    j.kind = kWaitEvent;
    j.stream = static_cast<hipStream_t>(stream);
    j.event = static_cast<hipEvent_t>(event);
    return push(q, j, ticket);
}

int32_t ss_issue_record_event(ss_issue_queue *q, void *event, void *stream,
                              uint64_t *ticket)
{
    if (!q || !event)
        return fail(SS_ERR_INVALID_ARG, "ss_issue_record_event: queue or event is NULL");
    Job j{};
    j.kind = kRecordEvent;
    j.stream = static_cast<hipStream_t>(stream);
    j.event = static_cast<hipEvent_t>(event);
    return push(q, j, ticket);
}

int32_t ss_issue_wait(ss_issue_queue *q, uint64_t ticket)
{
    if (!q) return fail(SS_ERR_INVALID_ARG, "ss_issue_wait: queue is NULL");
    std::unique_lock<std::mutex> lk(q->mu);
    if (ticket > q->submitted)
        return fail(SS_ERR_INVALID_ARG, "ss_issue_wait: no such job");
    q->job_issued.wait(lk, [q, ticket] { return q->issued >= ticket; });
    if (q->first_error != SS_OK)
        return fail(q->first_error, "%s", q->first_error_text.c_str());
    return SS_OK;
}

int32_t ss_event_create(void **event)
{
    if (!event) return fail(SS_ERR_INVALID_ARG, "ss_event_create: event is NULL");
    hipEvent_t e;
    // Device-scope release: these events order streams of one device.  The default
    // (a system-scope fence, for the host's benefit) writes caches back and
    // invalidates them at every record, which the kernels that follow pay for.
    if (hipEventCreateWithFlags(&e, hipEventDisableTiming | hipEventReleaseToDevice) !=
        hipSuccess)
        return fail(SS_ERR_HIP, "ss_event_create: hipEventCreateWithFlags failed");
    *event = e;
    return SS_OK;
}

int32_t ss_event_destroy(void *event)
{
    if (event && hipEventDestroy(static_cast<hipEvent_t>(event)) != hipSuccess)
        return fail(SS_ERR_HIP, "ss_event_destroy: hipEventDestroy failed");
    return SS_OK;
}

int32_t ss_event_record(void *event, void *stream)
{
    if (!event) return fail(SS_ERR_INVALID_ARG, "ss_event_record: event is NULL");
    if (hipEventRecord(static_cast<hipEvent_t>(event), static_cast<hipStream_t>(stream)) !=
        hipSuccess)
        return fail(SS_ERR_HIP, "ss_event_record: hipEventRecord failed");
    return SS_OK;
}

int32_t ss_stream_wait_event(void *stream, void *event)
{
    if (!event) return fail(SS_ERR_INVALID_ARG, "ss_stream_wait_event: event is NULL");
    if (hipStreamWaitEvent(static_cast<hipStream_t>(stream), static_cast<hipEvent_t>(event),
                           0) != hipSuccess)
        return fail(SS_ERR_HIP, "ss_stream_wait_event: hipStreamWaitEvent failed");
    after_stream_wait(static_cast<hipStream_t>(stream));
    return SS_OK;
}

}  // extern "C"
