// Asynchronous scheduler of libhzp: the multi-stream dispatch of Section 4.2 for the local halves
// of the collectives.
//
// What the paper describes and what is kept here:
//   - parameter all-gathers and gradient reduce-scatters are issued from an extra host thread on
//     dedicated streams, so that issuing them never blocks the thread that drives the compute
//     stream and puts nothing on that stream at issue time;
//   - all-gather results live in a pre-allocated, fixed-capacity, persistent pool: one contiguous
//     buffer used as a ring by this one kind of operation.  A prefetch takes the next region of
//     the ring (a whole layer bucket, or a single parameter: the paper launches communication at
//     parameter granularity), a release gives the oldest region back, so the live data is always
//     one run of the ring and the only space lost is what is skipped where a region does not fit
//     before the end of the buffer;
//   - parameters are pre-launched ahead of their use (prefetch) and gradients are consumed as
//     soon as they exist ("hungrily").
// Ordering between the side streams and the consumer's stream is carried by events: the consumer
// waits for a region's `ready` event when it acquires it, and the gather stream waits for the
// events that mark the last use of every earlier region a new one overlaps.  Host-side waits
// carry a time limit and turn into an error status instead of hanging.
#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <chrono>
#include <cstdio>
#include <condition_variable>
#include <deque>
#include <new>
#include <thread>

#include "hzp_internal.hpp"

using namespace hzp;

namespace {

constexpr auto kHostWaitLimit = std::chrono::seconds(30);
constexpr uint64_t kTensorKey = 1ull << 32;     // keys: layer, or kTensorKey | tensor id
constexpr size_t kFreedSweep = 64;              // sweep finished entries when the list grows past this

enum AllocState { A_ASSIGNED, A_READY, A_ACQUIRED, A_RELEASED };

// A region of the ring between prefetch and release, oldest first in hzp_sched::live.
struct Alloc {
    uint64_t key = 0;
    uint64_t off = 0, bytes = 0;    // position in the pool; bytes is a multiple of 256
    uint64_t payload = 0;           // bytes of the bucket or tensor held
    AllocState state = A_ASSIGNED;
    hipEvent_t ready = nullptr;     // recorded on the gather stream behind the gather
};

// A region that was given back; `ev` marks the consumer's last use of it.
struct FreedRegion {
    uint64_t off, bytes;
    hipEvent_t ev;
};

struct Cmd {
    enum Kind { PREFETCH, REDUCE, FENCE, STOP } kind = STOP;
    // PREFETCH
    uint64_t key = 0;
    uint32_t id = 0;                // layer or tensor id (REDUCE: layer)
    bool is_tensor = false;
    uint64_t off = 0;               // destination in the pool
    hipEvent_t ready = nullptr;
    std::vector<hipEvent_t> wait;   // last uses of the regions the destination overlaps
    // REDUCE
    uint32_t R = 0, grad_dtype = 0, rank = 0;
    int level = 0, accumulate = 0;
    float scale = 1.0f;
    float *out = nullptr;
    hipEvent_t after = nullptr;     // both kinds: recorded on the producer's stream at submission
    std::vector<const void *> ptrs; // both kinds
};

}  // namespace

struct hzp_sched {
    const hzp_plan_t *plan = nullptr;
    uint32_t cls = 0, max_live = 0, queue_capacity = 0;
    int device = 0;
    uint64_t pool_bytes = 0;
    uint64_t uniform_bytes = 0;                 // non-zero: every region takes this much (equal slots)
    char *pool = nullptr;
    hipStream_t gather_stream = nullptr, reduce_stream = nullptr;
    std::deque<Alloc> live;                     // ring order: front is the oldest region
    std::vector<FreedRegion> freed;
    std::deque<Cmd> queue;
    std::vector<hipEvent_t> spare_events;
    hipEvent_t fence_gather = nullptr, fence_reduce = nullptr;
    uint64_t submitted = 0, processed = 0;
    hzp_status_t failed = HZP_OK;
    char fail_text[256] = "";
    hzp_sched_stats_t stats{};
    std::mutex mu;
    std::condition_variable cv;
    std::thread worker;

    void set_failed(hzp_status_t st, const char *text)
    {
        if (failed == HZP_OK) {
            failed = st;
            snprintf(fail_text, sizeof fail_text, "%s", text);
        }
        cv.notify_all();
    }
    // The region held for `key`, if it is between prefetch and release.  Caller holds the lock.
    Alloc *find(uint64_t key)
    {
        for (Alloc &a : live)
            if (a.key == key && a.state != A_RELEASED) return &a;
        return nullptr;
    }
};

namespace {

hzp_status_t hip_fail(hzp_sched *s, const char *what, hipError_t e)
{
    char text[256];
    snprintf(text, sizeof text, "%s: %s", what, hipGetErrorString(e));
    s->set_failed(HZP_ERR_HIP, text);
    return fail(HZP_ERR_HIP, "%s", text);
}

// An event from the spare list, or a new one.  Caller holds the lock.
hipError_t take_event(hzp_sched *s, hipEvent_t *ev)
{
    if (!s->spare_events.empty()) {
        *ev = s->spare_events.back();
        s->spare_events.pop_back();
        return hipSuccess;
    }
    return hipEventCreateWithFlags(ev, hipEventDisableTiming);
}

// The live run of the ring: [tail, head) if head > tail, else [tail, cap) and [0, head).
struct RingSpan {
    bool empty;
    uint64_t tail, head;
};

RingSpan ring_span(const hzp_sched *s)
{
    if (s->live.empty()) return RingSpan{true, 0, 0};
    return RingSpan{false, s->live.front().off, s->live.back().off + s->live.back().bytes};
}

// Next region of the ring for `bytes`, or false if the live data leaves no room.  `skipped` is the
// space lost at the end of the buffer when the region has to start over at offset 0.
bool ring_take(uint64_t cap, const RingSpan &r, uint64_t bytes, uint64_t *off, uint64_t *skipped)
{
    *skipped = 0;
    if (bytes > cap) return false;
    if (r.empty) {
        *off = 0;
        return true;
    }
    if (r.head > r.tail) {                  // live data is the single run [tail, head)
        if (r.head + bytes <= cap) {
            *off = r.head;
            return true;
        }
        if (bytes <= r.tail) {              // start over; [head, cap) stays unused this time round
            *off = 0;
            *skipped = cap - r.head;
            return true;
        }
        return false;
    }
    if (r.head + bytes <= r.tail) {         // live data wraps: [tail, cap) and [0, head)
        *off = r.head;
        return true;
    }
    return false;
}

// Background thread: takes commands in submission order and launches them on the side streams.
void worker_main(hzp_sched *s)
{
    (void)hipSetDevice(s->device);
    for (;;) {
        Cmd cmd;
        {
            std::unique_lock<std::mutex> lock(s->mu);
            s->cv.wait(lock, [&] { return !s->queue.empty(); });
            cmd = std::move(s->queue.front());
            s->queue.pop_front();
        }
        if (cmd.kind == Cmd::STOP) break;
        if (cmd.kind == Cmd::PREFETCH) {
            // The shards exist once the producer's work enqueued before the prefetch has run.
            // (a command that follows another of the same submission carries no event of its own)
            hipError_t e = cmd.after ? hipStreamWaitEvent(s->gather_stream, cmd.after, 0) : hipSuccess;
            for (hipEvent_t ev : cmd.wait)          // earlier users of this part of the ring
                if (e == hipSuccess) e = hipStreamWaitEvent(s->gather_stream, ev, 0);
            hzp_status_t st = HZP_OK;
            if (e == hipSuccess) {
                char *dst = s->pool + cmd.off;
                if (cmd.is_tensor) {
                    st = hzp_gather_tensor(s->plan, cmd.id, cmd.ptrs.data(), (uint32_t)cmd.ptrs.size(), dst,
                                           s->gather_stream);
                } else {
                    st = hzp_gather_layer(s->plan, cmd.id, s->cls, 3, cmd.ptrs.data(), (uint32_t)cmd.ptrs.size(),
                                          dst, nullptr, s->gather_stream);
                }
            }
            if (e == hipSuccess && st == HZP_OK) e = hipEventRecord(cmd.ready, s->gather_stream);
            std::lock_guard<std::mutex> lock(s->mu);
            if (cmd.after) s->spare_events.push_back(cmd.after);
            for (hipEvent_t ev : cmd.wait) s->spare_events.push_back(ev);   // their waits are enqueued: reusable
            if (e != hipSuccess || st != HZP_OK) {
                s->set_failed(st != HZP_OK ? st : HZP_ERR_HIP, st != HZP_OK ? hzp_last_error() : hipGetErrorString(e));
            } else {
                Alloc *a = s->find(cmd.key);        // still there: it cannot be released before it is acquired
                if (a) a->state = A_READY;
                s->stats.gathers_issued++;
            }
        } else if (cmd.kind == Cmd::REDUCE) {
            hipError_t e = hipStreamWaitEvent(s->reduce_stream, cmd.after, 0);
            hzp_status_t st = HZP_OK;
            if (e == hipSuccess)
                st = hzp_reduce_shard(s->plan, cmd.id, s->cls, cmd.level, cmd.rank, cmd.ptrs.data(), cmd.R,
                                      cmd.grad_dtype, cmd.scale, cmd.accumulate, cmd.out, s->reduce_stream);
            std::lock_guard<std::mutex> lock(s->mu);
            s->spare_events.push_back(cmd.after);       // its wait has been enqueued: reusable
            if (e != hipSuccess || st != HZP_OK)
                s->set_failed(st != HZP_OK ? st : HZP_ERR_HIP, st != HZP_OK ? hzp_last_error() : hipGetErrorString(e));
            else
                s->stats.reduces_issued++;
        } else if (cmd.kind == Cmd::FENCE) {
            hipError_t e = hipEventRecord(s->fence_gather, s->gather_stream);
            if (e == hipSuccess) e = hipEventRecord(s->fence_reduce, s->reduce_stream);
            if (e != hipSuccess) {
                std::lock_guard<std::mutex> lock(s->mu);
                s->set_failed(HZP_ERR_HIP, hipGetErrorString(e));
            }
        }
        {
            std::lock_guard<std::mutex> lock(s->mu);
            s->processed++;
        }
        s->cv.notify_all();
    }
}

// Queue a command; blocks (with the time limit) while the queue is full.  `cmd` is moved from
// only if the call succeeds.
hzp_status_t submit(hzp_sched *s, std::unique_lock<std::mutex> &lock, Cmd &cmd, uint64_t *seq)
{
    bool ok = s->cv.wait_for(lock, kHostWaitLimit,
                             [&] { return s->failed != HZP_OK || s->queue.size() < s->queue_capacity; });
    if (s->failed != HZP_OK) return fail(s->failed, "scheduler failed earlier: %s", s->fail_text);
    if (!ok) return fail(HZP_ERR_HIP, "scheduler: command queue stayed full for the time limit");
    s->queue.push_back(std::move(cmd));
    s->submitted++;
    if (seq) *seq = s->submitted;
    s->cv.notify_all();
    return HZP_OK;
}

// Drop entries of the freed list whose consumers have finished (keeps the list short when regions
// of many different sizes move through the ring).  Caller holds the lock.
void sweep_freed(hzp_sched *s)
{
    size_t kept = 0;
    for (size_t i = 0; i < s->freed.size(); ++i) {
        if (hipEventQuery(s->freed[i].ev) == hipSuccess)
            s->spare_events.push_back(s->freed[i].ev);
        else
            s->freed[kept++] = s->freed[i];
    }
    s->freed.resize(kept);
}

// Common part of the prefetch calls; `ptrs` have been validated and the caller holds the lock.
// `mark_producer`: record an event on the producer's stream for the gather to wait for (the later
// commands of one submission are ordered behind the first on the gather stream and need none).
hzp_status_t prefetch_region(hzp_sched *s, std::unique_lock<std::mutex> &lock, const char *who, uint64_t key,
                             bool is_tensor, uint32_t id, uint64_t payload, const void *const *ptrs, uint32_t n,
                             hipStream_t producer, bool mark_producer)
{
    if (s->failed != HZP_OK) return fail(s->failed, "scheduler failed earlier: %s", s->fail_text);
    if (s->find(key)) return fail(HZP_ERR_INVALID_ARG, "%s %u is already in the pool", who, id);
    if (s->live.size() >= s->max_live)
        return fail(HZP_ERR_NOMEM, "%s %u: %u regions are between prefetch and release already", who, id, s->max_live);
    const uint64_t bytes = s->uniform_bytes ? s->uniform_bytes : (payload + 255) / 256 * 256;
    uint64_t off = 0, skipped = 0;
    if (!ring_take(s->pool_bytes, ring_span(s), bytes, &off, &skipped))
        return fail(HZP_ERR_NOMEM, "%s %u: the pool has no room for %llu bytes until older regions are released; "
                                   "release in the order of the prefetches", who, id, (unsigned long long)bytes);
    Cmd cmd;
    cmd.kind = Cmd::PREFETCH;
    cmd.key = key;
    cmd.id = id;
    cmd.is_tensor = is_tensor;
    cmd.off = off;
    cmd.ptrs.assign(ptrs, ptrs + n);
    hipError_t e = take_event(s, &cmd.ready);
    if (e != hipSuccess) return hip_fail(s, who, e);
    if (mark_producer) {
        e = take_event(s, &cmd.after);
        if (e == hipSuccess) {
            e = hipEventRecord(cmd.after, producer);
            if (e != hipSuccess) s->spare_events.push_back(cmd.after);
        }
        if (e != hipSuccess) {
            s->spare_events.push_back(cmd.ready);
            cmd.after = nullptr;
            return hip_fail(s, who, e);
        }
    }
    const hipEvent_t after = cmd.after;
    // The gather must run after the last use of everything that lay in [off, off+bytes) before.
    std::vector<FreedRegion> taken;
    size_t kept = 0;
    for (size_t i = 0; i < s->freed.size(); ++i) {
        const FreedRegion f = s->freed[i];
        if (f.off < off + bytes && off < f.off + f.bytes) {
            cmd.wait.push_back(f.ev);
            taken.push_back(f);
        } else {
            s->freed[kept++] = f;
        }
    }
    s->freed.resize(kept);
    Alloc a;
    a.key = key;
    a.off = off;
    a.bytes = bytes;
    a.payload = payload;
    a.state = A_ASSIGNED;
    a.ready = cmd.ready;
    s->live.push_back(a);           // in place before the background thread can see the command
    hzp_status_t st = submit(s, lock, cmd, nullptr);
    if (st != HZP_OK) {             // not queued: undo
        s->live.pop_back();
        s->spare_events.push_back(a.ready);
        if (after) s->spare_events.push_back(after);
        s->freed.insert(s->freed.end(), taken.begin(), taken.end());
        return st;
    }
    s->stats.wrap_skipped_bytes += skipped;
    uint64_t live_bytes = 0;
    uint32_t live_count = 0;
    for (const Alloc &x : s->live)
        if (x.state != A_RELEASED) {
            live_bytes += x.payload;
            live_count++;
        }
    s->stats.peak_live_bytes = std::max(s->stats.peak_live_bytes, live_bytes);
    s->stats.peak_live_slots = std::max(s->stats.peak_live_slots, live_count);
    return HZP_OK;
}

hzp_status_t acquire_region(hzp_sched *s, const char *who, uint64_t key, uint32_t id, hipStream_t consumer, void **out)
{
    std::unique_lock<std::mutex> lock(s->mu);
    Alloc *a = s->find(key);
    if (!a) return fail(HZP_ERR_INVALID_ARG, "%s %u was not prefetched", who, id);
    if (a->state == A_ACQUIRED) return fail(HZP_ERR_INVALID_ARG, "%s %u is already acquired", who, id);
    // Host-side wait until the background thread has launched the gather (not until it has run).
    const auto t0 = std::chrono::steady_clock::now();
    bool ok = s->cv.wait_for(lock, kHostWaitLimit, [&] {
        const Alloc *x = s->find(key);
        return s->failed != HZP_OK || (x && x->state == A_READY);
    });
    s->stats.acquire_host_wait_us += (uint64_t)std::chrono::duration_cast<std::chrono::microseconds>(
                                         std::chrono::steady_clock::now() - t0).count();
    if (s->failed != HZP_OK) return fail(s->failed, "scheduler failed earlier: %s", s->fail_text);
    if (!ok) {
        s->set_failed(HZP_ERR_HIP, "scheduler: a prefetch was not issued within the time limit");
        return fail(HZP_ERR_HIP, "%s", s->fail_text);
    }
    a = s->find(key);
    hipError_t e = hipStreamWaitEvent(consumer, a->ready, 0);
    if (e != hipSuccess) return hip_fail(s, who, e);
    a->state = A_ACQUIRED;
    *out = s->pool + a->off;
    return HZP_OK;
}

hzp_status_t release_region(hzp_sched *s, const char *who, uint64_t key, uint32_t id, hipStream_t consumer)
{
    std::unique_lock<std::mutex> lock(s->mu);
    Alloc *a = s->find(key);
    if (!a || a->state != A_ACQUIRED) return fail(HZP_ERR_INVALID_ARG, "%s %u is not acquired", who, id);
    hipEvent_t ev = nullptr;
    hipError_t e = take_event(s, &ev);
    if (e == hipSuccess) {
        e = hipEventRecord(ev, consumer);
        if (e != hipSuccess) s->spare_events.push_back(ev);
    }
    if (e != hipSuccess) return hip_fail(s, who, e);
    if (s->freed.size() >= kFreedSweep) sweep_freed(s);
    s->freed.push_back(FreedRegion{a->off, a->bytes, ev});
    s->spare_events.push_back(a->ready);        // the consumer's wait on it was enqueued at acquire
    a->ready = nullptr;
    a->state = A_RELEASED;
    // The ring gives space back oldest first: a region released out of order stays in place until
    // everything older has been released too.
    while (!s->live.empty() && s->live.front().state == A_RELEASED) s->live.pop_front();
    s->cv.notify_all();
    return HZP_OK;
}

}  // namespace

extern "C" hzp_status_t hzp_sched_create(const hzp_plan_t *plan, const hzp_sched_desc_t *d, hzp_sched_t **out)
{
    if (!plan || !d || !out) return fail(HZP_ERR_INVALID_ARG, "hzp_sched_create: NULL argument");
    *out = nullptr;
    if (d->cls > 1) return fail(HZP_ERR_RANGE, "hzp_sched_create: class %u", d->cls);
    if (d->gather_slots == 0 || d->queue_capacity == 0)
        return fail(HZP_ERR_INVALID_ARG, "hzp_sched_create: needs at least one pool slot and one queue entry");
    if (d->pool_bytes % 256 != 0)
        return fail(HZP_ERR_INVALID_ARG, "hzp_sched_create: pool_bytes must be a multiple of 256");
    uint64_t max_p = 0;
    for (const BucketRec &b : plan->buckets)
        if (b.cls == d->cls) max_p = std::max(max_p, b.P);
    if (max_p == 0) return fail(HZP_ERR_RANGE, "hzp_sched_create: the plan has no bucket of class %u", d->cls);
    const uint64_t slot_bytes = (max_p * (d->cls == HZP_CLASS_F32 ? 4 : 2) + 255) / 256 * 256;
    hzp_sched *s = new (std::nothrow) hzp_sched;
    if (!s) return fail(HZP_ERR_NOMEM, "hzp_sched_create: out of host memory");
    s->plan = plan;
    s->cls = d->cls;
    s->max_live = d->gather_slots;
    s->queue_capacity = d->queue_capacity;
    // Without an explicit size the ring is cut into equal slots of the largest bucket, so that any
    // `gather_slots` regions fit whatever their sizes; with one, a region takes its own size.
    s->pool_bytes = d->pool_bytes ? d->pool_bytes : slot_bytes * d->gather_slots;
    s->uniform_bytes = d->pool_bytes ? 0 : slot_bytes;
    // The plan's device tables are made here, so that no gather launched by the background thread
    // has to allocate or block.
    hzp_status_t pst = hzp_plan_prepare(plan, nullptr);
    if (pst != HZP_OK) {
        delete s;
        return pst;
    }
    hipError_t e = hipGetDevice(&s->device);
    // One allocation for the whole pool: contiguous, never freed or grown until destroy.
    if (e == hipSuccess) e = hipMalloc((void **)&s->pool, s->pool_bytes);
    if (e == hipSuccess) e = hipStreamCreateWithFlags(&s->gather_stream, hipStreamNonBlocking);
    if (e == hipSuccess) e = hipStreamCreateWithFlags(&s->reduce_stream, hipStreamNonBlocking);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&s->fence_gather, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&s->fence_reduce, hipEventDisableTiming);
    if (e != hipSuccess) {
        const hzp_status_t st = fail(e == hipErrorOutOfMemory ? HZP_ERR_NOMEM : HZP_ERR_HIP, "hzp_sched_create: %s",
                                     hipGetErrorString(e));
        hzp_sched_destroy(s);
        return st;
    }
    s->stats.pool_bytes = s->pool_bytes;
    s->stats.slot_bytes = slot_bytes;
    s->worker = std::thread(worker_main, s);
    *out = s;
    return HZP_OK;
}

extern "C" void hzp_sched_destroy(hzp_sched_t *s)
{
    if (!s) return;
    if (s->worker.joinable()) {
        {
            // Commands still queued are launched first, then the thread leaves.
            std::lock_guard<std::mutex> lock(s->mu);
            Cmd stop;
            stop.kind = Cmd::STOP;
            s->queue.push_back(std::move(stop));
        }
        s->cv.notify_all();
        s->worker.join();
    }
    if (s->gather_stream) (void)hipStreamSynchronize(s->gather_stream);
    if (s->reduce_stream) (void)hipStreamSynchronize(s->reduce_stream);
    for (Alloc &a : s->live)
        if (a.ready) (void)hipEventDestroy(a.ready);
    for (FreedRegion &f : s->freed) (void)hipEventDestroy(f.ev);
    for (hipEvent_t ev : s->spare_events) (void)hipEventDestroy(ev);
    if (s->fence_gather) (void)hipEventDestroy(s->fence_gather);
    if (s->fence_reduce) (void)hipEventDestroy(s->fence_reduce);
    if (s->gather_stream) (void)hipStreamDestroy(s->gather_stream);
    if (s->reduce_stream) (void)hipStreamDestroy(s->reduce_stream);
    if (s->pool) (void)hipFree(s->pool);
    delete s;
}

extern "C" hzp_status_t hzp_sched_prefetch(hzp_sched_t *s, uint32_t layer, const void *const *shard_ptrs,
                                           uint32_t n_shards, hipStream_t producer)
{
    if (!s || !shard_ptrs) return fail(HZP_ERR_INVALID_ARG, "hzp_sched_prefetch: NULL argument");
    const BucketRec *b = find_bucket(s->plan, layer, s->cls);
    if (!b) return fail(HZP_ERR_RANGE, "hzp_sched_prefetch: no bucket (layer %u, class %u)", layer, s->cls);
    if (n_shards != s->plan->z3)
        return fail(HZP_ERR_INVALID_ARG, "hzp_sched_prefetch: takes %u shards, got %u", s->plan->z3, n_shards);
    if (n_shards > HZP_MAX_GROUP)
        return fail(HZP_ERR_UNSUPPORTED, "hzp_sched_prefetch: %u shards exceed %u", n_shards, HZP_MAX_GROUP);
    for (uint32_t i = 0; i < n_shards; ++i) {
        if (!shard_ptrs[i]) return fail(HZP_ERR_INVALID_ARG, "hzp_sched_prefetch: shard %u is NULL", i);
        if (reinterpret_cast<uintptr_t>(shard_ptrs[i]) & 15u)
            return fail(HZP_ERR_ALIGN, "hzp_sched_prefetch: shard %u is not 16-byte aligned", i);
    }
    std::unique_lock<std::mutex> lock(s->mu);
    return prefetch_region(s, lock, "hzp_sched_prefetch: layer", layer, false, layer,
                           b->P * (s->cls == HZP_CLASS_F32 ? 4 : 2), shard_ptrs, n_shards, producer, true);
}

extern "C" hzp_status_t hzp_sched_prefetch_ahead(hzp_sched_t *s, uint32_t first_layer, uint32_t n_layers,
                                                 const void *const *shard_ptrs, uint32_t n_shards,
                                                 hipStream_t producer, uint32_t *issued)
{
    if (!s || !shard_ptrs || !issued) return fail(HZP_ERR_INVALID_ARG, "hzp_sched_prefetch_ahead: NULL argument");
    *issued = 0;
    if ((uint64_t)first_layer + n_layers > s->plan->n_layers)
        return fail(HZP_ERR_RANGE, "hzp_sched_prefetch_ahead: layers [%u, %u + %u) of %u", first_layer, first_layer,
                    n_layers, s->plan->n_layers);
    for (uint32_t l = 0; l < n_layers; ++l) {
        if (!find_bucket(s->plan, first_layer + l, s->cls)) {      // no bucket of the class: nothing to gather
            ++*issued;
            continue;
        }
        hzp_status_t st = hzp_sched_prefetch(s, first_layer + l, shard_ptrs + (size_t)l * n_shards, n_shards, producer);
        if (st == HZP_ERR_NOMEM) return HZP_OK;     // the pool is full: as far ahead as the memory allows
        if (st != HZP_OK) return st;
        ++*issued;
    }
    return HZP_OK;
}

extern "C" hzp_status_t hzp_sched_prefetch_tensor(hzp_sched_t *s, uint32_t tensor_id, const void *const *shard_ptrs,
                                                  uint32_t n_shards, hipStream_t producer)
{
    if (!s || !shard_ptrs) return fail(HZP_ERR_INVALID_ARG, "hzp_sched_prefetch_tensor: NULL argument");
    if (tensor_id >= s->plan->tensors.size())
        return fail(HZP_ERR_RANGE, "hzp_sched_prefetch_tensor: tensor %u of %zu", tensor_id, s->plan->tensors.size());
    const TensorRec &t = s->plan->tensors[tensor_id];
    if (t.cls != s->cls)
        return fail(HZP_ERR_RANGE, "hzp_sched_prefetch_tensor: tensor %u is of class %u, the scheduler of class %u",
                    tensor_id, t.cls, s->cls);
    const BucketRec &b = s->plan->buckets[t.bucket];
    if (n_shards != s->plan->z3)
        return fail(HZP_ERR_INVALID_ARG, "hzp_sched_prefetch_tensor: takes %u shards, got %u", s->plan->z3, n_shards);
    if (n_shards > HZP_MAX_GROUP)
        return fail(HZP_ERR_UNSUPPORTED, "hzp_sched_prefetch_tensor: %u shards exceed %u", n_shards, HZP_MAX_GROUP);
    for (uint64_t j = t.offset / b.S3; j <= (t.offset + t.numel - 1) / b.S3; ++j) {      // the shards it lies in
        if (!shard_ptrs[j])
            return fail(HZP_ERR_INVALID_ARG, "hzp_sched_prefetch_tensor: shard %llu is NULL", (unsigned long long)j);
        if (reinterpret_cast<uintptr_t>(shard_ptrs[j]) & 15u)
            return fail(HZP_ERR_ALIGN, "hzp_sched_prefetch_tensor: shard %llu is not 16-byte aligned",
                        (unsigned long long)j);
    }
    std::unique_lock<std::mutex> lock(s->mu);
    return prefetch_region(s, lock, "hzp_sched_prefetch_tensor: tensor", kTensorKey | tensor_id, true, tensor_id,
                           t.numel * (s->cls == HZP_CLASS_F32 ? 4 : 2), shard_ptrs, n_shards, producer, true);
}

// The parameters of one layer at the granularity Section 4.2 prefers -- one gather and one region of
// the pool per parameter -- submitted, acquired and released with one call each, so that the host
// calls and the stream operations on the consumer's stream do not grow with the number of parameters.
extern "C" hzp_status_t hzp_sched_prefetch_params(hzp_sched_t *s, uint32_t layer, const void *const *shard_ptrs,
                                                  uint32_t n_shards, hipStream_t producer)
{
    if (!s || !shard_ptrs) return fail(HZP_ERR_INVALID_ARG, "hzp_sched_prefetch_params: NULL argument");
    const BucketRec *b = find_bucket(s->plan, layer, s->cls);
    if (!b) return fail(HZP_ERR_RANGE, "hzp_sched_prefetch_params: no bucket (layer %u, class %u)", layer, s->cls);
    if (n_shards != s->plan->z3)
        return fail(HZP_ERR_INVALID_ARG, "hzp_sched_prefetch_params: takes %u shards, got %u", s->plan->z3, n_shards);
    if (n_shards > HZP_MAX_GROUP)
        return fail(HZP_ERR_UNSUPPORTED, "hzp_sched_prefetch_params: %u shards exceed %u", n_shards, HZP_MAX_GROUP);
    for (uint32_t i = 0; i < n_shards; ++i) {
        if (!shard_ptrs[i]) return fail(HZP_ERR_INVALID_ARG, "hzp_sched_prefetch_params: shard %u is NULL", i);
        if (reinterpret_cast<uintptr_t>(shard_ptrs[i]) & 15u)
            return fail(HZP_ERR_ALIGN, "hzp_sched_prefetch_params: shard %u is not 16-byte aligned", i);
    }
    const uint64_t es = s->cls == HZP_CLASS_F32 ? 4 : 2;
    std::unique_lock<std::mutex> lock(s->mu);
    if (s->failed != HZP_OK) return fail(s->failed, "scheduler failed earlier: %s", s->fail_text);
    for (uint32_t tid : b->tensor_ids)
        if (s->find(kTensorKey | tid))
            return fail(HZP_ERR_INVALID_ARG, "hzp_sched_prefetch_params: tensor %u is already in the pool", tid);
    // All or nothing: walk the ring for every parameter first.
    if (s->live.size() + b->tensor_ids.size() > s->max_live)
        return fail(HZP_ERR_NOMEM, "hzp_sched_prefetch_params: layer %u: %zu more regions do not fit beside the %zu "
                                   "between prefetch and release (at most %u)", layer, b->tensor_ids.size(), s->live.size(),
                    s->max_live);
    RingSpan span = ring_span(s);
    for (uint32_t tid : b->tensor_ids) {
        const uint64_t payload = s->plan->tensors[tid].numel * es;
        const uint64_t bytes = s->uniform_bytes ? s->uniform_bytes : (payload + 255) / 256 * 256;
        uint64_t off = 0, skipped = 0;
        if (!ring_take(s->pool_bytes, span, bytes, &off, &skipped))
            return fail(HZP_ERR_NOMEM, "hzp_sched_prefetch_params: layer %u: the pool has no room for all of its "
                                       "parameters until older regions are released", layer);
        if (span.empty) span = RingSpan{false, off, off + bytes};
        else span.head = off + bytes;
    }
    bool first = true;
    for (uint32_t tid : b->tensor_ids) {
        const hzp_status_t st = prefetch_region(s, lock, "hzp_sched_prefetch_params: tensor", kTensorKey | tid, true, tid,
                                                s->plan->tensors[tid].numel * es, shard_ptrs, n_shards, producer, first);
        if (st != HZP_OK) return st;        // the queue stayed full or a HIP call failed: the scheduler is failed
        first = false;
    }
    return HZP_OK;
}

extern "C" hzp_status_t hzp_sched_acquire_params(hzp_sched_t *s, uint32_t layer, hipStream_t consumer, void **tensors)
{
    if (!s || !tensors) return fail(HZP_ERR_INVALID_ARG, "hzp_sched_acquire_params: NULL argument");
    const BucketRec *b = find_bucket(s->plan, layer, s->cls);
    if (!b) return fail(HZP_ERR_RANGE, "hzp_sched_acquire_params: no bucket (layer %u, class %u)", layer, s->cls);
    std::unique_lock<std::mutex> lock(s->mu);
    for (uint32_t tid : b->tensor_ids) {
        const Alloc *a = s->find(kTensorKey | tid);
        if (!a) return fail(HZP_ERR_INVALID_ARG, "hzp_sched_acquire_params: tensor %u was not prefetched", tid);
        if (a->state == A_ACQUIRED)
            return fail(HZP_ERR_INVALID_ARG, "hzp_sched_acquire_params: tensor %u is already acquired", tid);
    }
    // Host-side wait until the background thread has launched every gather of the layer (not until
    // they have run): an event that has not been recorded yet cannot be waited for.
    const auto t0 = std::chrono::steady_clock::now();
    const bool ok = s->cv.wait_for(lock, kHostWaitLimit, [&] {
        if (s->failed != HZP_OK) return true;
        for (uint32_t tid : b->tensor_ids) {
            const Alloc *x = s->find(kTensorKey | tid);
            if (!x || x->state != A_READY) return false;
        }
        return true;
    });
    s->stats.acquire_host_wait_us += (uint64_t)std::chrono::duration_cast<std::chrono::microseconds>(
                                         std::chrono::steady_clock::now() - t0).count();
    if (s->failed != HZP_OK) return fail(s->failed, "scheduler failed earlier: %s", s->fail_text);
    if (!ok) {
        s->set_failed(HZP_ERR_HIP, "scheduler: a prefetch was not issued within the time limit");
        return fail(HZP_ERR_HIP, "%s", s->fail_text);
    }
    // One wait on the consumer's stream: the gathers run in order on the one gather stream, so the
    // last one's event covers them all -- unless some were prefetched one by one in another order,
    // in which case every event is waited for.
    bool in_order = true;
    {
        size_t next = 0;                        // entries of the deque lie in prefetch order
        for (const Alloc &x : s->live) {
            if (x.state == A_RELEASED || !(x.key & kTensorKey)) continue;
            const uint32_t tid = (uint32_t)(x.key & 0xFFFFFFFFull);
            if (next < b->tensor_ids.size() && tid == b->tensor_ids[next]) {
                ++next;
            } else if (s->plan->tensors[tid].bucket == (uint32_t)(b - s->plan->buckets.data()) && next < b->tensor_ids.size()) {
                in_order = false;               // one of this layer's, but not the next one
            }
        }
        if (next != b->tensor_ids.size()) in_order = false;
    }
    for (size_t i = 0; i < b->tensor_ids.size(); ++i) {
        Alloc *a = s->find(kTensorKey | b->tensor_ids[i]);
        if (!in_order || i + 1 == b->tensor_ids.size()) {
            const hipError_t e = hipStreamWaitEvent(consumer, a->ready, 0);
            if (e != hipSuccess) return hip_fail(s, "hzp_sched_acquire_params", e);
        }
    }
    for (size_t i = 0; i < b->tensor_ids.size(); ++i) {
        Alloc *a = s->find(kTensorKey | b->tensor_ids[i]);
        a->state = A_ACQUIRED;
        tensors[i] = s->pool + a->off;
    }
    return HZP_OK;
}

extern "C" hzp_status_t hzp_sched_release_params(hzp_sched_t *s, uint32_t layer, hipStream_t consumer)
{
    if (!s) return fail(HZP_ERR_INVALID_ARG, "hzp_sched_release_params: NULL scheduler");
    const BucketRec *b = find_bucket(s->plan, layer, s->cls);
    if (!b) return fail(HZP_ERR_RANGE, "hzp_sched_release_params: no bucket (layer %u, class %u)", layer, s->cls);
    std::unique_lock<std::mutex> lock(s->mu);
    for (uint32_t tid : b->tensor_ids) {
        const Alloc *a = s->find(kTensorKey | tid);
        if (!a || a->state != A_ACQUIRED)
            return fail(HZP_ERR_INVALID_ARG, "hzp_sched_release_params: tensor %u is not acquired", tid);
    }
    // Regions that lie back to back in the pool are given back as one, behind one event on the
    // consumer's stream (a layer's parameters form one run, two where the ring wrapped).
    if (s->freed.size() >= kFreedSweep) sweep_freed(s);
    uint64_t run_off = 0, run_bytes = 0;
    auto give_back = [&]() -> hipError_t {
        if (run_bytes == 0) return hipSuccess;
        hipEvent_t ev = nullptr;
        hipError_t e = take_event(s, &ev);
        if (e == hipSuccess) {
            e = hipEventRecord(ev, consumer);
            if (e != hipSuccess) s->spare_events.push_back(ev);
        }
        if (e == hipSuccess) s->freed.push_back(FreedRegion{run_off, run_bytes, ev});
        run_bytes = 0;
        return e;
    };
    for (uint32_t tid : b->tensor_ids) {
        Alloc *a = s->find(kTensorKey | tid);
        if (run_bytes != 0 && a->off != run_off + run_bytes) {
            const hipError_t e = give_back();
            if (e != hipSuccess) return hip_fail(s, "hzp_sched_release_params", e);
        }
        if (run_bytes == 0) run_off = a->off;
        run_bytes += a->bytes;
        s->spare_events.push_back(a->ready);    // the consumer's wait on it (or on a later one) was enqueued at acquire
        a->ready = nullptr;
        a->state = A_RELEASED;
    }
    const hipError_t e = give_back();
    if (e != hipSuccess) return hip_fail(s, "hzp_sched_release_params", e);
    while (!s->live.empty() && s->live.front().state == A_RELEASED) s->live.pop_front();
    s->cv.notify_all();
    return HZP_OK;
}

extern "C" hzp_status_t hzp_sched_acquire(hzp_sched_t *s, uint32_t layer, hipStream_t consumer, void **bucket)
{
    if (!s || !bucket) return fail(HZP_ERR_INVALID_ARG, "hzp_sched_acquire: NULL argument");
    return acquire_region(s, "hzp_sched_acquire: layer", layer, layer, consumer, bucket);
}

extern "C" hzp_status_t hzp_sched_acquire_tensor(hzp_sched_t *s, uint32_t tensor_id, hipStream_t consumer,
                                                 void **tensor)
{
    if (!s || !tensor) return fail(HZP_ERR_INVALID_ARG, "hzp_sched_acquire_tensor: NULL argument");
    return acquire_region(s, "hzp_sched_acquire_tensor: tensor", kTensorKey | tensor_id, tensor_id, consumer, tensor);
}

extern "C" hzp_status_t hzp_sched_release(hzp_sched_t *s, uint32_t layer, hipStream_t consumer)
{
    if (!s) return fail(HZP_ERR_INVALID_ARG, "hzp_sched_release: NULL scheduler");
    return release_region(s, "hzp_sched_release: layer", layer, layer, consumer);
}

extern "C" hzp_status_t hzp_sched_release_tensor(hzp_sched_t *s, uint32_t tensor_id, hipStream_t consumer)
{
    if (!s) return fail(HZP_ERR_INVALID_ARG, "hzp_sched_release_tensor: NULL scheduler");
    return release_region(s, "hzp_sched_release_tensor: tensor", kTensorKey | tensor_id, tensor_id, consumer);
}

extern "C" hzp_status_t hzp_sched_reduce(hzp_sched_t *s, uint32_t layer, int level, uint32_t rank,
                                         const void *const *grad_slices, uint32_t R, uint32_t grad_dtype, float scale,
                                         int accumulate, float *out_f32, hipStream_t producer)
{
    if (!s || !grad_slices || !out_f32) return fail(HZP_ERR_INVALID_ARG, "hzp_sched_reduce: NULL argument");
    if (R == 0 || R > HZP_MAX_REPLICAS) return fail(HZP_ERR_UNSUPPORTED, "hzp_sched_reduce: R=%u", R);
    const BucketRec *b = find_bucket(s->plan, layer, s->cls);
    if (!b) return fail(HZP_ERR_RANGE, "hzp_sched_reduce: no bucket (layer %u, class %u)", layer, s->cls);
    // Everything hzp_reduce_shard would refuse is refused here, at submission: an error found
    // later, on the background thread, could only be reported by failing the whole scheduler.
    if (level < 1 || level > 3) return fail(HZP_ERR_RANGE, "hzp_sched_reduce: level %d is not 1, 2 or 3", level);
    if (rank >= s->plan->world)
        return fail(HZP_ERR_RANGE, "hzp_sched_reduce: rank %u of %u", rank, s->plan->world);
    if (grad_dtype > HZP_GRAD_F32)
        return fail(HZP_ERR_INVALID_ARG, "hzp_sched_reduce: unknown gradient type %u", grad_dtype);
    if ((level == 1 ? b->S1 : level == 2 ? b->S2 : b->S3) >= (1ull << 30))
        return fail(HZP_ERR_UNSUPPORTED, "hzp_sched_reduce: shard of 2^30 elements or more");
    for (uint32_t r = 0; r < R; ++r) {
        if (!grad_slices[r]) return fail(HZP_ERR_INVALID_ARG, "hzp_sched_reduce: slice %u is NULL", r);
        if (reinterpret_cast<uintptr_t>(grad_slices[r]) & 15u)
            return fail(HZP_ERR_ALIGN, "hzp_sched_reduce: slice %u is not 16-byte aligned", r);
    }
    if (reinterpret_cast<uintptr_t>(out_f32) & 15u)
        return fail(HZP_ERR_ALIGN, "hzp_sched_reduce: output is not 16-byte aligned");
    std::unique_lock<std::mutex> lock(s->mu);
    if (s->failed != HZP_OK) return fail(s->failed, "scheduler failed earlier: %s", s->fail_text);
    Cmd cmd;
    cmd.kind = Cmd::REDUCE;
    cmd.id = layer;
    cmd.level = level;
    cmd.rank = rank;
    cmd.R = R;
    cmd.grad_dtype = grad_dtype;
    cmd.scale = scale;
    cmd.accumulate = accumulate;
    cmd.out = out_f32;
    cmd.ptrs.assign(grad_slices, grad_slices + R);
    hipError_t e = take_event(s, &cmd.after);
    if (e != hipSuccess) return hip_fail(s, "hzp_sched_reduce", e);
    // The gradients exist once the producer's work enqueued so far has run.
    e = hipEventRecord(cmd.after, producer);
    if (e != hipSuccess) {
        s->spare_events.push_back(cmd.after);
        return hip_fail(s, "hzp_sched_reduce", e);
    }
    hipEvent_t ev = cmd.after;
    hzp_status_t st = submit(s, lock, cmd, nullptr);
    if (st != HZP_OK) s->spare_events.push_back(ev);
    return st;
}

// Wait (host) until every command submitted so far has been launched by the background thread.
static hzp_status_t wait_processed(hzp_sched *s, std::unique_lock<std::mutex> &lock, uint64_t seq)
{
    bool ok = s->cv.wait_for(lock, kHostWaitLimit, [&] { return s->failed != HZP_OK || s->processed >= seq; });
    if (s->failed != HZP_OK) return fail(s->failed, "scheduler failed earlier: %s", s->fail_text);
    if (!ok) {
        s->set_failed(HZP_ERR_HIP, "scheduler: commands were not issued within the time limit");
        return fail(HZP_ERR_HIP, "%s", s->fail_text);
    }
    return HZP_OK;
}

extern "C" hzp_status_t hzp_sched_join(hzp_sched_t *s, hipStream_t consumer)
{
    if (!s) return fail(HZP_ERR_INVALID_ARG, "hzp_sched_join: NULL scheduler");
    std::unique_lock<std::mutex> lock(s->mu);
    if (s->failed != HZP_OK) return fail(s->failed, "scheduler failed earlier: %s", s->fail_text);
    Cmd cmd;
    cmd.kind = Cmd::FENCE;
    uint64_t seq = 0;
    hzp_status_t st = submit(s, lock, cmd, &seq);
    if (st == HZP_OK) st = wait_processed(s, lock, seq);
    if (st != HZP_OK) return st;
    hipError_t e = hipStreamWaitEvent(consumer, s->fence_gather, 0);
    if (e == hipSuccess) e = hipStreamWaitEvent(consumer, s->fence_reduce, 0);
    if (e != hipSuccess) return hip_fail(s, "hzp_sched_join", e);
    return HZP_OK;
}

extern "C" hzp_status_t hzp_sched_drain(hzp_sched_t *s)
{
    if (!s) return fail(HZP_ERR_INVALID_ARG, "hzp_sched_drain: NULL scheduler");
    {
        std::unique_lock<std::mutex> lock(s->mu);
        hzp_status_t st = wait_processed(s, lock, s->submitted);
        if (st != HZP_OK) return st;
    }
    hipError_t e = hipStreamSynchronize(s->gather_stream);
    if (e == hipSuccess) e = hipStreamSynchronize(s->reduce_stream);
    if (e != hipSuccess) return hip_fail(s, "hzp_sched_drain", e);
    return HZP_OK;
}

extern "C" hzp_status_t hzp_sched_stats(hzp_sched_t *s, hzp_sched_stats_t *out)
{
    if (!s || !out) return fail(HZP_ERR_INVALID_ARG, "hzp_sched_stats: NULL argument");
    std::lock_guard<std::mutex> lock(s->mu);
    *out = s->stats;
    return HZP_OK;
}
