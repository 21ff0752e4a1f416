// Asynchronous scheduler of libhzp: the multi-stream dispatch of Section 4.2 for the local halves
// of the collectives.
//
// What the paper describes and what is kept here:
//   - parameter all-gathers and gradient reduce-scatters are issued from an extra host thread on
//     dedicated streams, so that issuing them never blocks the thread that drives the compute
//     stream and puts nothing on that stream at issue time;
//   - all-gather results live in a pre-allocated, fixed-capacity, persistent pool whose
//     contiguous buffers are reused cyclically by this one kind of operation, which keeps
//     fragmentation negligible; a layer's buffer is given back right after its use;
//   - parameters are pre-launched ahead of their use (prefetch) and gradients are consumed as
//     soon as they exist ("hungrily").
// Ordering between the side streams and the consumer's stream is carried by events: the consumer
// waits for a layer's `ready` event when it acquires the layer, and the gather stream waits for the
// slot's `freed` event before it overwrites the slot.  Host-side waits carry a time limit and turn
// into an error status instead of hanging.
#include <hip/hip_runtime_api.h>

#include <chrono>
#include <cstdio>
#include <condition_variable>
#include <deque>
#include <map>
#include <new>
#include <thread>

#include "hzp_internal.hpp"

using namespace hzp;

namespace {

constexpr auto kHostWaitLimit = std::chrono::seconds(30);

enum SlotState { SLOT_FREE, SLOT_ASSIGNED, SLOT_READY, SLOT_ACQUIRED, SLOT_RELEASED };

struct Slot {
    SlotState state = SLOT_FREE;
    uint64_t ticket = 0;            // prefetch that owns (or is about to own) the slot
    uint64_t issued = 0;            // ticket whose gather has been launched into the slot
    uint32_t layer = 0;
    uint64_t bytes = 0;             // bytes of the bucket held
    bool freed_recorded = false;
    hipEvent_t ready = nullptr, freed = nullptr;
};

struct Cmd {
    enum Kind { PREFETCH, REDUCE, FENCE, STOP } kind = STOP;
    uint32_t layer = 0, R = 0, grad_dtype = 0, rank = 0;
    int level = 0, accumulate = 0, slot = -1;
    float scale = 1.0f;
    float *out = nullptr;
    uint64_t ticket = 0;
    hipEvent_t after = nullptr;     // REDUCE: recorded on the producer's stream at submission
    std::vector<const void *> ptrs;
};

}  // namespace

struct hzp_sched {
    const hzp_plan_t *plan = nullptr;
    uint32_t cls = 0, n_slots = 0, queue_capacity = 0;
    int device = 0;
    uint64_t slot_bytes = 0;
    char *pool = nullptr;
    hipStream_t gather_stream = nullptr, reduce_stream = nullptr;
    std::vector<Slot> slots;
    std::map<uint32_t, int> slot_of_layer;      // layers prefetched and not yet released
    std::deque<Cmd> queue;
    std::vector<hipEvent_t> spare_events;
    hipEvent_t fence_gather = nullptr, fence_reduce = nullptr;
    uint64_t next_ticket = 1, submitted = 0, processed = 0;
    uint32_t next_slot = 0;
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
};

namespace {

hzp_status_t hip_fail(hzp_sched *s, const char *what, hipError_t e)
{
    char text[256];
    snprintf(text, sizeof text, "%s: %s", what, hipGetErrorString(e));
    s->set_failed(HZP_ERR_HIP, text);
    return fail(HZP_ERR_HIP, "%s", text);
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
        bool ok = true;
        if (cmd.kind == Cmd::PREFETCH) {
            Slot &slot = s->slots[cmd.slot];
            bool wait_freed = false;
            {
                // The slot is reused cyclically: wait until the layer that held it has been released.
                std::unique_lock<std::mutex> lock(s->mu);
                ok = s->cv.wait_for(lock, kHostWaitLimit, [&] {
                    return s->failed != HZP_OK || (slot.ticket == cmd.ticket && slot.state == SLOT_ASSIGNED);
                });
                if (!ok) s->set_failed(HZP_ERR_HIP, "scheduler: a pool slot was not released within the time limit");
                ok = ok && s->failed == HZP_OK;
                wait_freed = slot.freed_recorded;
            }
            if (ok) {
                hipError_t e = wait_freed ? hipStreamWaitEvent(s->gather_stream, slot.freed, 0) : hipSuccess;
                hzp_status_t st = HZP_OK;
                if (e == hipSuccess)
                    st = hzp_gather_layer(s->plan, cmd.layer, s->cls, 3, cmd.ptrs.data(), (uint32_t)cmd.ptrs.size(),
                                          s->pool + (size_t)cmd.slot * s->slot_bytes, nullptr, s->gather_stream);
                if (e == hipSuccess && st == HZP_OK) e = hipEventRecord(slot.ready, s->gather_stream);
                std::lock_guard<std::mutex> lock(s->mu);
                if (e != hipSuccess || st != HZP_OK) {
                    s->set_failed(st != HZP_OK ? st : HZP_ERR_HIP, st != HZP_OK ? hzp_last_error() : hipGetErrorString(e));
                } else {
                    slot.issued = cmd.ticket;
                    slot.state = SLOT_READY;
                    s->stats.gathers_issued++;
                }
            }
        } else if (cmd.kind == Cmd::REDUCE) {
            hipError_t e = hipStreamWaitEvent(s->reduce_stream, cmd.after, 0);
            hzp_status_t st = HZP_OK;
            if (e == hipSuccess)
                st = hzp_reduce_shard(s->plan, cmd.layer, s->cls, cmd.level, cmd.rank, cmd.ptrs.data(), cmd.R,
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

// Queue a command; blocks (with the time limit) while the queue is full.
hzp_status_t submit(hzp_sched *s, std::unique_lock<std::mutex> &lock, Cmd &&cmd, uint64_t *seq)
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

}  // namespace

extern "C" hzp_status_t hzp_sched_create(const hzp_plan_t *plan, const hzp_sched_desc_t *d, hzp_sched_t **out)
{
    if (!plan || !d || !out) return fail(HZP_ERR_INVALID_ARG, "hzp_sched_create: NULL argument");
    *out = nullptr;
    if (d->cls > 1) return fail(HZP_ERR_RANGE, "hzp_sched_create: class %u", d->cls);
    if (d->gather_slots == 0 || d->queue_capacity == 0)
        return fail(HZP_ERR_INVALID_ARG, "hzp_sched_create: needs at least one pool slot and one queue entry");
    uint64_t max_p = 0;
    for (const BucketRec &b : plan->buckets)
        if (b.cls == d->cls) max_p = std::max(max_p, b.P);
    if (max_p == 0) return fail(HZP_ERR_RANGE, "hzp_sched_create: the plan has no bucket of class %u", d->cls);
    hzp_sched *s = new (std::nothrow) hzp_sched;
    if (!s) return fail(HZP_ERR_NOMEM, "hzp_sched_create: out of host memory");
    s->plan = plan;
    s->cls = d->cls;
    s->n_slots = d->gather_slots;
    s->queue_capacity = d->queue_capacity;
    s->slot_bytes = (max_p * (d->cls == HZP_CLASS_F32 ? 4 : 2) + 255) / 256 * 256;
    hipError_t e = hipGetDevice(&s->device);
    // One allocation for the whole pool: contiguous slots, never freed or grown until destroy.
    if (e == hipSuccess) e = hipMalloc((void **)&s->pool, s->slot_bytes * s->n_slots);
    if (e == hipSuccess) e = hipStreamCreateWithFlags(&s->gather_stream, hipStreamNonBlocking);
    if (e == hipSuccess) e = hipStreamCreateWithFlags(&s->reduce_stream, hipStreamNonBlocking);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&s->fence_gather, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&s->fence_reduce, hipEventDisableTiming);
    s->slots.resize(s->n_slots);
    for (Slot &slot : s->slots) {
        if (e == hipSuccess) e = hipEventCreateWithFlags(&slot.ready, hipEventDisableTiming);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&slot.freed, hipEventDisableTiming);
    }
    if (e != hipSuccess) {
        const hzp_status_t st = fail(e == hipErrorOutOfMemory ? HZP_ERR_NOMEM : HZP_ERR_HIP, "hzp_sched_create: %s",
                                     hipGetErrorString(e));
        hzp_sched_destroy(s);
        return st;
    }
    s->stats.pool_bytes = s->slot_bytes * s->n_slots;
    s->stats.slot_bytes = s->slot_bytes;
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
    for (Slot &slot : s->slots) {
        if (slot.ready) (void)hipEventDestroy(slot.ready);
        if (slot.freed) (void)hipEventDestroy(slot.freed);
    }
    for (hipEvent_t ev : s->spare_events) (void)hipEventDestroy(ev);
    for (Cmd &c : s->queue)
        if (c.after) (void)hipEventDestroy(c.after);
    if (s->fence_gather) (void)hipEventDestroy(s->fence_gather);
    if (s->fence_reduce) (void)hipEventDestroy(s->fence_reduce);
    if (s->gather_stream) (void)hipStreamDestroy(s->gather_stream);
    if (s->reduce_stream) (void)hipStreamDestroy(s->reduce_stream);
    if (s->pool) (void)hipFree(s->pool);
    delete s;
}

extern "C" hzp_status_t hzp_sched_prefetch(hzp_sched_t *s, uint32_t layer, const void *const *shard_ptrs,
                                           uint32_t n_shards)
{
    if (!s || !shard_ptrs) return fail(HZP_ERR_INVALID_ARG, "hzp_sched_prefetch: NULL argument");
    const BucketRec *b = find_bucket(s->plan, layer, s->cls);
    if (!b) return fail(HZP_ERR_RANGE, "hzp_sched_prefetch: no bucket (layer %u, class %u)", layer, s->cls);
    if (n_shards != s->plan->z3)
        return fail(HZP_ERR_INVALID_ARG, "hzp_sched_prefetch: takes %u shards, got %u", s->plan->z3, n_shards);
    for (uint32_t i = 0; i < n_shards; ++i) {
        if (!shard_ptrs[i]) return fail(HZP_ERR_INVALID_ARG, "hzp_sched_prefetch: shard %u is NULL", i);
        if (reinterpret_cast<uintptr_t>(shard_ptrs[i]) & 15u)
            return fail(HZP_ERR_ALIGN, "hzp_sched_prefetch: shard %u is not 16-byte aligned", i);
    }
    std::unique_lock<std::mutex> lock(s->mu);
    if (s->failed != HZP_OK) return fail(s->failed, "scheduler failed earlier: %s", s->fail_text);
    if (s->slot_of_layer.count(layer))
        return fail(HZP_ERR_INVALID_ARG, "hzp_sched_prefetch: layer %u is already in the pool", layer);
    if (s->slot_of_layer.size() >= s->n_slots)
        return fail(HZP_ERR_NOMEM, "hzp_sched_prefetch: all %u pool slots hold unreleased layers", s->n_slots);
    // Cyclic reuse: the next slot in order; it is free or will be once its layer is released.
    const int idx = (int)(s->next_slot % s->n_slots);
    Slot &slot = s->slots[idx];
    if (slot.state != SLOT_FREE && slot.state != SLOT_RELEASED)
        return fail(HZP_ERR_NOMEM, "hzp_sched_prefetch: the next slot in the cycle still holds layer %u; release "
                                   "layers in the order they were prefetched", slot.layer);
    Cmd cmd;
    cmd.kind = Cmd::PREFETCH;
    cmd.layer = layer;
    cmd.slot = idx;
    cmd.ticket = s->next_ticket;
    cmd.ptrs.assign(shard_ptrs, shard_ptrs + n_shards);
    hzp_status_t st = submit(s, lock, std::move(cmd), nullptr);
    if (st != HZP_OK) return st;
    s->next_slot++;
    slot.ticket = s->next_ticket++;
    slot.state = SLOT_ASSIGNED;
    slot.layer = layer;
    slot.bytes = b->P * (s->cls == HZP_CLASS_F32 ? 4 : 2);
    s->slot_of_layer[layer] = idx;
    uint64_t live = 0;
    for (const Slot &x : s->slots)
        if (x.state != SLOT_FREE && x.state != SLOT_RELEASED) live += x.bytes;
    s->stats.peak_live_bytes = std::max(s->stats.peak_live_bytes, live);
    s->stats.peak_live_slots = std::max<uint32_t>(s->stats.peak_live_slots, (uint32_t)s->slot_of_layer.size());
    s->cv.notify_all();
    return HZP_OK;
}

extern "C" hzp_status_t hzp_sched_acquire(hzp_sched_t *s, uint32_t layer, hipStream_t consumer, void **bucket)
{
    if (!s || !bucket) return fail(HZP_ERR_INVALID_ARG, "hzp_sched_acquire: NULL argument");
    std::unique_lock<std::mutex> lock(s->mu);
    auto it = s->slot_of_layer.find(layer);
    if (it == s->slot_of_layer.end())
        return fail(HZP_ERR_INVALID_ARG, "hzp_sched_acquire: layer %u was not prefetched", layer);
    Slot &slot = s->slots[it->second];
    if (slot.state == SLOT_ACQUIRED) return fail(HZP_ERR_INVALID_ARG, "hzp_sched_acquire: layer %u is already acquired", layer);
    // Host-side wait until the background thread has launched the gather (not until it has run).
    const auto t0 = std::chrono::steady_clock::now();
    bool ok = s->cv.wait_for(lock, kHostWaitLimit, [&] { return s->failed != HZP_OK || slot.state == SLOT_READY; });
    s->stats.acquire_host_wait_us += (uint64_t)std::chrono::duration_cast<std::chrono::microseconds>(
                                         std::chrono::steady_clock::now() - t0).count();
    if (s->failed != HZP_OK) return fail(s->failed, "scheduler failed earlier: %s", s->fail_text);
    if (!ok) {
        s->set_failed(HZP_ERR_HIP, "scheduler: a prefetch was not issued within the time limit");
        return fail(HZP_ERR_HIP, "%s", s->fail_text);
    }
    hipError_t e = hipStreamWaitEvent(consumer, slot.ready, 0);
    if (e != hipSuccess) return hip_fail(s, "hzp_sched_acquire", e);
    slot.state = SLOT_ACQUIRED;
    *bucket = s->pool + (size_t)it->second * s->slot_bytes;
    return HZP_OK;
}

extern "C" hzp_status_t hzp_sched_release(hzp_sched_t *s, uint32_t layer, hipStream_t consumer)
{
    if (!s) return fail(HZP_ERR_INVALID_ARG, "hzp_sched_release: NULL scheduler");
    std::unique_lock<std::mutex> lock(s->mu);
    auto it = s->slot_of_layer.find(layer);
    if (it == s->slot_of_layer.end() || s->slots[it->second].state != SLOT_ACQUIRED)
        return fail(HZP_ERR_INVALID_ARG, "hzp_sched_release: layer %u is not acquired", layer);
    Slot &slot = s->slots[it->second];
    hipError_t e = hipEventRecord(slot.freed, consumer);
    if (e != hipSuccess) return hip_fail(s, "hzp_sched_release", e);
    slot.freed_recorded = true;
    slot.state = SLOT_RELEASED;
    s->slot_of_layer.erase(it);
    s->cv.notify_all();
    return HZP_OK;
}

extern "C" hzp_status_t hzp_sched_reduce(hzp_sched_t *s, uint32_t layer, int level, uint32_t rank,
                                         const void *const *grad_slices, uint32_t R, uint32_t grad_dtype, float scale,
                                         int accumulate, float *out_f32, hipStream_t producer)
{
    if (!s || !grad_slices || !out_f32) return fail(HZP_ERR_INVALID_ARG, "hzp_sched_reduce: NULL argument");
    if (R == 0 || R > HZP_MAX_REPLICAS) return fail(HZP_ERR_UNSUPPORTED, "hzp_sched_reduce: R=%u", R);
    if (!find_bucket(s->plan, layer, s->cls))
        return fail(HZP_ERR_RANGE, "hzp_sched_reduce: no bucket (layer %u, class %u)", layer, s->cls);
    // Everything hzp_reduce_shard would refuse is refused here, at submission: an error found
    // later, on the background thread, could only be reported by failing the whole scheduler.
    if (level < 1 || level > 3) return fail(HZP_ERR_RANGE, "hzp_sched_reduce: level %d is not 1, 2 or 3", level);
    if (rank >= s->plan->world)
        return fail(HZP_ERR_RANGE, "hzp_sched_reduce: rank %u of %u", rank, s->plan->world);
    if (grad_dtype > HZP_GRAD_F32)
        return fail(HZP_ERR_INVALID_ARG, "hzp_sched_reduce: unknown gradient type %u", grad_dtype);
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
    cmd.layer = layer;
    cmd.level = level;
    cmd.rank = rank;
    cmd.R = R;
    cmd.grad_dtype = grad_dtype;
    cmd.scale = scale;
    cmd.accumulate = accumulate;
    cmd.out = out_f32;
    cmd.ptrs.assign(grad_slices, grad_slices + R);
    if (!s->spare_events.empty()) {
        cmd.after = s->spare_events.back();
        s->spare_events.pop_back();
    } else {
        hipError_t e = hipEventCreateWithFlags(&cmd.after, hipEventDisableTiming);
        if (e != hipSuccess) return hip_fail(s, "hzp_sched_reduce", e);
    }
    // The gradients exist once the producer's work enqueued so far has run.
    hipError_t e = hipEventRecord(cmd.after, producer);
    if (e != hipSuccess) {
        s->spare_events.push_back(cmd.after);
        return hip_fail(s, "hzp_sched_reduce", e);
    }
    hipEvent_t ev = cmd.after;
    hzp_status_t st = submit(s, lock, std::move(cmd), nullptr);
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
    hzp_status_t st = submit(s, lock, std::move(cmd), &seq);
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
