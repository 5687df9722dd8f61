// The runtime around the three calls: the double-buffered cache (C_s / C_sec, swapped at the
// epoch boundary) and the rolling prefetch queue of depth Q (Sec. 3 "Rolling prefetch and
// execution"; Alg. 1: the secondary-cache build and the prefetch of the next Q batches that run
// beside an epoch's batch loop, and the swap at the epoch's end if the secondary cache is ready;
// Sec. 4 par. (4), (6), (7)).  Host-side orchestration of the library's own kernels: threads,
// streams and events, no new device code.
#include "rg_internal.h"

#include <atomic>
#include <string>
#include <thread>

// ---------------------------------------------------------------- double-buffered cache
struct rg_cache_pair {
    rg_cache *primary = nullptr;       // C_s, serves the running epoch
    rg_cache *secondary = nullptr;     // C_sec, being built or ready for the next epoch
    rg_features feat{};
    uint64_t K = 0;
    rg_allocator alloc{};
    bool has_alloc = false;
    int device = 0;
    hipStream_t build_stream = nullptr;
    std::thread worker;
    std::atomic<int> state{0};         // 0 idle, 1 building, 2 ready, 3 failed
    std::atomic<uint64_t> building_bytes{0};   // table bytes of the C_sec under construction, once its table exists
    rg_status worker_status = RG_OK;
    std::string worker_error;
};

namespace rg {

static void build_secondary(rg_cache_pair *p, const rg_schedule *next)
{
    (void)hipSetDevice(p->device);
    rg_cache *c = nullptr;
    const rg_schedule *eps[1] = {next};
    tls_table_bytes_sink = &p->building_bytes;
    rg_status rc = rg_build_cache(eps, 1, &p->feat, p->K, p->has_alloc ? &p->alloc : nullptr, p->build_stream, &c);
    tls_table_bytes_sink = nullptr;
    if (rc != RG_OK) p->building_bytes.store(0, std::memory_order_release);
    if (rc == RG_OK) {
        p->secondary = c;
        p->worker_status = RG_OK;
        p->state.store(2, std::memory_order_release);
    } else {
        p->worker_status = rc;
        p->worker_error = rg_last_error();
        p->state.store(3, std::memory_order_release);
    }
}

}  // namespace rg

using namespace rg;

extern "C" {

rg_status rg_cache_pair_create(const rg_schedule *first_epoch, const rg_features *f, uint64_t K, const rg_allocator *a, void *stream,
                               rg_cache_pair **out)
{
    if (!first_epoch || !f || !out) { set_error("rg_cache_pair_create: null argument"); return RG_EINVAL; }
    rg_cache_pair *p = new (std::nothrow) rg_cache_pair();
    if (!p) { set_error("rg_cache_pair_create: out of host memory"); return RG_ENOMEM; }
    p->feat = *f;
    p->K = K;
    if (a) { p->alloc = *a; p->has_alloc = true; }
    rg_status rc = RG_OK;
    if (hipGetDevice(&p->device) != hipSuccess || hipStreamCreateWithFlags(&p->build_stream, hipStreamNonBlocking) != hipSuccess) {
        set_error("rg_cache_pair_create: cannot create the build stream");
        rc = RG_EHIP;
    }
    if (rc == RG_OK) {
        const rg_schedule *eps[1] = {first_epoch};
        rc = rg_build_cache(eps, 1, f, K, a, stream, &p->primary);
    }
    if (rc != RG_OK) {
        if (p->build_stream) (void)hipStreamDestroy(p->build_stream);
        delete p;
        return rc;
    }
    *out = p;
    return RG_OK;
}

rg_status rg_cache_pair_begin_next(rg_cache_pair *p, const rg_schedule *next_epoch)
{
    if (!p || !next_epoch) { set_error("rg_cache_pair_begin_next: null argument"); return RG_EINVAL; }
    const int st = p->state.load(std::memory_order_acquire);
    if (st == 1) { set_error("rg_cache_pair_begin_next: a secondary build is already running"); return RG_EINVAL; }
    if (p->worker.joinable()) p->worker.join();
    if (p->secondary) { rg_cache_destroy(p->secondary); p->secondary = nullptr; }      // an unused C_sec is dropped
    p->building_bytes.store(0, std::memory_order_release);
    p->state.store(1, std::memory_order_release);
    try {
        p->worker = std::thread(build_secondary, p, next_epoch);
    } catch (...) {
        p->state.store(0, std::memory_order_release);
        set_error("rg_cache_pair_begin_next: cannot start the build thread");
        return RG_ENOMEM;
    }
    return RG_OK;
}

rg_status rg_cache_pair_swap(rg_cache_pair *p, int wait, int *swapped)
{
    if (!p) { set_error("rg_cache_pair_swap: null argument"); return RG_EINVAL; }
    if (swapped) *swapped = 0;
    int st = p->state.load(std::memory_order_acquire);
    if (st == 1 && !wait) return RG_OK;                       // not ready: the old cache keeps serving (Alg. 1, the swap is conditional)
    if (p->worker.joinable()) p->worker.join();
    st = p->state.load(std::memory_order_acquire);
    if (st == 3) {
        p->state.store(0, std::memory_order_release);
        set_error("secondary cache build failed: %s", p->worker_error.c_str());
        return p->worker_status;
    }
    if (st != 2) return RG_OK;                                // nothing was being built
    rg_cache *old = p->primary;
    p->primary = p->secondary;
    p->secondary = nullptr;
    p->state.store(0, std::memory_order_release);
    rg_cache_destroy(old);                                    // released once the gathers that still read the old table have finished; nothing waits here
    if (swapped) *swapped = 1;
    return RG_OK;
}

const rg_cache *rg_cache_pair_primary(const rg_cache_pair *p) { return p ? p->primary : nullptr; }

uint64_t rg_cache_pair_table_bytes(const rg_cache_pair *p)
{
    if (!p) return 0;
    uint64_t b = 0;
    if (p->primary) b += p->primary->K_eff * p->primary->stride;
    const int st = p->state.load(std::memory_order_acquire);
    if (st == 2 && p->secondary) b += p->secondary->K_eff * p->secondary->stride;
    else if (st == 1) b += p->building_bytes.load(std::memory_order_acquire);       // a C_sec whose table is already allocated
    return b;
}

void rg_cache_pair_destroy(rg_cache_pair *p)
{
    if (!p) return;
    if (p->worker.joinable()) p->worker.join();
    if (p->secondary) rg_cache_destroy(p->secondary);
    if (p->primary) rg_cache_destroy(p->primary);
    if (p->build_stream) (void)hipStreamDestroy(p->build_stream);
    delete p;
}

}  // extern "C"

// ---------------------------------------------------------------- rolling prefetch queue
struct rg_prefetcher {
    const rg_schedule *s = nullptr;
    const rg_cache *c = nullptr;
    rg_features feat{};
    uint32_t Q = 0;
    std::vector<void *> slot;              // Q output buffers (caller's)
    uint64_t out_stride = 0, capacity_rows = 0;
    hipStream_t stream = nullptr, side = nullptr;
    std::vector<hipEvent_t> ready, freed;  // per slot: data staged / consumer done
    std::vector<char> freed_valid;
    std::vector<rg_gather_stats> stats;    // per slot
    uint32_t staged = 0;                   // batches [acquired, staged) are in the queue
    uint32_t acquired = 0;                 // batches [released, acquired) are held by the consumer
    uint32_t released = 0;
};

extern "C" {

rg_status rg_prefetcher_create(const rg_schedule *s, const rg_cache *c, const rg_features *f, uint32_t Q, void *const *slot_buffers,
                               uint64_t out_stride, uint64_t slot_capacity_rows, rg_prefetcher **out)
{
    if (!s || !f || !slot_buffers || !out) { set_error("rg_prefetcher_create: null argument"); return RG_EINVAL; }
    if (Q == 0) { set_error("rg_prefetcher_create: Q must be >= 1"); return RG_EINVAL; }
    const HopData &h = s->hop[s->L];
    for (uint32_t b = 0; b < s->n_batches; ++b)
        if ((uint64_t)(h.off_host[b + 1] - h.off_host[b]) > slot_capacity_rows) {
            set_error("rg_prefetcher_create: batch %u has %lld rows, a slot holds %llu", b, (long long)(h.off_host[b + 1] - h.off_host[b]),
                      (unsigned long long)slot_capacity_rows);
            return RG_ERANGE;
        }
    rg_prefetcher *p = new (std::nothrow) rg_prefetcher();
    if (!p) { set_error("rg_prefetcher_create: out of host memory"); return RG_ENOMEM; }
    p->s = s; p->c = c; p->feat = *f; p->Q = Q;
    p->slot.assign(slot_buffers, slot_buffers + Q);
    p->out_stride = out_stride; p->capacity_rows = slot_capacity_rows;
    p->ready.assign(Q, nullptr); p->freed.assign(Q, nullptr); p->freed_valid.assign(Q, 0); p->stats.assign(Q, rg_gather_stats{0, 0, 0, 0});
    bool ok = hipStreamCreateWithFlags(&p->stream, hipStreamNonBlocking) == hipSuccess &&
              hipStreamCreateWithFlags(&p->side, hipStreamNonBlocking) == hipSuccess;
    for (uint32_t q = 0; ok && q < Q; ++q)
        ok = hipEventCreateWithFlags(&p->ready[q], hipEventDisableTiming) == hipSuccess &&
             hipEventCreateWithFlags(&p->freed[q], hipEventDisableTiming) == hipSuccess;
    if (!ok) {
        set_error("rg_prefetcher_create: cannot create streams / events");
        rg_prefetcher_destroy(p);
        return RG_EHIP;
    }
    *out = p;
    return RG_OK;
}

// Stages batches, in order, until the queue and the consumer together hold Q slots or the epoch is exhausted.
rg_status rg_prefetcher_fill(rg_prefetcher *p, uint32_t *issued)
{
    if (!p) { set_error("rg_prefetcher_fill: null argument"); return RG_EINVAL; }
    uint32_t n = 0;
    while (p->staged < p->s->n_batches && p->staged - p->released < p->Q) {
        const uint32_t b = p->staged, q = b % p->Q;
        if (p->freed_valid[q]) RG_HIP(hipStreamWaitEvent(p->stream, p->freed[q], 0));      // the consumer's last use of this slot
        RG_TRY(rg_gather_batch(p->s, p->c, &p->feat, b, p->slot[q], p->out_stride, p->capacity_rows, p->stream, p->side, &p->stats[q]));
        RG_HIP(hipEventRecord(p->ready[q], p->stream));
        ++p->staged;
        ++n;
    }
    if (issued) *issued = n;
    return RG_OK;
}

// The next batch of the epoch, in order.  If it was staged, `consumer_stream` is made to wait for its data;
// if the prefetcher has not got to it (the race of Sec. 3), it is gathered now on the consumer's stream.
rg_status rg_prefetcher_acquire(rg_prefetcher *p, void *consumer_stream, uint32_t *batch, void **out, rg_gather_stats *stats, int *was_staged)
{
    if (!p) { set_error("rg_prefetcher_acquire: null argument"); return RG_EINVAL; }
    if (p->acquired >= p->s->n_batches) { set_error("rg_prefetcher_acquire: the epoch is exhausted"); return RG_ERANGE; }
    if (p->acquired - p->released >= p->Q) { set_error("rg_prefetcher_acquire: all %u slots are held; release one first", p->Q); return RG_EINVAL; }
    const uint32_t b = p->acquired, q = b % p->Q;
    hipStream_t cs = as_stream(consumer_stream);
    if (b < p->staged) {
        RG_HIP(hipStreamWaitEvent(cs, p->ready[q], 0));
        if (was_staged) *was_staged = 1;
    } else {
        if (p->freed_valid[q]) RG_HIP(hipStreamWaitEvent(cs, p->freed[q], 0));
        RG_TRY(rg_gather_batch(p->s, p->c, &p->feat, b, p->slot[q], p->out_stride, p->capacity_rows, cs, nullptr, &p->stats[q]));
        p->staged = b + 1;
        if (was_staged) *was_staged = 0;
    }
    ++p->acquired;
    if (batch) *batch = b;
    if (out) *out = p->slot[q];
    if (stats) *stats = p->stats[q];
    return RG_OK;
}

// The consumer has finished (as of the work queued on consumer_stream) with the oldest slot it holds.
rg_status rg_prefetcher_release(rg_prefetcher *p, void *consumer_stream)
{
    if (!p) { set_error("rg_prefetcher_release: null argument"); return RG_EINVAL; }
    if (p->released >= p->acquired) { set_error("rg_prefetcher_release: no slot is held"); return RG_EINVAL; }
    const uint32_t q = p->released % p->Q;
    RG_HIP(hipEventRecord(p->freed[q], as_stream(consumer_stream)));
    p->freed_valid[q] = 1;
    ++p->released;
    return RG_OK;
}

rg_status rg_prefetcher_depth(const rg_prefetcher *p, uint32_t *staged_not_acquired, uint32_t *held)
{
    if (!p) { set_error("rg_prefetcher_depth: null argument"); return RG_EINVAL; }
    if (staged_not_acquired) *staged_not_acquired = p->staged - p->acquired;
    if (held) *held = p->acquired - p->released;
    return RG_OK;
}

void rg_prefetcher_destroy(rg_prefetcher *p)
{
    if (!p) return;
    if (p->stream) (void)hipStreamSynchronize(p->stream);
    if (p->side) (void)hipStreamSynchronize(p->side);
    for (hipEvent_t e : p->ready) if (e) (void)hipEventDestroy(e);
    for (hipEvent_t e : p->freed) if (e) (void)hipEventDestroy(e);
    if (p->stream) (void)hipStreamDestroy(p->stream);
    if (p->side) (void)hipStreamDestroy(p->side);
    delete p;
}

}  // extern "C"
