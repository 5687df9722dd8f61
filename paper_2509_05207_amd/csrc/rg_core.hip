// Error reporting, memory arena, kernel-group timers, the device prefix sum,
// graph validation and the handle accessors.
#include "rg_internal.h"

#include <cstring>

#include <atomic>
#include <cstdarg>
#include <cstdio>
#include <map>
#include <mutex>

namespace rg {

// ---------------------------------------------------------------- errors
static thread_local char g_err[512] = "";

void set_error(const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

// ---------------------------------------------------------------- device block cache
// hipMalloc / hipFree cost tens of microseconds to milliseconds each and hipFree synchronises the
// device.  An epoch's build allocates a few dozen buffers whose sizes repeat from epoch to epoch, so
// released blocks are kept (per device) and handed out again to requests of nearly the same size.
// Blocks only come back here after the work that used them has completed: a call's scratch arena drains
// the call's stream before it lets go (on every way out of the call), and a handle is released only once
// the gathers that read it have finished (UseLog).  rg_trim_memory() returns everything to the driver.
namespace {
struct BlockCache {
    std::mutex mu;
    std::multimap<std::pair<int, uint64_t>, void *> free_blocks;      // (device, bytes) -> block
    std::multimap<std::pair<int, uint64_t>, void *> zero_blocks;      // the same, blocks whose every byte is known to be zero
    std::map<void *, std::pair<int, uint64_t>> live;                  // blocks handed out
    uint64_t cached_bytes = 0;

    static uint64_t round_up(uint64_t bytes)
    {
        if (bytes <= 4096) return 4096;
        if (bytes < (1ull << 20)) { uint64_t r = 4096; while (r < bytes) r <<= 1; return r; }
        return (bytes + (1ull << 20) - 1) >> 20 << 20;
    }

    // zeroed: prefer a block that is known to hold nothing but zero bytes (*was_zero says whether one was found;
    // otherwise the caller clears what it got).  A request that finds no ordinary block takes a zeroed one.
    void *take(uint64_t bytes, hipError_t *err, bool zeroed = false, bool *was_zero = nullptr)
    {
        int dev = 0;
        (void)hipGetDevice(&dev);
        const uint64_t want = round_up(bytes);
        if (was_zero) *was_zero = false;
        {
            std::lock_guard<std::mutex> lk(mu);
            auto fits = [&](std::multimap<std::pair<int, uint64_t>, void *> &pool) -> void * {
                auto it = pool.lower_bound({dev, want});
                if (it == pool.end() || it->first.first != dev || it->first.second > want + want / 8 + (1ull << 20)) return nullptr;
                void *p = it->second;
                live[p] = it->first;
                cached_bytes -= it->first.second;
                pool.erase(it);
                return p;
            };
            if (zeroed) {
                if (void *p = fits(zero_blocks)) { if (was_zero) *was_zero = true; return p; }
                if (void *p = fits(free_blocks)) return p;
            } else {
                if (void *p = fits(free_blocks)) return p;
                if (void *p = fits(zero_blocks)) return p;
            }
        }
        void *p = nullptr;
        hipError_t e = hipMalloc(&p, want);
        if (e != hipSuccess) {                       // release what waits for its readers, give the cache back to the driver, try once more
            (void)hipGetLastError();
            reap_retired(true);
            trim();
            e = hipMalloc(&p, want);
        }
        if (e != hipSuccess) { (void)hipGetLastError(); *err = e; return nullptr; }
        std::lock_guard<std::mutex> lk(mu);
        live[p] = {dev, want};
        return p;
    }

    uint64_t size_of(void *p)
    {
        std::lock_guard<std::mutex> lk(mu);
        auto it = live.find(p);
        return it == live.end() ? 0 : it->second.second;
    }

    // all_zero: the caller vouches that every byte of the block is zero and that nothing will write it any more
    void give(void *p, bool all_zero = false)
    {
        std::lock_guard<std::mutex> lk(mu);
        auto it = live.find(p);
        if (it == live.end()) { (void)hipFree(p); return; }
        (all_zero ? zero_blocks : free_blocks).insert({it->second, p});
        cached_bytes += it->second.second;
        live.erase(it);
    }

    void trim()
    {
        std::lock_guard<std::mutex> lk(mu);
        for (auto &kv : free_blocks) (void)hipFree(kv.second);
        for (auto &kv : zero_blocks) (void)hipFree(kv.second);
        free_blocks.clear();
        zero_blocks.clear();
        cached_bytes = 0;
    }
};
BlockCache g_blocks;
}  // namespace

// ---------------------------------------------------------------- small readbacks
namespace {
constexpr size_t STAGE_BYTES = 8192;
struct StagePool {
    std::mutex mu;
    std::vector<uint8_t *> free_blocks;
    uint8_t *take()
    {
        {
            std::lock_guard<std::mutex> lk(mu);
            if (!free_blocks.empty()) { uint8_t *p = free_blocks.back(); free_blocks.pop_back(); return p; }
        }
        void *p = nullptr;
        if (hipHostMalloc(&p, STAGE_BYTES, hipHostMallocDefault) != hipSuccess) { (void)hipGetLastError(); return nullptr; }
        return static_cast<uint8_t *>(p);
    }
    void give(uint8_t *p) { std::lock_guard<std::mutex> lk(mu); free_blocks.push_back(p); }
};
StagePool g_stages;
}  // namespace

// Several small pieces are fetched by one kernel that writes them straight into the pinned block (host memory the
// device can address), not by a copy each: a copy is a launch of its own, and they run one after the other.
constexpr int PACK_PARTS = 8;
struct PackArgs {
    const uint8_t *src[PACK_PARTS];
    uint32_t at[PACK_PARTS], bytes[PACK_PARTS];
    int n;
};
__global__ void __launch_bounds__(256) pack_pieces_kernel(PackArgs a, uint8_t *__restrict__ stage)
{
    for (int p = 0; p < a.n; ++p) {
        const uint8_t *src = a.src[p];
        uint8_t *dst = stage + a.at[p];
        const uint32_t bytes = a.bytes[p];
        if ((((uintptr_t)src | bytes) & 3u) == 0) {                     // (the block's offsets are multiples of 16)
            for (uint32_t i = threadIdx.x; i < bytes / 4; i += blockDim.x) reinterpret_cast<uint32_t *>(dst)[i] = reinterpret_cast<const uint32_t *>(src)[i];
        } else {
            for (uint32_t i = threadIdx.x; i < bytes; i += blockDim.x) dst[i] = src[i];
        }
    }
}

Readback::Readback(hipStream_t st) : st_(st) {}
Readback::~Readback()
{
    if (!stage_) return;
    if (in_flight_) (void)hipStreamSynchronize(st_);      // left in the middle of wait() (an error path): writes into the block may still be in flight
    g_stages.give(stage_);
}

rg_status Readback::add(void *host_dst, const void *dev_src, size_t bytes)
{
    if (bytes == 0) return RG_OK;
    if (!stage_) stage_ = g_stages.take();
    const size_t at = (used_ + 15) & ~(size_t)15;
    if (!stage_ || at + bytes > STAGE_BYTES) {           // too large for the block (or no pinned memory to be had): straight to the destination
        RG_HIP(hipMemcpyAsync(host_dst, dev_src, bytes, hipMemcpyDeviceToHost, st_));
        return RG_OK;
    }
    parts_.push_back({host_dst, dev_src, at, bytes});
    used_ = at + bytes;
    return RG_OK;
}

rg_status Readback::wait()
{
    in_flight_ = true;
    if (parts_.size() == 1) {
        RG_HIP(hipMemcpyAsync(stage_ + parts_[0].at, parts_[0].src, parts_[0].bytes, hipMemcpyDeviceToHost, st_));
    } else {
        for (size_t first = 0; first < parts_.size(); first += PACK_PARTS) {
            PackArgs a{};
            a.n = (int)std::min<size_t>(PACK_PARTS, parts_.size() - first);
            for (int p = 0; p < a.n; ++p) {
                const Part &part = parts_[first + p];
                a.src[p] = static_cast<const uint8_t *>(part.src);
                a.at[p] = (uint32_t)part.at;
                a.bytes[p] = (uint32_t)part.bytes;
            }
            hipLaunchKernelGGL(pack_pieces_kernel, dim3(1), dim3(256), 0, st_, a, stage_);
            RG_HIP(hipGetLastError());
        }
    }
    RG_HIP(hipStreamSynchronize(st_));
    in_flight_ = false;
    for (const Part &p : parts_) memcpy(p.dst, stage_ + p.at, p.bytes);
    parts_.clear();
    used_ = 0;
    return RG_OK;
}

// ---------------------------------------------------------------- arena
Arena::Arena(const rg_allocator *a)
{
    custom_ = (a != nullptr && a->alloc != nullptr && a->free != nullptr);
    if (custom_) a_ = *a; else a_ = rg_allocator{nullptr, nullptr, nullptr};
}

Arena::Arena(const rg_allocator *a, hipStream_t st) : Arena(a)
{
    drain_ = true;
    drain_stream_ = st;
}

Arena::~Arena() { release_all(); }

rg_status Arena::dev(uint64_t bytes, void **out)
{
    uint64_t want = bytes ? bytes : 256;
    void *p = nullptr;
    if (custom_) {
        p = a_.alloc(want, 1, a_.ctx);
        if (!p) { set_error("allocator callback returned NULL for %llu device bytes", (unsigned long long)want); return RG_ENOMEM; }
    } else {
        hipError_t e = hipSuccess;
        p = g_blocks.take(want, &e);
        if (!p) {
            set_error("hipMalloc(%llu) failed: %s", (unsigned long long)want, hipGetErrorString(e));
            return RG_ENOMEM;
        }
    }
    items_.push_back({p, 1, want});
    in_use_ += want;
    *out = p;
    return RG_OK;
}

rg_status Arena::dev_zeroed(uint64_t bytes, void **out, hipStream_t st)
{
    if (custom_) {
        RG_TRY(dev(bytes, out));
        RG_HIP(hipMemsetAsync(*out, 0, bytes ? bytes : 256, st));
        return RG_OK;
    }
    const uint64_t want = bytes ? bytes : 256;
    hipError_t e = hipSuccess;
    bool was_zero = false;
    void *p = g_blocks.take(want, &e, true, &was_zero);
    if (!p) {
        set_error("hipMalloc(%llu) failed: %s", (unsigned long long)want, hipGetErrorString(e));
        return RG_ENOMEM;
    }
    items_.push_back({p, 1, want});
    in_use_ += want;
    *out = p;
    if (!was_zero) RG_HIP(hipMemsetAsync(p, 0, g_blocks.size_of(p), st));      // the whole block: it may come back as all-zero for a larger request
    return RG_OK;
}

void Arena::free_zeroed(void *p)
{
    if (!p) return;
    for (size_t i = 0; i < items_.size(); ++i) {
        if (items_[i].p == p) {
            if (custom_) a_.free(p, items_[i].kind, a_.ctx);
            else g_blocks.give(p, true);
            in_use_ -= items_[i].bytes;
            items_[i] = items_.back();
            items_.pop_back();
            return;
        }
    }
}

rg_status Arena::pinned(uint64_t bytes, void **out)
{
    uint64_t want = bytes ? bytes : 256;
    void *p = nullptr;
    if (custom_) {
        p = a_.alloc(want, 0, a_.ctx);
        if (!p) { set_error("allocator callback returned NULL for %llu pinned bytes", (unsigned long long)want); return RG_ENOMEM; }
    } else {
        hipError_t e = hipHostMalloc(&p, want, hipHostMallocDefault);
        if (e != hipSuccess) {
            (void)hipGetLastError();
            set_error("hipHostMalloc(%llu) failed: %s", (unsigned long long)want, hipGetErrorString(e));
            return RG_ENOMEM;
        }
    }
    items_.push_back({p, 0, want});
    in_use_ += want;
    *out = p;
    return RG_OK;
}

void Arena::free_one(void *p)
{
    if (!p) return;
    for (size_t i = 0; i < items_.size(); ++i) {
        if (items_[i].p == p) {
            if (custom_) a_.free(p, items_[i].kind, a_.ctx);
            else if (items_[i].kind == 1) g_blocks.give(p);
            else (void)hipHostFree(p);
            in_use_ -= items_[i].bytes;
            items_[i] = items_.back();
            items_.pop_back();
            return;
        }
    }
}

void Arena::release_all()
{
    if (drain_ && !items_.empty()) (void)hipStreamSynchronize(drain_stream_);     // kernels of the call that owns this scratch may still run
    drain_ = false;
    for (auto &it : items_) {
        if (custom_) a_.free(it.p, it.kind, a_.ctx);
        else if (it.kind == 1) g_blocks.give(it.p);
        else (void)hipHostFree(it.p);
    }
    items_.clear();
    in_use_ = 0;
}

// ---------------------------------------------------------------- last uses, retired handles
UseLog::~UseLog()
{
    for (Use &u : uses_) (void)hipEventDestroy(u.ev);
}

void UseLog::note(hipStream_t st)
{
    std::lock_guard<std::mutex> lk(mu_);
    for (Use &u : uses_)
        if (u.st == st) {
            if (hipEventRecord(u.ev, st) != hipSuccess) { (void)hipGetLastError(); lost_ = true; }
            return;
        }
    hipEvent_t ev = nullptr;
    if (hipEventCreateWithFlags(&ev, hipEventDisableTiming) != hipSuccess) { (void)hipGetLastError(); lost_ = true; return; }
    if (hipEventRecord(ev, st) != hipSuccess) { (void)hipGetLastError(); (void)hipEventDestroy(ev); lost_ = true; return; }
    uses_.push_back({st, ev});
}

bool UseLog::idle()
{
    std::lock_guard<std::mutex> lk(mu_);
    if (lost_) return false;
    for (Use &u : uses_) {
        const hipError_t e = hipEventQuery(u.ev);
        if (e == hipErrorNotReady) return false;
        if (e != hipSuccess) { (void)hipGetLastError(); return false; }
    }
    return true;
}

void UseLog::wait()
{
    std::lock_guard<std::mutex> lk(mu_);
    if (lost_) { (void)hipDeviceSynchronize(); lost_ = false; return; }
    for (Use &u : uses_)
        if (hipEventSynchronize(u.ev) != hipSuccess) { (void)hipGetLastError(); (void)hipDeviceSynchronize(); return; }
}

namespace {
struct Retired {
    std::mutex mu;
    std::vector<rg_schedule *> schedules;
    std::vector<rg_cache *> caches;
};
Retired &retired() { static Retired *r = new Retired(); return *r; }     // (never destructed: no HIP calls at process exit)

template <typename H> void reap_list(std::vector<H *> &list, bool wait)
{
    size_t kept = 0;
    for (H *h : list) {
        if (wait) h->uses.wait();
        if (wait || h->uses.idle()) delete h;
        else list[kept++] = h;
    }
    list.resize(kept);
}

// A handle leaves: at once when nothing reads it any more; with a caller's allocator after a wait for its own
// readers (the allocator may not outlive the call); otherwise it is parked until a later call finds it idle.
template <typename H> void retire(H *h, std::vector<H *> Retired::*list)
{
    reap_retired(false);
    if (h->arena.allocator()) h->uses.wait();
    if (h->arena.allocator() || h->uses.idle()) { delete h; return; }
    Retired &r = retired();
    std::lock_guard<std::mutex> lk(r.mu);
    (r.*list).push_back(h);
}
}  // namespace

rg_status helper_stream(hipStream_t *out)
{
    static std::mutex mu;
    static hipStream_t streams[64] = {};
    int dev = 0;
    RG_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= 64) { set_error("helper_stream: device %d out of range", dev); return RG_EINVAL; }
    std::lock_guard<std::mutex> lk(mu);
    if (!streams[dev]) RG_HIP(hipStreamCreateWithFlags(&streams[dev], hipStreamNonBlocking));
    *out = streams[dev];
    return RG_OK;
}

void reap_retired(bool wait)
{
    Retired &r = retired();
    std::lock_guard<std::mutex> lk(r.mu);
    reap_list(r.schedules, wait);
    reap_list(r.caches, wait);
}

// ---------------------------------------------------------------- profiling
static std::atomic<int> g_prof_on{0};
static std::mutex g_prof_mu;
struct Pending { int group; hipEvent_t e0, e1; };
static std::vector<Pending> g_pending;
static std::vector<hipEvent_t> g_free_events;
static double g_ms[RG_N_KERNEL_GROUPS];
static uint64_t g_launches[RG_N_KERNEL_GROUPS];

bool profiling_on() { return g_prof_on.load(std::memory_order_relaxed) != 0; }

ScopedTimer::ScopedTimer(int g, hipStream_t s) : group(g), st(s)
{
    if (g < 0 || !profiling_on()) return;       // group -1: a launch that is never timed
    {
        std::lock_guard<std::mutex> lk(g_prof_mu);
        if (g_free_events.size() >= 2) {
            e0 = g_free_events.back(); g_free_events.pop_back();
            e1 = g_free_events.back(); g_free_events.pop_back();
        }
    }
    if (!e0 && (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess)) { e0 = e1 = nullptr; return; }
    (void)hipEventRecord(e0, st);
}

ScopedTimer::~ScopedTimer()
{
    if (!e0) return;
    (void)hipEventRecord(e1, st);
    std::lock_guard<std::mutex> lk(g_prof_mu);
    g_pending.push_back({group, e0, e1});
}

static void drain_pending_locked()
{
    for (auto &p : g_pending) {
        float ms = 0.f;
        if (hipEventSynchronize(p.e1) == hipSuccess && hipEventElapsedTime(&ms, p.e0, p.e1) == hipSuccess) {
            g_ms[p.group] += ms;
            g_launches[p.group] += 1;
        }
        g_free_events.push_back(p.e0);
        g_free_events.push_back(p.e1);
    }
    g_pending.clear();
}

// ---------------------------------------------------------------- prefix sum
// Per-block totals, then per-block local scans plus the sum of the totals in front: one launch for a single block,
// two while a block can add up its predecessors' totals itself, three (with a scan of the totals between) beyond.
// Each block covers SCAN_TILE consecutive elements.
constexpr int SCAN_THREADS = 256;
constexpr int SCAN_PER_THREAD = 16;
constexpr int SCAN_TILE = SCAN_THREADS * SCAN_PER_THREAD;

__device__ __forceinline__ int64_t block_exclusive_scan_i64(int64_t x, int64_t *total, int64_t *lds /* [SCAN_THREADS/64 + 1] */)
{
    // wave-level inclusive scan by shuffles, then across the block's waves through LDS
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int64_t incl = x;
    for (int d = 1; d < 64; d <<= 1) {
        int64_t y = __shfl_up(incl, d, 64);
        if (lane >= d) incl += y;
    }
    if (lane == 63) lds[wave] = incl;
    __syncthreads();
    int64_t base = 0, tot = 0;
    const int nw = blockDim.x >> 6;
    for (int w = 0; w < nw; ++w) {
        int64_t s = lds[w];
        if (w < wave) base += s;
        tot += s;
    }
    __syncthreads();
    *total = tot;
    return base + incl - x;
}

__global__ void __launch_bounds__(SCAN_THREADS) scan_block_totals(const int32_t *__restrict__ in, int64_t n, int64_t *__restrict__ block_tot)
{
    __shared__ int64_t lds[SCAN_THREADS / 64 + 1];
    const int64_t base = (int64_t)blockIdx.x * SCAN_TILE;
    int64_t s = 0;
    for (int k = 0; k < SCAN_PER_THREAD; ++k) {
        int64_t i = base + (int64_t)k * SCAN_THREADS + threadIdx.x;
        if (i < n) s += in[i];
    }
    int64_t tot;
    (void)block_exclusive_scan_i64(s, &tot, lds);
    if (threadIdx.x == 0) block_tot[blockIdx.x] = tot;
}

__global__ void __launch_bounds__(SCAN_THREADS) scan_of_totals(int64_t *__restrict__ block_tot, int64_t n_blocks, int64_t *__restrict__ grand_total)
{
    __shared__ int64_t lds[SCAN_THREADS / 64 + 1];
    int64_t carry = 0;
    for (int64_t base = 0; base < n_blocks; base += SCAN_THREADS) {
        int64_t i = base + threadIdx.x;
        int64_t x = i < n_blocks ? block_tot[i] : 0;
        int64_t tot;
        int64_t ex = block_exclusive_scan_i64(x, &tot, lds);
        if (i < n_blocks) block_tot[i] = carry + ex;
        carry += tot;
    }
    if (threadIdx.x == 0) *grand_total = carry;
}

// FUSED: block_base is the raw per-block totals; the block adds up the totals in front of its own (a few thousand
// at most, see scan_i32_to_i64) instead of reading a scanned table, and the last block writes the grand total.
template <bool FUSED>
__global__ void __launch_bounds__(SCAN_THREADS) scan_apply(const int32_t *__restrict__ in, int64_t n, const int64_t *__restrict__ block_base,
                                                           int64_t *__restrict__ out)
{
    __shared__ int64_t lds[SCAN_THREADS / 64 + 1];
    int64_t base;
    if (FUSED) {
        int64_t part = 0;
        for (int64_t j = threadIdx.x; j < (int64_t)blockIdx.x; j += SCAN_THREADS) part += block_base[j];
        (void)block_exclusive_scan_i64(part, &base, lds);
    } else base = block_base[blockIdx.x];
    // thread t owns SCAN_PER_THREAD consecutive elements so one block scan suffices
    const int64_t first = (int64_t)blockIdx.x * SCAN_TILE + (int64_t)threadIdx.x * SCAN_PER_THREAD;
    int32_t v[SCAN_PER_THREAD];
    int64_t s = 0;
    for (int k = 0; k < SCAN_PER_THREAD; ++k) {
        int64_t i = first + k;
        v[k] = i < n ? in[i] : 0;
        s += v[k];
    }
    int64_t tot;
    int64_t run = base + block_exclusive_scan_i64(s, &tot, lds);
    for (int k = 0; k < SCAN_PER_THREAD; ++k) {
        int64_t i = first + k;
        if (i < n) out[i] = run;
        run += v[k];
    }
    if (FUSED && blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) out[n] = base + tot;
}

constexpr int64_t SCAN_FUSED_BLOCKS = 4096;      // up to here a block adds up its predecessors' totals itself (16 M elements)

rg_status scan_i32_to_i64(const int32_t *in, int64_t *out, int64_t n, Arena &tmp, hipStream_t st)
{
    const int64_t n_blocks = (n + SCAN_TILE - 1) / SCAN_TILE;
    if (n_blocks <= 1) {
        // one block: nothing in front of it, its own total is the grand total (n = 0 writes out[0] = 0)
        hipLaunchKernelGGL(scan_apply<true>, dim3(1), dim3(SCAN_THREADS), 0, st, in, n, (const int64_t *)nullptr, out);
        RG_HIP(hipGetLastError());
        return RG_OK;
    }
    int64_t *block_tot = nullptr;
    RG_TRY(tmp.dev_n<int64_t>((uint64_t)n_blocks, &block_tot));
    hipLaunchKernelGGL(scan_block_totals, dim3((unsigned)n_blocks), dim3(SCAN_THREADS), 0, st, in, n, block_tot);
    if (n_blocks <= SCAN_FUSED_BLOCKS) {
        hipLaunchKernelGGL(scan_apply<true>, dim3((unsigned)n_blocks), dim3(SCAN_THREADS), 0, st, in, n, block_tot, out);
    } else {
        hipLaunchKernelGGL(scan_of_totals, dim3(1), dim3(SCAN_THREADS), 0, st, block_tot, n_blocks, out + n);
        hipLaunchKernelGGL(scan_apply<false>, dim3((unsigned)n_blocks), dim3(SCAN_THREADS), 0, st, in, n, block_tot, out);
    }
    RG_HIP(hipGetLastError());
    return RG_OK;
}

// ---------------------------------------------------------------- graph validation
__global__ void validate_rows(int64_t n_nodes, const int64_t *__restrict__ indptr, const int32_t *__restrict__ indices,
                              unsigned long long *__restrict__ n_bad)
{
    // one wave per row, grid-stride
    const int lane = threadIdx.x & 63;
    const int64_t wave0 = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int64_t n_waves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    unsigned long long bad = 0;
    for (int64_t v = wave0; v < n_nodes; v += n_waves) {
        const int64_t b = indptr[v], e = indptr[v + 1];
        if (e < b || (v == 0 && b != 0)) { if (lane == 0) ++bad; continue; }
        for (int64_t j = b + lane; j < e; j += 64) {
            const int32_t u = indices[j];
            if (u < 0 || u >= n_nodes) ++bad;
            else if (j > b && indices[j - 1] >= u) ++bad;
        }
    }
    if (bad) atomicAdd(n_bad, bad);
}

}  // namespace rg

rg_cache::~rg_cache()
{
    if (ev_fork) (void)hipEventDestroy(ev_fork);
    if (ev_join) (void)hipEventDestroy(ev_join);
}

using namespace rg;

extern "C" {

const char *rg_last_error(void) { return g_err; }

void rg_profile_enable(int on) { g_prof_on.store(on ? 1 : 0); }

void rg_profile_reset(void)
{
    std::lock_guard<std::mutex> lk(g_prof_mu);
    drain_pending_locked();
    for (int i = 0; i < RG_N_KERNEL_GROUPS; ++i) { g_ms[i] = 0.0; g_launches[i] = 0; }
}

rg_status rg_profile_read(double *ms, uint64_t *launches)
{
    if (!ms || !launches) { set_error("rg_profile_read: null output"); return RG_EINVAL; }
    std::lock_guard<std::mutex> lk(g_prof_mu);
    drain_pending_locked();
    for (int i = 0; i < RG_N_KERNEL_GROUPS; ++i) { ms[i] = g_ms[i]; launches[i] = g_launches[i]; }
    return RG_OK;
}

rg_status rg_graph_validate(const rg_graph *g, void *stream, uint64_t *n_bad)
{
    if (!g || !n_bad || !g->indptr) { set_error("rg_graph_validate: null argument"); return RG_EINVAL; }
    if (g->n_nodes < 0 || g->n_nodes >= ((int64_t)1 << 31)) { set_error("rg_graph_validate: n_nodes out of range"); return RG_ERANGE; }
    hipStream_t st = as_stream(stream);
    unsigned long long *d = nullptr;
    RG_HIP(hipMalloc((void **)&d, sizeof(unsigned long long)));
    rg_status rc = RG_OK;
    do {
        if (hipMemsetAsync(d, 0, sizeof(unsigned long long), st) != hipSuccess) { rc = RG_EHIP; break; }
        if (g->n_nodes > 0) {
            int64_t blocks = (g->n_nodes + 3) / 4;
            if (blocks > 65536) blocks = 65536;
            hipLaunchKernelGGL(validate_rows, dim3((unsigned)blocks), dim3(256), 0, st, g->n_nodes, g->indptr, g->indices, d);
        }
        unsigned long long h = 0;
        if (hipMemcpyAsync(&h, d, sizeof(h), hipMemcpyDeviceToHost, st) != hipSuccess) { rc = RG_EHIP; break; }
        if (hipStreamSynchronize(st) != hipSuccess) { rc = RG_EHIP; break; }
        *n_bad = h;
    } while (0);
    if (rc != RG_OK) set_error("rg_graph_validate: HIP call failed: %s", hipGetErrorString(hipGetLastError()));
    (void)hipFree(d);
    return rc;
}

rg_status rg_schedule_info(const rg_schedule *s, uint32_t *n_batches, uint32_t *L, int64_t *n_nodes)
{
    if (!s) { set_error("rg_schedule_info: null schedule"); return RG_EINVAL; }
    if (n_batches) *n_batches = s->n_batches;
    if (L) *L = s->L;
    if (n_nodes) *n_nodes = s->n_nodes;
    return RG_OK;
}

rg_status rg_schedule_frontier(const rg_schedule *s, uint32_t hop, const int32_t **ids_dev,
                               const int64_t **batch_off_dev, const int64_t **batch_off_host)
{
    if (!s) { set_error("rg_schedule_frontier: null schedule"); return RG_EINVAL; }
    if (hop > s->L) { set_error("rg_schedule_frontier: hop %u > L = %u", hop, s->L); return RG_ERANGE; }
    const HopData &h = s->hop[hop];
    if (ids_dev) *ids_dev = h.ids;
    if (batch_off_dev) *batch_off_dev = h.off_dev;
    if (batch_off_host) *batch_off_host = h.off_host.data();
    return RG_OK;
}

rg_status rg_schedule_seeds(const rg_schedule *s, const int32_t **seeds_dev, const int64_t **batch_off_dev)
{
    if (!s) { set_error("rg_schedule_seeds: null schedule"); return RG_EINVAL; }
    return rg_schedule_frontier(s, 0, seeds_dev, batch_off_dev, nullptr);
}

rg_status rg_schedule_samples(const rg_schedule *s, uint32_t hop, const int64_t **samp_off_dev,
                              const int32_t **samp_nbr_dev, int64_t *n_samples)
{
    if (!s) { set_error("rg_schedule_samples: null schedule"); return RG_EINVAL; }
    if (hop >= s->L) { set_error("rg_schedule_samples: hop %u >= L = %u", hop, s->L); return RG_ERANGE; }
    const HopData &h = s->hop[hop];
    if (samp_off_dev) *samp_off_dev = h.samp_off;
    if (samp_nbr_dev) *samp_nbr_dev = h.samp_nbr;
    if (n_samples) *n_samples = h.n_samples;
    return RG_OK;
}

rg_status rg_cache_view(const rg_cache *c, uint64_t *K_eff, const int32_t **cache_ids_dev, const uint32_t **freq_dev,
                        const int32_t **slot_of_dev, const void **rows_dev, uint64_t *stride)
{
    if (!c) { set_error("rg_cache_view: null cache"); return RG_EINVAL; }
    if (K_eff) *K_eff = c->K_eff;
    if (cache_ids_dev) *cache_ids_dev = c->cache_ids;
    if (freq_dev) RG_TRY(cache_freq_view(c, freq_dev));
    if (slot_of_dev) RG_TRY(cache_slot_view(c, slot_of_dev));
    if (rows_dev) *rows_dev = c->rows;
    if (stride) *stride = c->stride;
    return RG_OK;
}

void rg_schedule_destroy(rg_schedule *s)
{
    if (s) retire(s, &Retired::schedules);
}

void rg_trim_memory(void)
{
    reap_retired(true);
    g_blocks.trim();
}

void rg_cache_destroy(rg_cache *c)
{
    if (c) retire(c, &Retired::caches);
}

}  // extern "C"
