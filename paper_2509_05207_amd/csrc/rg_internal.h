// Internal declarations shared by the translation units of librapidgnn_hip.so.
// Nothing in here is part of the ABI (see include/rapidgnn.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include <atomic>
#include <mutex>
#include <string>
#include <vector>
#include <utility>

#include "rapidgnn.h"

namespace rg {

// ---------------------------------------------------------------- errors
void set_error(const char *fmt, ...);

#define RG_HIP(call)                                                                        \
    do {                                                                                    \
        hipError_t e__ = (call);                                                            \
        if (e__ != hipSuccess) {                                                            \
            rg::set_error("%s failed: %s (%s:%d)", #call, hipGetErrorString(e__), __FILE__, \
                          __LINE__);                                                        \
            return RG_EHIP;                                                                 \
        }                                                                                   \
    } while (0)

#define RG_TRY(expr)                  \
    do {                              \
        rg_status s__ = (expr);       \
        if (s__ != RG_OK) return s__; \
    } while (0)

// ---------------------------------------------------------------- memory
// Owns every buffer it hands out; frees them (through the same allocator) on
// destruction or release_all().
class Arena {
  public:
    explicit Arena(const rg_allocator *a);
    // Scratch of a call that launches kernels on `st`: the stream is drained before the buffers go back (they may be
    // handed to another thread's build at once), on every way out of the call -- unless the call has waited for the
    // stream itself and says so with drained().
    Arena(const rg_allocator *a, hipStream_t st);
    void drained() { drain_ = false; }
    ~Arena();
    Arena(const Arena &) = delete;
    Arena &operator=(const Arena &) = delete;

    // Device memory, 256-byte aligned by the underlying allocator.  bytes == 0
    // still returns a valid (tiny) allocation so kernels can take the pointer.
    rg_status dev(uint64_t bytes, void **out);
    rg_status pinned(uint64_t bytes, void **out);
    template <typename T> rg_status dev_n(uint64_t n, T **out) { return dev(n * sizeof(T), (void **)out); }
    // Device memory that holds zero bytes: a block that an earlier call handed back as all-zero (free_zeroed), or a
    // fresh one cleared on `st`.  The big per-batch bitmaps of a schedule build come and go this way, so that an
    // epoch clears only the parts the epoch before it touched instead of gigabytes.
    rg_status dev_zeroed(uint64_t bytes, void **out, hipStream_t st);
    // Hands a buffer back as all-zero: every byte is zero and the work that wrote it has completed.
    void free_zeroed(void *p);
    void free_one(void *p);     // early release of a single buffer
    void release_all();
    uint64_t bytes_in_use() const { return in_use_; }
    // The allocator this arena draws from (NULL = the library's own), for scratch that should come from the same place.
    const rg_allocator *allocator() const { return custom_ ? &a_ : nullptr; }

  private:
    struct Item { void *p; int kind; uint64_t bytes; };
    rg_allocator a_;
    bool custom_;
    std::vector<Item> items_;
    uint64_t in_use_ = 0;
    bool drain_ = false;
    hipStream_t drain_stream_ = nullptr;
};

// ---------------------------------------------------------------- last uses of a handle
// A gather served from a prepared plan returns while its kernels still read the schedule and the cache.  Each such
// call records, per stream, an event behind its last launch; a destroy call then knows exactly what it has to wait
// for (that handle's own readers), not for the whole device.
class UseLog {
  public:
    UseLog() = default;
    ~UseLog();
    UseLog(const UseLog &) = delete;
    UseLog &operator=(const UseLog &) = delete;
    void note(hipStream_t st);      // work just enqueued on st reads the handle
    bool idle();                    // every noted use has completed
    void wait();                    // blocks until idle
  private:
    struct Use { hipStream_t st; hipEvent_t ev; };
    std::mutex mu_;
    std::vector<Use> uses_;
    bool lost_ = false;             // an event could not be created or recorded: only a device-wide wait is safe
};

// ---------------------------------------------------------------- profiling
enum KernelGroup {
    KG_SAMPLER = 0, KG_FRONTIER = 1, KG_SORT = 2, KG_HIST = 3, KG_TOPK = 4,
    KG_PLAN = 5, KG_FILL = 6, KG_GATHER = 7, KG_MISS = 8, KG_OFFSETS = 9, KG_BLOCKS = 10
};
bool profiling_on();
// Records an event pair around a launch when profiling is enabled.
struct ScopedTimer {
    ScopedTimer(int group, hipStream_t st);
    ~ScopedTimer();
    int group; hipStream_t st; hipEvent_t e0 = nullptr, e1 = nullptr;
};

// ---------------------------------------------------------------- handles
struct HopData {
    int32_t *ids = nullptr;          // dev, frontier U_l, batches concatenated
    int64_t *off_dev = nullptr;      // dev, [beta + 1]
    std::vector<int64_t> off_host;   // [beta + 1]
    int64_t *samp_off = nullptr;     // dev, [|U_l| + 1]  (hops 0..L-1)
    int32_t *samp_nbr = nullptr;     // dev
    int64_t n_samples = 0;
    int32_t *src_pos = nullptr;      // dev, [n_samples]: block-local source index of every sample (after rg_schedule_build_blocks)
};

}  // namespace rg

struct rg_schedule {
    rg::Arena arena;
    int64_t n_nodes = 0;
    uint32_t n_batches = 0, L = 0;
    uint64_t T = 0;
    uint64_t uid = 0;                // identity for plan lookup (pointers can be reused)
    std::vector<rg::HopData> hop;    // L + 1 entries
    bool blocks_built = false;
    uint32_t *epoch_freq = nullptr;  // dev, [n_nodes]: in how many of the epoch's input sets each node is, or NULL (then the lists are tallied)
    mutable rg::UseLog uses;         // gathers in flight that read this schedule
    explicit rg_schedule(const rg_allocator *a) : arena(a) {}
};

namespace rg {

struct Plan {
    uint64_t schedule_uid = 0;
    int64_t *entry = nullptr;            // dev, [|U_L| total]: (tag << 62) | source row
    int32_t *miss_rows = nullptr;        // dev, output-row index of every miss, batches concatenated
    std::vector<int64_t> miss_off;       // host, [beta + 1]
    std::vector<rg_gather_stats> stats;  // host, [beta]
};

// Routing entry: source tag in the top two bits, source row below (handled as unsigned bits).
constexpr int64_t TAG_LOCAL = 0, TAG_CACHE = 1, TAG_REMOTE = 2;
constexpr int TAG_SHIFT = 62;
constexpr uint64_t ROW_MASK = ((uint64_t)1 << TAG_SHIFT) - 1;
__host__ __device__ inline int64_t make_entry(int64_t tag, int64_t row) { return (int64_t)(((uint64_t)tag << TAG_SHIFT) | ((uint64_t)row & ROW_MASK)); }

// ---------------------------------------------------------------- slot of a cached node
// Slot j of the cache table holds the j-th smallest cached ID, so a node's slot is its rank among the cached IDs.
// The cache keeps that as one record per 32 node IDs -- x: which of them are cached, y: how many cached IDs lie in
// front of the 32, z: which of them are local (the caller's is_local as bits), w: unused -- half a byte per node
// instead of the four of a dense slot_of array plus the byte of is_local (55 MB against 555 MB on a graph of 10^8
// nodes, so lookups meet cached lines and the select pass has next to nothing to write).
typedef uint4 SlotRec;
__device__ __forceinline__ int32_t slot_lookup(const SlotRec *__restrict__ recs, uint32_t v)
{
    const SlotRec p = recs[v >> 5];
    const uint32_t bit = 1u << (v & 31);
    return (p.x & bit) ? (int32_t)(p.y + __popc(p.x & (bit - 1))) : -1;
}

__host__ __device__ inline int64_t entry_tag(int64_t e) { return (int64_t)((uint64_t)e >> TAG_SHIFT); }
__host__ __device__ inline int64_t entry_row(int64_t e) { return (int64_t)((uint64_t)e & ROW_MASK); }

}  // namespace rg

struct rg_cache {
    rg::Arena arena;
    int64_t n_nodes = 0;
    uint64_t K_eff = 0;
    uint32_t row_bytes = 0;
    uint64_t stride = 0;
    int32_t *cache_ids = nullptr;    // dev, ascending
    uint32_t *freq = nullptr;        // dev, [n_nodes]; where the tally was kept in bytes: NULL until rg_cache_view asks for it
    uint8_t *freq8 = nullptr;        // dev, [n_nodes rounded up to 16]: the tally in bytes (no frequency can exceed 255), or NULL
    std::mutex view_mu;              // guards the making of freq and slot_of for rg_cache_view
    rg::SlotRec *slot_pairs = nullptr;   // dev, one record per 32 node IDs: the slot map (see slot_lookup)
    int32_t *slot_of = nullptr;      // dev, [n_nodes]: NULL until rg_cache_view asks for it
    void *rows = nullptr;            // dev, K_eff * stride
    std::vector<rg::Plan> plans;
    hipEvent_t ev_fork = nullptr, ev_join = nullptr;
    const void *remote_rows_seen = nullptr;   // the remote table the cache was built over ...
    bool remote_is_device = false;            // ... and whether it is device memory
    mutable rg::UseLog uses;                  // gathers in flight that read this cache
    explicit rg_cache(const rg_allocator *a) : arena(a) {}
    ~rg_cache();
};

namespace rg {

// ---------------------------------------------------------------- shared device-side helpers (host launchers)
// Exclusive prefix sum of n int32 counts into n + 1 int64 offsets (out[n] = total).
rg_status scan_i32_to_i64(const int32_t *in, int64_t *out, int64_t n, Arena &tmp, hipStream_t st);

// Copies rows selected by plan entries; see rg_gather.hip.
struct RowSources {
    const uint8_t *local_rows; uint64_t local_stride;
    const uint8_t *cache_rows; uint64_t cache_stride;
    const uint8_t *remote_rows; uint64_t remote_stride;
};
// mode 0: copy rows whose tag is local or cache (skip misses); mode 1: copy every row;
// list != nullptr: only the rows list[0..n_list) (used for the miss set).
rg_status launch_gather(const int64_t *entries, int64_t n_rows, const int32_t *list, int64_t n_list, int mode,
                        const RowSources &src, uint32_t row_bytes, uint8_t *out, uint64_t out_stride,
                        hipStream_t st, int group);

// A few small values read back from the device behind one stream synchronisation.  They travel through a pinned
// staging block (kept in a pool for the life of the process): a copy into pageable memory costs the runtime
// about 8 us more, and the builds read back a dozen such values per epoch.
class Readback {
  public:
    explicit Readback(hipStream_t st);
    ~Readback();
    Readback(const Readback &) = delete;
    Readback &operator=(const Readback &) = delete;
    rg_status add(void *host_dst, const void *dev_src, size_t bytes);    // notes the piece (dev_src is read when wait() runs, in stream order)
    rg_status wait();                                                    // fetches the pieces and synchronises the stream; the destinations are valid afterwards
  private:
    struct Part { void *dst; const void *src; size_t at, bytes; };
    hipStream_t st_;
    uint8_t *stage_ = nullptr;
    size_t used_ = 0;
    std::vector<Part> parts_;
    bool in_flight_ = false;
};

// Handles whose destroy call found readers still in flight wait here (default allocator only); they are released by
// a later library call once their readers have finished.  reap_retired(true) waits for all of them.
void reap_retired(bool wait);

// freq as rg_cache_view hands it out (widened from the byte tally at the first request)
rg_status cache_freq_view(const rg_cache *c, const uint32_t **out);
rg_status cache_slot_view(const rg_cache *c, const int32_t **out);

// One non-blocking stream per device, owned by the library and kept until the process ends: a call that has two
// independent pieces of device work forks the second onto it (event from the caller's stream, event back) so that
// both run at once.  Calls from several threads share it, which orders their forked pieces but changes no result.
rg_status helper_stream(hipStream_t *out);

// Where a cache build on this thread reports the bytes of its table as soon as the table is allocated (NULL: nowhere).
// The double-buffered cache sets it on its build thread so that the memory bound counts a C_sec under construction.
extern thread_local std::atomic<uint64_t> *tls_table_bytes_sink;

// True when p is device memory on the current device (false for pinned host memory).
bool is_device_memory(const void *p);

inline hipStream_t as_stream(void *p) { return reinterpret_cast<hipStream_t>(p); }

}  // namespace rg
