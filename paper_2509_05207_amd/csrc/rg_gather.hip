// rg_gather_batch: the feature block of one batch (Alg. 1 inner loop).
//
// A batch's block is n_rows byte rows; the kernel works on the flat space of
// (row, vector) pairs so that consecutive lanes copy consecutive vectors of a
// row and run on into the next row: no lane idles whatever the row width.
// Each thread keeps CHUNKS_IN_FLIGHT independent loads outstanding before it
// stores (stores are non-temporal: the block is consumed by a later kernel,
// not by this one).  The source of a row comes from its 8-byte routing entry:
// local table, cache table or remote table.
//
// The miss set is copied by the same kernel over the batch's miss list.  When
// the remote table is pinned host memory (mapped into the device's address
// space) that launch goes to the side stream and its loads cross the host
// link -- SyncPull without host-side packing or staging.  When the remote
// table is device memory, one launch on the main stream copies every row.
#include "rg_internal.h"

#include <algorithm>
#include <mutex>

namespace rg {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

template <int W> struct VecT;
template <> struct VecT<16> { using type = u32x4; };
template <> struct VecT<8> { using type = u32x2; };
template <> struct VecT<4> { using type = uint32_t; };
template <> struct VecT<2> { using type = uint16_t; };
template <> struct VecT<1> { using type = uint8_t; };

// A piece of W bytes at an address that is only known to be a multiple of A bytes.  Global memory takes
// vector accesses at any dword-aligned address, so rows whose base and stride are multiples of 4 (any
// fp32 width, even bf16/fp16 widths) are copied with 16-byte vectors whatever their 16-byte phase.
template <int W, int A> struct PieceT { typedef typename VecT<W>::type type __attribute__((aligned(A < W ? A : W))); };

template <int W, int A>
__device__ __forceinline__ void copy_piece(const uint8_t *src, uint8_t *dst)
{
    using P = typename PieceT<W, A>::type;
    *reinterpret_cast<P *>(dst) = *reinterpret_cast<const P *>(src);
}

template <int VEC, int A>
__device__ __forceinline__ void copy_tail(const uint8_t *src, uint8_t *dst, uint32_t tail)
{
    // tail < VEC, at an offset that is a multiple of VEC; pieces of decreasing power-of-two width
    if constexpr (VEC > 8) { if (tail & 8u) { copy_piece<8, A>(src, dst); src += 8; dst += 8; } }
    if constexpr (VEC > 4) { if (tail & 4u) { copy_piece<4, A>(src, dst); src += 4; dst += 4; } }
    if constexpr (VEC > 2) { if (tail & 2u) { copy_piece<2, A>(src, dst); src += 2; dst += 2; } }
    if constexpr (VEC > 1) { if (tail & 1u) { copy_piece<1, A>(src, dst); } }
}

constexpr int GATHER_THREADS = 256;
constexpr int CHUNKS_IN_FLIGHT = 8;

// TAILPIECE = false: every piece is a full vector.  Either row_bytes is a multiple of VEC, or the last piece of a
// row is the vector that ENDS at the row's end and overlaps its predecessor (both write the same bytes there), so
// that no lane leaves the vector path.  TAILPIECE = true (row widths that are no multiple of 4, or below VEC): the
// last piece is copied in 8/4/2/1-byte parts.
template <int VEC, int A, bool TAILPIECE>
__global__ void __launch_bounds__(GATHER_THREADS) gather_rows_kernel(const int64_t *__restrict__ entries, int64_t n_rows,
                                                                     const int32_t *__restrict__ list, int64_t n_list, int mode,
                                                                     RowSources src, uint32_t row_bytes,
                                                                     uint8_t *__restrict__ out, uint64_t out_stride, int chunks)
{
    using T = typename VecT<VEC>::type;
    using P = typename PieceT<VEC, A>::type;
    const uint32_t cpr = row_bytes / VEC, tail = row_bytes % VEC;
    const uint32_t cpt = cpr + (tail ? 1u : 0u);                  // pieces per row: full vectors, then the last piece
    const uint32_t last_off = TAILPIECE ? cpr * VEC : row_bytes - VEC;     // where the piece after the full vectors starts
    const uint64_t n_work = (uint64_t)(list ? n_list : n_rows);
    const uint64_t total = n_work * cpt;
    // A workgroup takes GATHER_THREADS * chunks consecutive pieces per round (chunks <= CHUNKS_IN_FLIGHT, fewer for
    // a block of rows too small to fill the chip otherwise): one contiguous span of the output, 32 KB with 16-byte
    // pieces.  Within a round the flat index -> (work item, piece) pair is advanced by GATHER_THREADS without
    // dividing again.
    const uint32_t ROUND = GATHER_THREADS * (uint32_t)chunks;
    const uint32_t dq = GATHER_THREADS / cpt;
    const uint32_t dr = GATHER_THREADS - dq * cpt;

    for (uint64_t base = (uint64_t)blockIdx.x * ROUND + threadIdx.x; base < total; base += (uint64_t)gridDim.x * ROUND) {
        uint64_t idx = base;
        uint64_t w = idx / cpt;
        uint32_t c = (uint32_t)(idx - w * cpt);
        T v[CHUNKS_IN_FLIGHT];
        const uint8_t *sp[CHUNKS_IN_FLIGHT];
        uint8_t *dp[CHUNKS_IN_FLIGHT];
        int kind[CHUNKS_IN_FLIGHT];                                // 0 nothing, 1 full vector, 2 last piece in parts
#pragma unroll
        for (int k = 0; k < CHUNKS_IN_FLIGHT; ++k) {
            kind[k] = 0;
            sp[k] = nullptr; dp[k] = nullptr;
            if (k < chunks && idx < total) {
                const int64_t r = list ? (int64_t)list[w] : (int64_t)w;
                const int64_t e = entries[r];
                const int64_t tag = entry_tag(e), row = entry_row(e);
                if (!(mode == 0 && tag == TAG_REMOTE)) {
                    const uint8_t *base = tag == TAG_LOCAL ? src.local_rows + (uint64_t)row * src.local_stride
                                        : tag == TAG_CACHE ? src.cache_rows + (uint64_t)row * src.cache_stride
                                                           : src.remote_rows + (uint64_t)row * src.remote_stride;
                    const uint32_t o = c < cpr ? c * VEC : last_off;
                    sp[k] = base + o;
                    dp[k] = out + (uint64_t)r * out_stride + o;
                    kind[k] = (!TAILPIECE || c < cpr) ? 1 : 2;
                    if (kind[k] == 1) v[k] = *reinterpret_cast<const P *>(sp[k]);
                }
            }
            idx += GATHER_THREADS;
            w += dq;
            c += dr;
            if (c >= cpt) { c -= cpt; ++w; }
        }
#pragma unroll
        for (int k = 0; k < CHUNKS_IN_FLIGHT; ++k) {
            if (kind[k] == 1) __builtin_nontemporal_store(v[k], reinterpret_cast<P *>(dp[k]));
            else if (TAILPIECE && kind[k] == 2) copy_tail<VEC, A>(sp[k], dp[k], tail);
        }
    }
}

static int common_alignment(const RowSources &s, const uint8_t *out, uint64_t out_stride)
{
    uint64_t bits = (uint64_t)(uintptr_t)s.local_rows | s.local_stride | (uint64_t)(uintptr_t)s.cache_rows | s.cache_stride |
                    (uint64_t)(uintptr_t)s.remote_rows | s.remote_stride | (uint64_t)(uintptr_t)out | out_stride;
    if ((bits & 15) == 0) return 16;
    if ((bits & 7) == 0) return 8;
    if ((bits & 3) == 0) return 4;
    return 1;
}

rg_status launch_gather(const int64_t *entries, int64_t n_rows, const int32_t *list, int64_t n_list, int mode, const RowSources &src,
                        uint32_t row_bytes, uint8_t *out, uint64_t out_stride, hipStream_t st, int group)
{
    const int64_t n_work = list ? n_list : n_rows;
    if (n_work <= 0) return RG_OK;
    int align = common_alignment(src, out, out_stride);
    const int vec = align >= 4 ? 16 : 1;                        // dword-aligned rows take 16-byte vectors, anything else goes byte by byte
    const uint32_t tail = row_bytes % (uint32_t)vec;
    // A row that ends between vectors: if its width is a multiple of 4 and at least one vector, the last piece is the
    // vector ending at the row's end, at the alignment the width leaves; otherwise the last piece goes in parts.
    const bool overlap_last = vec == 16 && tail != 0 && row_bytes >= 16 && row_bytes % 4 == 0;
    const bool tailpiece = tail != 0 && !overlap_last;
    if (overlap_last) align = std::min(align, (row_bytes % 8 == 0) ? 8 : 4);
    const uint64_t cpt = row_bytes / (uint32_t)vec + (tail ? 1 : 0);
    int dev = 0, n_cu = 256;
    RG_HIP(hipGetDevice(&dev));
    RG_HIP(hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev));
    // pieces per thread and round: as many as stay in flight, fewer when that would leave compute units without a workgroup
    const uint64_t total = (uint64_t)n_work * cpt;
    const uint64_t want_blocks = (uint64_t)n_cu * 8;
    int chunks = CHUNKS_IN_FLIGHT;
    while (chunks > 1 && (total + (uint64_t)GATHER_THREADS * chunks - 1) / ((uint64_t)GATHER_THREADS * chunks) < want_blocks) --chunks;
    const uint64_t per_block = (uint64_t)GATHER_THREADS * chunks;
    const uint64_t blocks = std::max<uint64_t>(1, std::min<uint64_t>((total + per_block - 1) / per_block, (uint64_t)n_cu * 32));
    ScopedTimer tm(group, st);
#define RG_GATHER_LAUNCH(V, AL)                                                                                                               \
    do {                                                                                                                                      \
        if (tailpiece)                                                                                                                        \
            hipLaunchKernelGGL((gather_rows_kernel<V, AL, true>), dim3((unsigned)blocks), dim3(GATHER_THREADS), 0, st, entries, n_rows, list,   \
                               n_list, mode, src, row_bytes, out, out_stride, chunks);                                                        \
        else                                                                                                                                  \
            hipLaunchKernelGGL((gather_rows_kernel<V, AL, false>), dim3((unsigned)blocks), dim3(GATHER_THREADS), 0, st, entries, n_rows, list,  \
                               n_list, mode, src, row_bytes, out, out_stride, chunks);                                                        \
    } while (0)
    switch (align) {
    case 16: RG_GATHER_LAUNCH(16, 16); break;
    case 8:  RG_GATHER_LAUNCH(16, 8); break;
    case 4:  RG_GATHER_LAUNCH(16, 4); break;
    default: RG_GATHER_LAUNCH(1, 1); break;
    }
#undef RG_GATHER_LAUNCH
    RG_HIP(hipGetLastError());
    return RG_OK;
}

// True when p is device memory (then "remote" rows are plain HBM reads and need no side stream).
bool is_device_memory(const void *p)
{
    if (!p) return false;
    hipPointerAttribute_t attr;
    if (hipPointerGetAttributes(&attr, p) != hipSuccess) { (void)hipGetLastError(); return false; }
    return attr.type == hipMemoryTypeDevice;
}

// Routing of a single batch computed on the spot (no cache, or a schedule the cache has no plan for).
__global__ void route_batch_kernel(const int32_t *__restrict__ ids, int64_t n, const uint8_t *__restrict__ is_local, const int32_t *__restrict__ row_of,
                                   const SlotRec *__restrict__ slot_pairs /* see slot_lookup; NULL: no cache */, int64_t *__restrict__ entry, unsigned long long *__restrict__ counts /* local, hit, miss */)
{
    const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t tag = -1;
    if (j < n) {
        const int32_t v = ids[j];
        int64_t row;
        if (is_local[v]) { tag = TAG_LOCAL; row = row_of[v]; }
        else {
            const int32_t slot = slot_pairs ? slot_lookup(slot_pairs, (uint32_t)v) : -1;
            if (slot >= 0) { tag = TAG_CACHE; row = slot; }
            else { tag = TAG_REMOTE; row = row_of[v]; }
        }
        entry[j] = make_entry(tag, row);
    }
    const unsigned long long ml = __ballot(tag == TAG_LOCAL), mh = __ballot(tag == TAG_CACHE), mm = __ballot(tag == TAG_REMOTE);
    if ((threadIdx.x & 63) == 0) {
        if (ml) atomicAdd(&counts[0], (unsigned long long)__popcll(ml));
        if (mh) atomicAdd(&counts[1], (unsigned long long)__popcll(mh));
        if (mm) atomicAdd(&counts[2], (unsigned long long)__popcll(mm));
    }
}

// ---------------------------------------------------------------- the entry point that allocates nothing
// Its scratch -- the three counters and one routing entry per row of the batch -- lives in the library's image: one
// copy per GPU, at an address of that GPU's own, which the host asks for once per device.  The array's name is only a
// stand-in on the host; kernels and copies get the pointer kept here.
constexpr uint64_t NOALLOC_HEAD_BYTES = 256;                       // the counters, in front of the entries
static __device__ __align__(256) unsigned char scratch[NOALLOC_HEAD_BYTES + RG_NOALLOC_MAX_ROWS * sizeof(int64_t)];

constexpr int MAX_DEVICES = 64;
static std::mutex g_scratch_mu;
static void *g_scratch_ptr[MAX_DEVICES];                           // per device; NULL until asked for

// The current device's copy of `scratch`.
static rg_status scratch_of_current_device(unsigned char **out)
{
    int dev = 0;
    RG_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= MAX_DEVICES) { set_error("rg_gather_batch_noalloc: device %d beyond the %d this build keeps scratch for", dev, MAX_DEVICES); return RG_ERANGE; }
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        RG_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) { set_error("rg_gather_batch_noalloc: no address for the scratch array on device %d", dev); return RG_EHIP; }
        g_scratch_ptr[dev] = p;
    }
    *out = static_cast<unsigned char *>(g_scratch_ptr[dev]);
    return RG_OK;
}

// (a fill kernel, not hipMemsetAsync: the call may be recorded into a graph)
__global__ void clear_counts_kernel(unsigned long long *__restrict__ counts)
{
    if (threadIdx.x < 3) counts[threadIdx.x] = 0ull;
}

}  // namespace rg

using namespace rg;

extern "C" rg_status rg_gather_batch_noalloc(const rg_schedule *s, const rg_cache *c, const rg_features *f, uint32_t batch, void *out,
                                             uint64_t out_stride, uint64_t out_capacity_rows, void *stream, rg_gather_stats *stats)
{
    if (!s || !f) { set_error("rg_gather_batch_noalloc: null schedule or features"); return RG_EINVAL; }
    if (batch >= s->n_batches) { set_error("rg_gather_batch_noalloc: batch %u >= n_batches = %u", batch, s->n_batches); return RG_ERANGE; }
    if (f->row_bytes == 0 || out_stride < f->row_bytes || f->local_stride < f->row_bytes || f->remote_stride < f->row_bytes) {
        set_error("rg_gather_batch_noalloc: row_bytes = %u with strides out %llu local %llu remote %llu", f->row_bytes,
                  (unsigned long long)out_stride, (unsigned long long)f->local_stride, (unsigned long long)f->remote_stride);
        return RG_EINVAL;
    }
    if (c && (c->n_nodes != s->n_nodes || c->row_bytes != f->row_bytes)) { set_error("rg_gather_batch_noalloc: cache does not match schedule / features"); return RG_EINVAL; }
    const HopData &h = s->hop[s->L];
    const int64_t off = h.off_host[batch];
    const int64_t m = h.off_host[batch + 1] - off;
    if ((uint64_t)m > RG_NOALLOC_MAX_ROWS) {
        set_error("rg_gather_batch_noalloc: batch %u has %lld rows, the built-in scratch holds RG_NOALLOC_MAX_ROWS = %llu", batch, (long long)m,
                  (unsigned long long)RG_NOALLOC_MAX_ROWS);
        return RG_ERANGE;
    }
    if ((uint64_t)m > out_capacity_rows) {
        set_error("rg_gather_batch_noalloc: batch %u has %lld rows, output holds %llu", batch, (long long)m, (unsigned long long)out_capacity_rows);
        return RG_ERANGE;
    }
    if (m > 0 && !out) { set_error("rg_gather_batch_noalloc: null output"); return RG_EINVAL; }
    unsigned char *base = nullptr;
    RG_TRY(scratch_of_current_device(&base));
    unsigned long long *counts = reinterpret_cast<unsigned long long *>(base);
    int64_t *entry = reinterpret_cast<int64_t *>(base + NOALLOC_HEAD_BYTES);
    hipStream_t st = as_stream(stream);
    RowSources src{(const uint8_t *)f->local_rows, f->local_stride, c ? (const uint8_t *)c->rows : (const uint8_t *)f->local_rows,
                   c ? c->stride : f->local_stride, (const uint8_t *)f->remote_rows, f->remote_stride};
    hipLaunchKernelGGL(clear_counts_kernel, dim3(1), dim3(64), 0, st, counts);
    if (m > 0) {
        hipLaunchKernelGGL(route_batch_kernel, dim3((unsigned)((m + 255) / 256)), dim3(256), 0, st, h.ids + off, m, f->is_local, f->row_of,
                           c ? c->slot_pairs : nullptr, entry, counts);
        RG_HIP(hipGetLastError());
        RG_TRY(launch_gather(entry, m, nullptr, 0, 1, src, f->row_bytes, (uint8_t *)out, out_stride, st, -1));      // (group -1: no event timers, they are created on demand)
    }
    RG_HIP(hipGetLastError());
    if (stats) {
        unsigned long long hc[3] = {0, 0, 0};
        RG_HIP(hipMemcpyAsync(hc, counts, sizeof(hc), hipMemcpyDeviceToHost, st));
        RG_HIP(hipStreamSynchronize(st));
        stats->n_rows = (uint64_t)m; stats->n_local = hc[0]; stats->n_hit = hc[1]; stats->n_miss = hc[2];
    }
    return RG_OK;
}

extern "C" rg_status rg_gather_batch(const rg_schedule *s, const rg_cache *c, const rg_features *f, uint32_t batch, void *out,
                                     uint64_t out_stride, uint64_t out_capacity_rows, void *stream, void *side_stream,
                                     rg_gather_stats *stats)
{
    if (!s || !f) { set_error("rg_gather_batch: null schedule or features"); return RG_EINVAL; }
    if (batch >= s->n_batches) { set_error("rg_gather_batch: batch %u >= n_batches = %u", batch, s->n_batches); return RG_ERANGE; }
    if (f->row_bytes == 0 || out_stride < f->row_bytes || f->local_stride < f->row_bytes || f->remote_stride < f->row_bytes) {
        set_error("rg_gather_batch: row_bytes = %u with strides out %llu local %llu remote %llu", f->row_bytes,
                  (unsigned long long)out_stride, (unsigned long long)f->local_stride, (unsigned long long)f->remote_stride);
        return RG_EINVAL;
    }
    if (c && (c->n_nodes != s->n_nodes || c->row_bytes != f->row_bytes)) { set_error("rg_gather_batch: cache does not match schedule / features"); return RG_EINVAL; }
    const HopData &h = s->hop[s->L];
    const int64_t off = h.off_host[batch];
    const int64_t m = h.off_host[batch + 1] - off;
    if ((uint64_t)m > out_capacity_rows) {
        set_error("rg_gather_batch: batch %u has %lld rows, output holds %llu", batch, (long long)m, (unsigned long long)out_capacity_rows);
        return RG_ERANGE;
    }
    if (m > 0 && !out) { set_error("rg_gather_batch: null output"); return RG_EINVAL; }
    hipStream_t st = as_stream(stream);
    hipStream_t side = side_stream ? as_stream(side_stream) : st;
    RowSources src{(const uint8_t *)f->local_rows, f->local_stride, c ? (const uint8_t *)c->rows : (const uint8_t *)f->local_rows,
                   c ? c->stride : f->local_stride, (const uint8_t *)f->remote_rows, f->remote_stride};

    const Plan *plan = nullptr;
    if (c)
        for (const Plan &p : c->plans)
            if (p.schedule_uid == s->uid) { plan = &p; break; }

    if (plan) {
        const int64_t n_miss = plan->miss_off[batch + 1] - plan->miss_off[batch];
        const int64_t *entries = plan->entry + off;
        const bool remote_in_hbm = n_miss > 0 && (f->remote_rows == c->remote_rows_seen ? c->remote_is_device : is_device_memory(f->remote_rows));
        if (n_miss == 0 || remote_in_hbm) {
            // every source is HBM: one launch copies the whole block
            RG_TRY(launch_gather(entries, m, nullptr, 0, 1, src, f->row_bytes, (uint8_t *)out, out_stride, st, KG_GATHER));
        } else if (side != st) {
            RG_HIP(hipEventRecord(c->ev_fork, st));            // earlier work on `stream` may still use `out`
            RG_HIP(hipStreamWaitEvent(side, c->ev_fork, 0));
            RG_TRY(launch_gather(entries, m, plan->miss_rows + plan->miss_off[batch], n_miss, 1, src, f->row_bytes, (uint8_t *)out, out_stride, side, KG_MISS));
            RG_HIP(hipEventRecord(c->ev_join, side));
            RG_TRY(launch_gather(entries, m, nullptr, 0, 0, src, f->row_bytes, (uint8_t *)out, out_stride, st, KG_GATHER));
            RG_HIP(hipStreamWaitEvent(st, c->ev_join, 0));
        } else {
            RG_TRY(launch_gather(entries, m, nullptr, 0, 0, src, f->row_bytes, (uint8_t *)out, out_stride, st, KG_GATHER));
            RG_TRY(launch_gather(entries, m, plan->miss_rows + plan->miss_off[batch], n_miss, 1, src, f->row_bytes, (uint8_t *)out, out_stride, st, KG_MISS));
        }
        s->uses.note(st);                                      // the launches above read the schedule's and the cache's arrays after this call returns
        c->uses.note(st);
        if (stats) *stats = plan->stats[batch];
        return RG_OK;
    }

    // No prepared plan: classify this batch now, copy every row on `stream`, wait for the counts.
    Arena tmp(s->arena.allocator(), st);     // scratch from the allocator the schedule was built with
    int64_t *entry = nullptr;
    unsigned long long *counts = nullptr;
    RG_TRY(tmp.dev_n<int64_t>((uint64_t)m, &entry));
    RG_TRY(tmp.dev_n<unsigned long long>(3, &counts));
    RG_HIP(hipMemsetAsync(counts, 0, 3 * sizeof(unsigned long long), st));
    if (m > 0) {
        {
            ScopedTimer tm(KG_PLAN, st);
            hipLaunchKernelGGL(route_batch_kernel, dim3((unsigned)((m + 255) / 256)), dim3(256), 0, st, h.ids + off, m, f->is_local, f->row_of,
                               c ? c->slot_pairs : nullptr, entry, counts);
        }
        RG_HIP(hipGetLastError());
        RG_TRY(launch_gather(entry, m, nullptr, 0, 1, src, f->row_bytes, (uint8_t *)out, out_stride, st, KG_GATHER));
    }
    unsigned long long hc[3] = {0, 0, 0};
    RG_HIP(hipMemcpyAsync(hc, counts, sizeof(hc), hipMemcpyDeviceToHost, st));
    RG_HIP(hipStreamSynchronize(st));
    tmp.drained();
    if (stats) { stats->n_rows = (uint64_t)m; stats->n_local = hc[0]; stats->n_hit = hc[1]; stats->n_miss = hc[2]; }
    return RG_OK;
}

// Blocks of consecutive batches, back to back in one output buffer.  A schedule keeps the frontiers of its batches
// concatenated, and so does a plan its routing entries: a range of batches is a range of rows, and one launch
// copies it (fewer, larger launches: the ramp and tail of a launch are paid once per range, not once per batch).
extern "C" rg_status rg_gather_batches(const rg_schedule *s, const rg_cache *c, const rg_features *f, uint32_t first_batch,
                                       uint32_t n_batches, void *out, uint64_t out_stride, uint64_t out_capacity_rows, void *stream,
                                       void *side_stream, rg_gather_stats *stats)
{
    if (!s || !f) { set_error("rg_gather_batches: null schedule or features"); return RG_EINVAL; }
    if ((uint64_t)first_batch + n_batches > s->n_batches) {
        set_error("rg_gather_batches: batches [%u, %u + %u) beyond n_batches = %u", first_batch, first_batch, n_batches, s->n_batches);
        return RG_ERANGE;
    }
    if (n_batches == 0) return RG_OK;
    const HopData &h = s->hop[s->L];
    const int64_t off0 = h.off_host[first_batch];
    const int64_t m = h.off_host[first_batch + n_batches] - off0;
    if ((uint64_t)m > out_capacity_rows) {
        set_error("rg_gather_batches: %u batches from %u have %lld rows, output holds %llu", n_batches, first_batch, (long long)m,
                  (unsigned long long)out_capacity_rows);
        return RG_ERANGE;
    }
    const Plan *plan = nullptr;
    if (c)
        for (const Plan &p : c->plans)
            if (p.schedule_uid == s->uid) { plan = &p; break; }
    if (!plan || n_batches == 1) {
        // no prepared routing for this schedule: batch by batch (each call classifies on the fly and waits for its counts)
        for (uint32_t k = 0; k < n_batches; ++k) {
            const uint32_t b = first_batch + k;
            const int64_t at = h.off_host[b] - off0;
            RG_TRY(rg_gather_batch(s, c, f, b, (uint8_t *)out + (uint64_t)at * out_stride, out_stride, out_capacity_rows - (uint64_t)at, stream,
                                   side_stream, stats ? stats + k : nullptr));
        }
        return RG_OK;
    }
    if (f->row_bytes == 0 || out_stride < f->row_bytes || f->local_stride < f->row_bytes || f->remote_stride < f->row_bytes) {
        set_error("rg_gather_batches: row_bytes = %u with strides out %llu local %llu remote %llu", f->row_bytes,
                  (unsigned long long)out_stride, (unsigned long long)f->local_stride, (unsigned long long)f->remote_stride);
        return RG_EINVAL;
    }
    if (c->n_nodes != s->n_nodes || c->row_bytes != f->row_bytes) { set_error("rg_gather_batches: cache does not match schedule / features"); return RG_EINVAL; }
    if (m > 0 && !out) { set_error("rg_gather_batches: null output"); return RG_EINVAL; }
    hipStream_t st = as_stream(stream);
    hipStream_t side = side_stream ? as_stream(side_stream) : st;
    RowSources src{(const uint8_t *)f->local_rows, f->local_stride, (const uint8_t *)c->rows, c->stride, (const uint8_t *)f->remote_rows, f->remote_stride};
    const int64_t n_miss = plan->miss_off[first_batch + n_batches] - plan->miss_off[first_batch];
    const int64_t *entries = plan->entry + off0;
    const bool remote_in_hbm = n_miss > 0 && (f->remote_rows == c->remote_rows_seen ? c->remote_is_device : is_device_memory(f->remote_rows));
    if (n_miss == 0 || remote_in_hbm) {
        RG_TRY(launch_gather(entries, m, nullptr, 0, 1, src, f->row_bytes, (uint8_t *)out, out_stride, st, KG_GATHER));
    } else {
        // rows with HBM sources in one launch; every batch's miss list (row indices within its own block) in a launch of its own
        if (side != st) {
            RG_HIP(hipEventRecord(c->ev_fork, st));
            RG_HIP(hipStreamWaitEvent(side, c->ev_fork, 0));
        }
        RG_TRY(launch_gather(entries, m, nullptr, 0, 0, src, f->row_bytes, (uint8_t *)out, out_stride, st, KG_GATHER));
        for (uint32_t k = 0; k < n_batches; ++k) {
            const uint32_t b = first_batch + k;
            const int64_t nm = plan->miss_off[b + 1] - plan->miss_off[b];
            if (nm == 0) continue;
            const int64_t at = h.off_host[b] - off0, mb = h.off_host[b + 1] - h.off_host[b];
            RG_TRY(launch_gather(plan->entry + h.off_host[b], mb, plan->miss_rows + plan->miss_off[b], nm, 1, src, f->row_bytes,
                                 (uint8_t *)out + (uint64_t)at * out_stride, out_stride, side, KG_MISS));
        }
        if (side != st) {
            RG_HIP(hipEventRecord(c->ev_join, side));
            RG_HIP(hipStreamWaitEvent(st, c->ev_join, 0));
        }
    }
    s->uses.note(st);
    c->uses.note(st);
    if (stats)
        for (uint32_t k = 0; k < n_batches; ++k) stats[k] = plan->stats[first_batch + k];
    return RG_OK;
}

// The batch's counts alone: a9 without the copy (Alg. 1 inner loop, rpc_e += |M_i^e|).
extern "C" rg_status rg_classify_batch(const rg_schedule *s, const rg_cache *c, const rg_features *f, uint32_t batch, void *stream,
                                       rg_gather_stats *stats)
{
    if (!s || !f || !stats) { set_error("rg_classify_batch: null argument"); return RG_EINVAL; }
    if (batch >= s->n_batches) { set_error("rg_classify_batch: batch %u >= n_batches = %u", batch, s->n_batches); return RG_ERANGE; }
    if (c && c->n_nodes != s->n_nodes) { set_error("rg_classify_batch: cache does not match the schedule"); return RG_EINVAL; }
    if (c)
        for (const Plan &p : c->plans)
            if (p.schedule_uid == s->uid) { *stats = p.stats[batch]; return RG_OK; }
    const HopData &h = s->hop[s->L];
    const int64_t off = h.off_host[batch], m = h.off_host[batch + 1] - off;
    hipStream_t st = as_stream(stream);
    Arena tmp(s->arena.allocator(), st);     // scratch from the allocator the schedule was built with
    int64_t *entry = nullptr;
    unsigned long long *counts = nullptr;
    RG_TRY(tmp.dev_n<int64_t>((uint64_t)m, &entry));
    RG_TRY(tmp.dev_n<unsigned long long>(3, &counts));
    RG_HIP(hipMemsetAsync(counts, 0, 3 * sizeof(unsigned long long), st));
    if (m > 0) {
        ScopedTimer tm(KG_PLAN, st);
        hipLaunchKernelGGL(route_batch_kernel, dim3((unsigned)((m + 255) / 256)), dim3(256), 0, st, h.ids + off, m, f->is_local, f->row_of,
                           c ? c->slot_pairs : nullptr, entry, counts);
    }
    unsigned long long hc[3] = {0, 0, 0};
    hipError_t e1 = hipGetLastError();
    hipError_t e2 = hipMemcpyAsync(hc, counts, sizeof(hc), hipMemcpyDeviceToHost, st);
    hipError_t e3 = hipStreamSynchronize(st);                    // also before `tmp` is released
    if (e3 == hipSuccess) tmp.drained();
    if (e1 != hipSuccess || e2 != hipSuccess || e3 != hipSuccess) { set_error("rg_classify_batch: HIP call failed"); return RG_EHIP; }
    stats->n_rows = (uint64_t)m; stats->n_local = hc[0]; stats->n_hit = hc[1]; stats->n_miss = hc[2];
    return RG_OK;
}
