// rg_build_cache: access-frequency tally, TopHot selection, VectorPull into the
// device table, and the per-batch routing plans (Alg. 1 steps 2-4).
#include "rg_internal.h"

#include <algorithm>

namespace rg {

thread_local std::atomic<uint64_t> *tls_table_bytes_sink = nullptr;

// ---------------------------------------------------------------- a6: freq(v)
// Every batch's input set is duplicate free, so each listed ID adds one.
// The counters are uint32_t, or -- when no frequency can exceed 255 (at most 255 batches over the epochs given) --
// uint8_t, four to a word: an add of 1 << 8 * (id & 3) to the word can then never carry into the next counter.  A
// tally of 10^8 nodes is a quarter of the bytes to clear and to read in every later pass, and small enough for
// its scattered adds to stay in the last-level cache.
template <typename F>
__global__ void tally_kernel(const int32_t *__restrict__ ids, int64_t n, F *__restrict__ freq)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        const uint32_t v = (uint32_t)ids[i];
        if (sizeof(F) == 1) atomicAdd(reinterpret_cast<uint32_t *>(freq) + (v >> 2), 1u << (8 * (v & 3)));
        else atomicAdd(reinterpret_cast<uint32_t *>(freq) + v, 1u);
    }
}

// freq += the frequencies an epoch's schedule already holds (computed from its bitmaps when it was built)
template <typename F>
__global__ void add_epoch_freq_kernel(const uint32_t *__restrict__ epoch_freq, int64_t n, F *__restrict__ freq)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) freq[i] = (F)(freq[i] + epoch_freq[i]);
}

// The uint8_t tally as the uint32_t array the cache's view hands out (made when first asked for).
__global__ void widen_freq_kernel(const uint8_t *__restrict__ freq8, int64_t n, uint32_t *__restrict__ freq)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) freq[i] = freq8[i];
}

// ---------------------------------------------------------------- a7: TopHot
// Candidates: remote IDs with freq > 0.  The K-th largest frequency t is found
// by a most-significant-digit-first radix select over the candidates' freq
// values (8-bit digits, as many passes as max_freq needs; LDS-privatised digit
// histograms merged with atomics).  Selected: freq > t, plus the first r
// candidates with freq == t in ascending ID order (the tie-break), found by one
// prefix sum over the nodes that also yields the slots: cache_ids ascending.
struct SelectState {
    uint32_t prefix;        // digits of t decided so far (high bits), already shifted into place
    uint32_t prefix_mask;   // which bits of prefix are decided
    uint64_t want;          // how many still to take among candidates matching the prefix
    uint64_t n_candidates;  // set by the first pass
    uint32_t take_all;      // 1: K >= #candidates, every candidate is selected
    uint32_t t;             // final threshold
    uint64_t r;             // how many of the freq == t candidates to take
    uint64_t k_eff;
};

constexpr int TOPK_THREADS = 256;
constexpr int DIGIT_BITS = 8;
constexpr int DIGIT_BINS = 1 << DIGIT_BITS;
constexpr int BIN_COPIES = 64;            // the digit histogram is kept in this many copies, summed when a digit is chosen

// QUADS: a lane takes four consecutive nodes per round (one 16-byte and one 4-byte load; is_local must be 4-byte
// aligned), the few nodes after the last whole quad one by one.
template <bool QUADS>
__global__ void __launch_bounds__(TOPK_THREADS) digit_histogram_kernel(const uint32_t *__restrict__ freq, const uint8_t *__restrict__ is_local, int64_t n,
                                                                       const SelectState *__restrict__ stp, int shift,
                                                                       unsigned long long *__restrict__ bins)
{
    __shared__ unsigned int h[DIGIT_BINS];
    for (int k = threadIdx.x; k < DIGIT_BINS; k += TOPK_THREADS) h[k] = 0;
    __syncthreads();
    const uint32_t prefix = stp->prefix, pmask = stp->prefix_mask;
    if (stp->take_all) return;
    auto count = [&](uint32_t fv, uint32_t local) {
        if (fv != 0 && !local && (fv & pmask) == prefix) atomicAdd(&h[(fv >> shift) & (DIGIT_BINS - 1)], 1u);
    };
    int64_t done = 0;
    if (QUADS) {
        auto count4 = [&](const uint4 fv, uint32_t loc) {
            if ((fv.x | fv.y | fv.z | fv.w) == 0u) return;                     // most nodes are never listed
            count(fv.x, loc & 0xFFu); count(fv.y, (loc >> 8) & 0xFFu); count(fv.z, (loc >> 16) & 0xFFu); count(fv.w, loc >> 24);
        };
        // a workgroup reads one contiguous span of quads, four independent loads of each kind in flight per lane
        const int64_t n_quads = n >> 2;
        const int64_t span = (n_quads + gridDim.x - 1) / gridDim.x;
        const int64_t q_end = min(n_quads, (int64_t)(blockIdx.x + 1) * span);
        int64_t q = (int64_t)blockIdx.x * span + threadIdx.x;
        for (; q + 3 * TOPK_THREADS < q_end; q += 4 * TOPK_THREADS) {
            uint4 fv[4]; uint32_t loc[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) fv[u] = reinterpret_cast<const uint4 *>(freq)[q + u * TOPK_THREADS];
#pragma unroll
            for (int u = 0; u < 4; ++u) loc[u] = reinterpret_cast<const uint32_t *>(is_local)[q + u * TOPK_THREADS];
#pragma unroll
            for (int u = 0; u < 4; ++u) count4(fv[u], loc[u]);
        }
        for (; q < q_end; q += TOPK_THREADS) count4(reinterpret_cast<const uint4 *>(freq)[q], reinterpret_cast<const uint32_t *>(is_local)[q]);
        done = n_quads << 2;
    }
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int64_t t0 = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (int64_t v = done + t0; v < n; v += stride) count(freq[v], is_local[v]);
    __syncthreads();
    // workgroups spread their adds over BIN_COPIES copies of the bins: few digits are in use, and thousands of adds
    // to the same few addresses would queue up behind each other
    unsigned long long *mine = bins + (size_t)(blockIdx.x % BIN_COPIES) * DIGIT_BINS;
    for (int k = threadIdx.x; k < DIGIT_BINS; k += TOPK_THREADS)
        if (h[k]) atomicAdd(&mine[k], (unsigned long long)h[k]);
}

// The same for the uint8_t tally: one digit, so no prefix to match.  WIDE (is_local 16-byte aligned; the tally always
// is): a lane takes sixteen consecutive nodes per round, one 16-byte load of each array, and visits only the
// bytes that are candidates (non-zero count, not local).
__device__ __forceinline__ uint32_t nonzero_bytes(uint32_t w) { return (w | ((w & 0x7F7F7F7Fu) + 0x7F7F7F7Fu)) & 0x80808080u; }   // bit 7 of every non-zero byte

template <bool WIDE>
__global__ void __launch_bounds__(TOPK_THREADS) digit_histogram8_kernel(const uint8_t *__restrict__ freq, const uint8_t *__restrict__ is_local, int64_t n,
                                                                        const SelectState *__restrict__ stp, unsigned long long *__restrict__ bins)
{
    __shared__ unsigned int h[DIGIT_BINS];
    for (int k = threadIdx.x; k < DIGIT_BINS; k += TOPK_THREADS) h[k] = 0;
    __syncthreads();
    if (stp->take_all) return;
    int64_t done = 0;
    if (WIDE) {
        auto count_word = [&](uint32_t fw, uint32_t lw) {
            uint32_t cand = nonzero_bytes(fw) & ~nonzero_bytes(lw);
            while (cand) {
                const int top = __ffs((int)cand) - 1;              // bit 7 of the candidate's byte
                cand &= cand - 1;
                atomicAdd(&h[(fw >> (top - 7)) & 0xFFu], 1u);
            }
        };
        auto count16 = [&](const uint4 fv, const uint4 lv) {
            if ((fv.x | fv.y | fv.z | fv.w) == 0u) return;
            count_word(fv.x, lv.x); count_word(fv.y, lv.y); count_word(fv.z, lv.z); count_word(fv.w, lv.w);
        };
        const int64_t n16 = n >> 4;
        const int64_t span = (n16 + gridDim.x - 1) / gridDim.x;
        const int64_t q_end = min(n16, (int64_t)(blockIdx.x + 1) * span);
        int64_t q = (int64_t)blockIdx.x * span + threadIdx.x;
        for (; q + TOPK_THREADS < q_end; q += 2 * TOPK_THREADS) {
            const uint4 f0 = reinterpret_cast<const uint4 *>(freq)[q], f1 = reinterpret_cast<const uint4 *>(freq)[q + TOPK_THREADS];
            const uint4 l0 = reinterpret_cast<const uint4 *>(is_local)[q], l1 = reinterpret_cast<const uint4 *>(is_local)[q + TOPK_THREADS];
            count16(f0, l0); count16(f1, l1);
        }
        for (; q < q_end; q += TOPK_THREADS) count16(reinterpret_cast<const uint4 *>(freq)[q], reinterpret_cast<const uint4 *>(is_local)[q]);
        done = n16 << 4;
    }
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t v = done + (int64_t)blockIdx.x * blockDim.x + threadIdx.x; v < n; v += stride) {
        const uint32_t fv = freq[v];
        if (fv != 0 && !is_local[v]) atomicAdd(&h[fv], 1u);
    }
    __syncthreads();
    unsigned long long *mine = bins + (size_t)(blockIdx.x % BIN_COPIES) * DIGIT_BINS;
    for (int k = threadIdx.x; k < DIGIT_BINS; k += TOPK_THREADS)
        if (h[k]) atomicAdd(&mine[k], (unsigned long long)h[k]);
}

// One workgroup of DIGIT_BINS threads: sum the copies of each bin (and clear them for the next pass), then one thread
// walks the bins from the top until `want` is covered.
__global__ void __launch_bounds__(DIGIT_BINS) choose_digit_kernel(SelectState *__restrict__ stp, unsigned long long *__restrict__ bins_copies, int shift,
                                                                  int first_pass, uint64_t K)
{
    __shared__ unsigned long long bins[DIGIT_BINS];
    {
        unsigned long long sum = 0;
        for (int cpy = 0; cpy < BIN_COPIES; ++cpy) {
            sum += bins_copies[(size_t)cpy * DIGIT_BINS + threadIdx.x];
            bins_copies[(size_t)cpy * DIGIT_BINS + threadIdx.x] = 0;
        }
        bins[threadIdx.x] = sum;
    }
    __syncthreads();
    if (threadIdx.x != 0) return;
    SelectState st = *stp;
    if (first_pass) {
        uint64_t tot = 0;
        for (int k = 0; k < DIGIT_BINS; ++k) tot += bins[k];
        st.n_candidates = tot;
        st.want = K;
        if (K >= tot) { st.take_all = 1; st.t = 0; st.r = 0; st.k_eff = tot; }
        else st.k_eff = K;
    }
    if (!st.take_all) {
        uint64_t above = 0;
        int d = DIGIT_BINS - 1;
        for (; d > 0; --d) {
            if (above + bins[d] >= st.want) break;
            above += bins[d];
        }
        st.want -= above;                         // still to take inside digit d
        st.prefix |= (uint32_t)d << shift;
        st.prefix_mask |= (uint32_t)(DIGIT_BINS - 1) << shift;
        if (shift == 0) { st.t = st.prefix; st.r = st.want; }
    }
    *stp = st;
}

// Packed counters per node: high 32 bits = selected outright (freq > t), low 32 bits = tied (freq == t).
__device__ __forceinline__ uint64_t classify_node(uint32_t fv, uint8_t local, const SelectState &st)
{
    if (fv == 0 || local) return 0;
    if (st.take_all || fv > st.t) return (uint64_t)1 << 32;
    return fv == st.t ? 1ull : 0ull;
}

constexpr int SEL_PER_THREAD = 8;         // runs of eight consecutive nodes: a quarter of a slot-map record per thread (sixteen measured 8 % slower over the byte tally)
constexpr int SEL_TILE = TOPK_THREADS * SEL_PER_THREAD;

// The eight consecutive nodes of a thread, classified.  ALIGNED8 (is_local 8-byte aligned; freq always is, and a
// thread's first node is a multiple of eight): two 16-byte loads and one 8-byte load when all eight exist.
template <bool ALIGNED8>
__device__ __forceinline__ void classify_eight(const uint32_t *__restrict__ freq, const uint8_t *__restrict__ is_local, int64_t first, int64_t n,
                                               const SelectState &st, uint64_t *c /* [8] */)
{
    if (ALIGNED8 && first + 8 <= n) {
        const uint4 a = *reinterpret_cast<const uint4 *>(freq + first), b = *reinterpret_cast<const uint4 *>(freq + first + 4);
        const uint64_t loc = *reinterpret_cast<const uint64_t *>(is_local + first);
        const uint32_t fv[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
#pragma unroll
        for (int k = 0; k < 8; ++k) c[k] = classify_node(fv[k], (uint8_t)(loc >> (8 * k)), st);
        return;
    }
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        const int64_t v = first + k;
        c[k] = v < n ? classify_node(freq[v], is_local[v], st) : 0;
    }
}
// The same over the uint8_t tally: one 8-byte load of each array.
template <bool ALIGNED8>
__device__ __forceinline__ void classify_eight(const uint8_t *__restrict__ freq, const uint8_t *__restrict__ is_local, int64_t first, int64_t n,
                                               const SelectState &st, uint64_t *c /* [8] */)
{
    if (ALIGNED8 && first + 8 <= n) {
        const uint64_t fw = *reinterpret_cast<const uint64_t *>(freq + first);
        if (fw == 0ull) {
#pragma unroll
            for (int k = 0; k < 8; ++k) c[k] = 0;
            return;
        }
        const uint64_t loc = *reinterpret_cast<const uint64_t *>(is_local + first);
#pragma unroll
        for (int k = 0; k < 8; ++k) c[k] = classify_node((uint32_t)(fw >> (8 * k)) & 0xFFu, (uint8_t)(loc >> (8 * k)), st);
        return;
    }
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        const int64_t v = first + k;
        c[k] = v < n ? classify_node(freq[v], is_local[v], st) : 0;
    }
}
// The SEL_PER_THREAD consecutive nodes of a thread.
template <bool ALIGNED8, typename F>
__device__ __forceinline__ void classify_mine(const F *__restrict__ freq, const uint8_t *__restrict__ is_local, int64_t first, int64_t n,
                                              const SelectState &st, uint64_t (&c)[SEL_PER_THREAD])
{
#pragma unroll
    for (int h = 0; h < SEL_PER_THREAD / 8; ++h) classify_eight<ALIGNED8>(freq, is_local, first + 8 * h, n, st, c + 8 * h);
}

__device__ __forceinline__ uint64_t block_exclusive_scan_u64(uint64_t x, uint64_t *total, uint64_t *lds)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint64_t incl = x;
    for (int d = 1; d < 64; d <<= 1) {
        uint64_t y = __shfl_up(incl, d, 64);
        if (lane >= d) incl += y;
    }
    if (lane == 63) lds[wave] = incl;
    __syncthreads();
    uint64_t base = 0, tot = 0;
    for (int w = 0; w < TOPK_THREADS / 64; ++w) {
        const uint64_t s = lds[w];
        if (w < wave) base += s;
        tot += s;
    }
    __syncthreads();
    *total = tot;
    return base + incl - x;
}

template <bool ALIGNED8, typename F>
__global__ void __launch_bounds__(TOPK_THREADS) select_block_totals(const F *__restrict__ freq, const uint8_t *__restrict__ is_local, int64_t n,
                                                                    const SelectState *__restrict__ stp, uint64_t *__restrict__ block_tot)
{
    __shared__ uint64_t lds[TOPK_THREADS / 64];
    const SelectState st = *stp;
    const int64_t first = (int64_t)blockIdx.x * SEL_TILE + (int64_t)threadIdx.x * SEL_PER_THREAD;
    uint64_t c[SEL_PER_THREAD];
    classify_mine<ALIGNED8, F>(freq, is_local, first, n, st, c);
    uint64_t s = 0;
#pragma unroll
    for (int k = 0; k < SEL_PER_THREAD; ++k) s += c[k];
    uint64_t tot;
    (void)block_exclusive_scan_u64(s, &tot, lds);
    if (threadIdx.x == 0) block_tot[blockIdx.x] = tot;
}

// The exclusive scan of the per-workgroup totals, in two levels: every workgroup scans its own SCAN_TILE totals in
// place and leaves their sum in tile_tot; one workgroup then scans tile_tot (select_scan_totals); the emit pass adds
// the two.  (10^8 nodes are 54,000 totals: one workgroup alone spends longer walking them than a pass over the nodes' flags takes.)
constexpr int SCAN_TILE = TOPK_THREADS * 8;
__global__ void __launch_bounds__(TOPK_THREADS) select_scan_tiles(uint64_t *__restrict__ block_tot, int64_t n_blocks, uint64_t *__restrict__ tile_tot)
{
    __shared__ uint64_t lds[TOPK_THREADS / 64];
    const int64_t i0 = (int64_t)blockIdx.x * SCAN_TILE + (int64_t)threadIdx.x * 8;
    uint64_t x[8], sum = 0;
#pragma unroll
    for (int k = 0; k < 8; ++k) { x[k] = i0 + k < n_blocks ? block_tot[i0 + k] : 0; sum += x[k]; }
    uint64_t tot;
    uint64_t run = block_exclusive_scan_u64(sum, &tot, lds);
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        if (i0 + k < n_blocks) block_tot[i0 + k] = run;
        run += x[k];
    }
    if (threadIdx.x == 0) tile_tot[blockIdx.x] = tot;
}

// One workgroup; a thread takes eight consecutive totals per round.
__global__ void __launch_bounds__(TOPK_THREADS) select_scan_totals(uint64_t *__restrict__ block_tot, int64_t n_blocks)
{
    __shared__ uint64_t lds[TOPK_THREADS / 64];
    uint64_t carry = 0;
    for (int64_t base = 0; base < n_blocks; base += (int64_t)TOPK_THREADS * 8) {
        const int64_t i0 = base + (int64_t)threadIdx.x * 8;
        uint64_t x[8], sum = 0;
#pragma unroll
        for (int k = 0; k < 8; ++k) { x[k] = i0 + k < n_blocks ? block_tot[i0 + k] : 0; sum += x[k]; }
        uint64_t tot;
        uint64_t run = carry + block_exclusive_scan_u64(sum, &tot, lds);
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            if (i0 + k < n_blocks) block_tot[i0 + k] = run;
            run += x[k];
        }
        carry += tot;
    }
}

template <bool ALIGNED8, typename F>
__global__ void __launch_bounds__(TOPK_THREADS) select_emit_kernel(const F *__restrict__ freq, const uint8_t *__restrict__ is_local, int64_t n,
                                                                   const SelectState *__restrict__ stp, const uint64_t *__restrict__ block_base,
                                                                   const uint64_t *__restrict__ tile_base, int32_t *__restrict__ cache_ids, SlotRec *__restrict__ slot_pairs,
                                                                   const int32_t *__restrict__ row_of, int64_t *__restrict__ fill_entries)
{
    // fill_entries[slot]: where VectorPull finds the row of the node in that slot (a8), written here while the node is at hand
    __shared__ uint64_t lds[TOPK_THREADS / 64];
    const SelectState st = *stp;
    const int64_t first = (int64_t)blockIdx.x * SEL_TILE + (int64_t)threadIdx.x * SEL_PER_THREAD;
    uint64_t c[SEL_PER_THREAD];
    classify_mine<ALIGNED8, F>(freq, is_local, first, n, st, c);
    uint64_t s = 0;
#pragma unroll
    for (int k = 0; k < SEL_PER_THREAD; ++k) s += c[k];
    uint64_t tot;
    uint64_t run = block_base[blockIdx.x] + tile_base[blockIdx.x / SCAN_TILE] + block_exclusive_scan_u64(s, &tot, lds);
    static_assert(SEL_PER_THREAD == 8, "four consecutive lanes make up one pair of the slot map");
    const uint64_t start = run;
    uint32_t mine = 0;                                      // which of this thread's eight nodes are selected
#pragma unroll
    for (int k = 0; k < SEL_PER_THREAD; ++k) {
        const int64_t v = first + k;
        const uint64_t gt_before = run >> 32, eq_before = run & 0xFFFFFFFFull;
        const bool sel = v < n && ((c[k] >> 32) != 0 || (c[k] == 1 && eq_before < st.r));
        if (sel) {
            const int64_t slot = (int64_t)(gt_before + (eq_before < st.r ? eq_before : st.r));
            cache_ids[slot] = (int32_t)v;
            fill_entries[slot] = make_entry(TAG_REMOTE, row_of[v]);
            mine |= 1u << k;
        }
        run += c[k];
    }
    // the slot map's record for 32 node IDs (see slot_lookup): bits from four lanes, the rank from the first of them
    uint32_t local8 = 0;                                    // which of this thread's eight nodes are local
    if (ALIGNED8 && first + SEL_PER_THREAD <= n) {
        const uint64_t loc = *reinterpret_cast<const uint64_t *>(is_local + first);
#pragma unroll
        for (int k = 0; k < SEL_PER_THREAD; ++k)
            if ((loc >> (8 * k)) & 0xFFull) local8 |= 1u << k;
    } else {
#pragma unroll
        for (int k = 0; k < SEL_PER_THREAD; ++k)
            if (first + k < n && is_local[first + k]) local8 |= 1u << k;
    }
    const int lane = threadIdx.x & 63;
    uint32_t word = mine << (8 * (lane & 3)), lword = local8 << (8 * (lane & 3));
    word |= __shfl_xor(word, 1, 64); lword |= __shfl_xor(lword, 1, 64);
    word |= __shfl_xor(word, 2, 64); lword |= __shfl_xor(lword, 2, 64);
    if ((lane & 3) == 0) {
        const uint64_t gt_before = start >> 32, eq_before = start & 0xFFFFFFFFull;
        slot_pairs[first >> 5] = make_uint4(word, (uint32_t)(gt_before + (eq_before < st.r ? eq_before : st.r)), lword, 0u);
    }
}

// The slot map as the int32_t[n_nodes] array the cache's view hands out (made when first asked for).
__global__ void widen_slots_kernel(const SlotRec *__restrict__ pairs, int64_t n, int32_t *__restrict__ slot_of)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; v < n; v += stride) slot_of[v] = slot_lookup(pairs, (uint32_t)v);
}

// ---------------------------------------------------------------- a5/a9: routing plan
__device__ __forceinline__ uint32_t batch_of_pos(const int64_t *__restrict__ off, uint32_t n_batches, int64_t i)
{
    uint32_t lo = 0, hi = n_batches;
    while (hi - lo > 1) {
        const uint32_t mid = (lo + hi) >> 1;
        if (off[mid] <= i) lo = mid; else hi = mid;
    }
    return lo;
}

// Where a request for v's feature row is served from: (tag << 62) | row.  One record of the slot map says whether v
// is local and whether (and where) it is cached; row_of is read for the others only.
struct RouteSources {
    const int32_t *row_of;
    const SlotRec *slot_pairs;       // see slot_lookup
};
__device__ __forceinline__ int64_t route_of(const RouteSources &r, int64_t v)
{
    const SlotRec p = r.slot_pairs[v >> 5];
    const uint32_t bit = 1u << (v & 31);
    if (p.z & bit) return make_entry(TAG_LOCAL, r.row_of[v]);
    if (p.x & bit) return make_entry(TAG_CACHE, (int64_t)(p.y + __popc(p.x & (bit - 1))));
    return make_entry(TAG_REMOTE, r.row_of[v]);
}

// entry[j] = route_of(ids[j]) for every listed input node, which of them are misses (one bit each, in position order:
// a wave's ballot is the 64-bit word of its 64 consecutive positions), the misses of every tile of PLAN_TILE
// positions, and per-batch counts of local rows and cache hits.  A block covers one tile and adds its counts once
// when it lies inside one batch (nearly always), else position by position.
constexpr int PLAN_THREADS = 256;
constexpr int PLAN_PER_THREAD = 4;
constexpr int PLAN_TILE = PLAN_THREADS * PLAN_PER_THREAD;
constexpr int PLAN_TILE_WORDS = PLAN_TILE / 64;          // miss-bit words per tile

__global__ void __launch_bounds__(PLAN_THREADS) plan_kernel(const int32_t *__restrict__ ids, int64_t n, const int64_t *__restrict__ batch_off, uint32_t n_batches,
                                                            RouteSources rs,
                                                            int64_t *__restrict__ entry, unsigned long long *__restrict__ miss_bits /* [tiles * PLAN_TILE_WORDS] */,
                                                            int32_t *__restrict__ tile_miss /* [tiles] */,
                                                            unsigned long long *__restrict__ counts /* [n_batches][2]: local, hit */)
{
    __shared__ unsigned int red[3][PLAN_THREADS / 64];
    const int64_t tile0 = (int64_t)blockIdx.x * PLAN_TILE;
    const int64_t tile_last = (tile0 + PLAN_TILE <= n ? tile0 + PLAN_TILE : n) - 1;
    const uint32_t b_first = batch_of_pos(batch_off, n_batches, tile0);
    const bool one_batch = batch_off[b_first + 1] > tile_last;                 // block-uniform
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    unsigned int n_local = 0, n_hit = 0, n_miss = 0;                           // n_miss: of the wave (the same in all its lanes)
#pragma unroll
    for (int k = 0; k < PLAN_PER_THREAD; ++k) {
        const int64_t j = tile0 + (int64_t)k * PLAN_THREADS + threadIdx.x;
        int64_t tag = -1;
        if (j < n) {
            const int64_t e = route_of(rs, ids[j]);
            tag = entry_tag(e);
            entry[j] = e;
            if (one_batch) { n_local += tag == TAG_LOCAL; n_hit += tag == TAG_CACHE; }
            else if (tag != TAG_REMOTE) {
                const uint32_t b = batch_of_pos(batch_off, n_batches, j);
                atomicAdd(&counts[2 * (uint64_t)b + (tag == TAG_CACHE ? 1 : 0)], 1ull);
            }
        }
        const unsigned long long m = __ballot(tag == TAG_REMOTE);
        if (lane == 0) miss_bits[(uint64_t)blockIdx.x * PLAN_TILE_WORDS + k * (PLAN_THREADS / 64) + wave] = m;
        n_miss += (unsigned int)__popcll(m);
    }
    for (int o = 32; o > 0; o >>= 1) { n_local += __shfl_down(n_local, o, 64); n_hit += __shfl_down(n_hit, o, 64); }
    if (lane == 0) { red[0][wave] = n_local; red[1][wave] = n_hit; red[2][wave] = n_miss; }
    __syncthreads();
    if (threadIdx.x == 0) {
        unsigned int a = 0, h = 0, m = 0;
        for (int w = 0; w < PLAN_THREADS / 64; ++w) { a += red[0][w]; h += red[1][w]; m += red[2][w]; }
        tile_miss[blockIdx.x] = (int32_t)m;
        if (one_batch) {
            if (a) atomicAdd(&counts[2 * (uint64_t)b_first], (unsigned long long)a);
            if (h) atomicAdd(&counts[2 * (uint64_t)b_first + 1], (unsigned long long)h);
        }
    }
}

// Misses in front of position pos: those of the tiles in front of its tile (tile_scan) and of the words and bits in front of it inside the tile.
__device__ __forceinline__ int64_t misses_before(const unsigned long long *__restrict__ miss_bits, const int64_t *__restrict__ tile_scan, int64_t pos)
{
    const int64_t tile = pos / PLAN_TILE, word = pos >> 6;
    int64_t cnt = tile_scan[tile];
    for (int64_t w = tile * PLAN_TILE_WORDS; w < word; ++w) cnt += __popcll(miss_bits[w]);
    const int bit = (int)(pos & 63);
    if (bit) cnt += __popcll(miss_bits[word] & ((1ull << bit) - 1ull));
    return cnt;
}

// miss_off[b] = misses in front of batch b's first position (miss_off[n_batches] = all of them)
__global__ void miss_offsets_kernel(const unsigned long long *__restrict__ miss_bits, const int64_t *__restrict__ tile_scan, int64_t n, int64_t n_tiles,
                                    const int64_t *__restrict__ batch_off, uint32_t n_batches, int64_t *__restrict__ miss_off)
{
    const uint32_t b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b > n_batches) return;
    const int64_t pos = batch_off[b];
    miss_off[b] = pos >= n ? tile_scan[n_tiles] : misses_before(miss_bits, tile_scan, pos);
}

// miss_rows[rank of the miss] = its position within its batch, for every miss.  A workgroup takes one tile: every
// wave reads the tile's PLAN_TILE_WORDS words of miss bits (one per lane), scans their bit counts, and writes the
// misses of every fourth word.
__global__ void __launch_bounds__(256) miss_list_kernel(const unsigned long long *__restrict__ miss_bits, const int64_t *__restrict__ tile_scan,
                                                        const int64_t *__restrict__ batch_off, uint32_t n_batches, int32_t *__restrict__ miss_rows)
{
    static_assert(PLAN_TILE_WORDS <= 64 && PLAN_TILE_WORDS % 4 == 0, "a lane per word; four waves share the words");
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t tile = blockIdx.x;
    const unsigned long long mine = lane < PLAN_TILE_WORDS ? miss_bits[tile * PLAN_TILE_WORDS + lane] : 0ull;
    if (__ballot(mine != 0ull) == 0ull) return;                  // no miss in the tile
    int incl = __popcll(mine);
    for (int d = 1; d < PLAN_TILE_WORDS; d <<= 1) {
        const int y = __shfl_up(incl, d, 64);
        if (lane >= d) incl += y;
    }
    const int before_word = incl - __popcll(mine);               // misses of the tile in front of this lane's word
    const int64_t tile0 = tile * PLAN_TILE, tile_base = tile_scan[tile];
    // almost every tile lies inside one batch: its first position's batch then serves all of its positions
    const uint32_t b_first = batch_of_pos(batch_off, n_batches, tile0);
    const int64_t start_first = batch_off[b_first], end_first = batch_off[b_first + 1];
    for (int w = wave; w < PLAN_TILE_WORDS; w += 4) {
        const unsigned long long m = __shfl(mine, w, 64);
        const int before = __shfl(before_word, w, 64);
        if (!((m >> lane) & 1ull)) continue;
        const int64_t j = tile0 + 64 * w + lane;
        const int64_t start = j < end_first ? start_first : batch_off[batch_of_pos(batch_off, n_batches, j)];
        miss_rows[tile_base + before + __popcll(m & ((1ull << lane) - 1ull))] = (int32_t)(j - start);
    }
}

// Routing entries, miss lists and counts of one schedule.  What the
// plan keeps lives in `keep`; scratch in `tmp`.
rg_status build_plan(const rg_schedule *s, const RouteSources &rs, Arena &keep, Arena &tmp, hipStream_t st, Plan *plan)
{
    const uint32_t beta = s->n_batches;
    const HopData &h = s->hop[s->L];
    const int64_t n = beta ? h.off_host[beta] : 0;
    plan->schedule_uid = s->uid;
    plan->miss_off.assign((size_t)beta + 1, 0);
    plan->stats.assign(beta, rg_gather_stats{0, 0, 0, 0});
    RG_TRY(keep.dev_n<int64_t>((uint64_t)n, &plan->entry));
    if (beta == 0) { RG_TRY(keep.dev_n<int32_t>(0, &plan->miss_rows)); return RG_OK; }

    const int64_t n_tiles = (n + PLAN_TILE - 1) / PLAN_TILE, n_words = n_tiles * PLAN_TILE_WORDS;
    unsigned long long *miss_bits = nullptr;
    int32_t *tile_miss = nullptr;
    int64_t *tile_scan = nullptr, *miss_off_dev = nullptr;
    unsigned long long *counts = nullptr;
    RG_TRY(tmp.dev_n<unsigned long long>((uint64_t)std::max<int64_t>(n_words, 1), &miss_bits));
    RG_TRY(tmp.dev_n<int32_t>((uint64_t)std::max<int64_t>(n_tiles, 1), &tile_miss));
    RG_TRY(tmp.dev_n<int64_t>((uint64_t)n_tiles + 1, &tile_scan));
    RG_TRY(tmp.dev_n<int64_t>((uint64_t)beta + 1, &miss_off_dev));
    RG_TRY(tmp.dev_n<unsigned long long>(2 * (uint64_t)beta, &counts));
    RG_HIP(hipMemsetAsync(counts, 0, 2 * (uint64_t)beta * sizeof(unsigned long long), st));
    {
        ScopedTimer tm(KG_PLAN, st);
        if (n > 0)
            hipLaunchKernelGGL(plan_kernel, dim3((unsigned)n_tiles), dim3(PLAN_THREADS), 0, st, h.ids, n, h.off_dev, beta,
                               rs, plan->entry, miss_bits, tile_miss, counts);
        RG_TRY(scan_i32_to_i64(tile_miss, tile_scan, n_tiles, tmp, st));
        hipLaunchKernelGGL(miss_offsets_kernel, dim3((beta + 1 + 255) / 256), dim3(256), 0, st, miss_bits, tile_scan, n, n_tiles, h.off_dev, beta, miss_off_dev);
    }
    std::vector<unsigned long long> hc(2 * (size_t)beta);
    {
        Readback rb(st);
        RG_TRY(rb.add(plan->miss_off.data(), miss_off_dev, ((size_t)beta + 1) * sizeof(int64_t)));
        RG_TRY(rb.add(hc.data(), counts, hc.size() * sizeof(unsigned long long)));
        RG_TRY(rb.wait());
    }
    const int64_t n_miss = plan->miss_off[beta];
    RG_TRY(keep.dev_n<int32_t>((uint64_t)n_miss, &plan->miss_rows));
    if (n_miss > 0) {
        ScopedTimer tm(KG_PLAN, st);
        hipLaunchKernelGGL(miss_list_kernel, dim3((unsigned)n_tiles), dim3(256), 0, st, miss_bits, tile_scan, h.off_dev, beta, plan->miss_rows);
    }
    RG_HIP(hipGetLastError());
    for (uint32_t b = 0; b < beta; ++b) {
        rg_gather_stats &g = plan->stats[b];
        g.n_rows = (uint64_t)(h.off_host[b + 1] - h.off_host[b]);
        g.n_local = hc[2 * (size_t)b];
        g.n_hit = hc[2 * (size_t)b + 1];
        g.n_miss = (uint64_t)(plan->miss_off[b + 1] - plan->miss_off[b]);
    }
    RG_HIP(hipStreamSynchronize(st));
    return RG_OK;
}

// The tally as uint32_t[n_nodes] for rg_cache_view: the array itself, or -- where the build counted in bytes -- a
// widened copy made at the first request (device memory from the cache's allocator; the call waits for the copy).
rg_status cache_freq_view(const rg_cache *cc, const uint32_t **out)
{
    rg_cache *c = const_cast<rg_cache *>(cc);
    std::lock_guard<std::mutex> lk(c->view_mu);
    if (!c->freq && c->freq8 && c->n_nodes > 0) {
        hipStream_t side = nullptr;
        RG_TRY(helper_stream(&side));
        uint32_t *wide = nullptr;
        RG_TRY(c->arena.dev_n<uint32_t>((uint64_t)c->n_nodes, &wide));
        const unsigned grid = (unsigned)std::max<int64_t>(1, std::min<int64_t>((c->n_nodes + 255) / 256, 1 << 16));
        hipLaunchKernelGGL(widen_freq_kernel, dim3(grid), dim3(256), 0, side, c->freq8, c->n_nodes, wide);
        RG_HIP(hipGetLastError());
        RG_HIP(hipStreamSynchronize(side));
        c->freq = wide;
    }
    *out = c->freq;
    return RG_OK;
}

// slot_of as int32_t[n_nodes] for rg_cache_view, made from the slot map at the first request in the same way.
rg_status cache_slot_view(const rg_cache *cc, const int32_t **out)
{
    rg_cache *c = const_cast<rg_cache *>(cc);
    std::lock_guard<std::mutex> lk(c->view_mu);
    if (!c->slot_of && c->slot_pairs && c->n_nodes > 0) {
        hipStream_t side = nullptr;
        RG_TRY(helper_stream(&side));
        int32_t *wide = nullptr;
        RG_TRY(c->arena.dev_n<int32_t>((uint64_t)c->n_nodes, &wide));
        const unsigned grid = (unsigned)std::max<int64_t>(1, std::min<int64_t>((c->n_nodes + 255) / 256, 1 << 16));
        hipLaunchKernelGGL(widen_slots_kernel, dim3(grid), dim3(256), 0, side, c->slot_pairs, c->n_nodes, wide);
        RG_HIP(hipGetLastError());
        RG_HIP(hipStreamSynchronize(side));
        c->slot_of = wide;
    }
    *out = c->slot_of;
    return RG_OK;
}

static rg_status build_cache_impl(const rg_schedule *const *epochs, uint32_t n_epochs, const rg_features *f, uint64_t K,
                                  const rg_allocator *a, hipStream_t st, rg_cache *c)
{
    const int64_t n = epochs[0]->n_nodes;
    c->n_nodes = n;
    c->row_bytes = f->row_bytes;
    c->stride = ((uint64_t)f->row_bytes + 15) / 16 * 16;
    c->remote_rows_seen = f->remote_rows;
    c->remote_is_device = is_device_memory(f->remote_rows);
    Arena tmp(a, st);
    RG_HIP(hipEventCreateWithFlags(&c->ev_fork, hipEventDisableTiming));
    RG_HIP(hipEventCreateWithFlags(&c->ev_join, hipEventDisableTiming));

    int dev = 0, n_cu = 256;
    RG_HIP(hipGetDevice(&dev));
    RG_HIP(hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev));

    // ---- a6: tally
    uint64_t max_freq = 0;
    bool from_bitmaps = false;
    for (uint32_t e = 0; e < n_epochs; ++e) { max_freq += epochs[e]->n_batches; from_bitmaps = from_bitmaps || epochs[e]->epoch_freq; }
    bool narrow = max_freq <= 255;                       // byte counters suffice
    if (const char *force = getenv("RAPIDGNN_NARROW_TALLY"); force && force[0] == '0') narrow = false;      // same results either way; for tests and tuning
    const uint64_t tally_bytes = narrow ? ((uint64_t)n + 15) / 16 * 16 : (uint64_t)n * sizeof(uint32_t);
    void *tally = nullptr;
    RG_TRY(c->arena.dev(tally_bytes ? tally_bytes : 16, &tally));
    if (narrow) c->freq8 = (uint8_t *)tally; else c->freq = (uint32_t *)tally;
    RG_HIP(hipMemsetAsync(tally, 0, tally_bytes, st));
    for (uint32_t e = 0; e < n_epochs; ++e) {
        const rg_schedule *s = epochs[e];
        if (s->n_batches == 0) continue;
        const HopData &h = s->hop[s->L];
        const int64_t m = h.off_host[s->n_batches];
        if (m == 0) continue;
        ScopedTimer tm(KG_HIST, st);
        if (s->epoch_freq) {
            const dim3 grid((unsigned)((n + 255) / 256));
            if (narrow) hipLaunchKernelGGL(add_epoch_freq_kernel<uint8_t>, grid, dim3(256), 0, st, s->epoch_freq, n, c->freq8);
            else hipLaunchKernelGGL(add_epoch_freq_kernel<uint32_t>, grid, dim3(256), 0, st, s->epoch_freq, n, c->freq);
            continue;
        }
        const unsigned grid = (unsigned)std::min<int64_t>((m + 255) / 256, (int64_t)n_cu * 32);
        if (narrow) hipLaunchKernelGGL(tally_kernel<uint8_t>, dim3(grid), dim3(256), 0, st, h.ids, m, c->freq8);
        else hipLaunchKernelGGL(tally_kernel<uint32_t>, dim3(grid), dim3(256), 0, st, h.ids, m, c->freq);
    }
    RG_HIP(hipGetLastError());

    // ---- a7: TopHot
    SelectState *stp = nullptr;
    unsigned long long *bins = nullptr;
    RG_TRY(tmp.dev_n<SelectState>(1, &stp));
    RG_TRY(tmp.dev_n<unsigned long long>((uint64_t)BIN_COPIES * DIGIT_BINS, &bins));
    RG_HIP(hipMemsetAsync(stp, 0, sizeof(SelectState), st));
    RG_HIP(hipMemsetAsync(bins, 0, (size_t)BIN_COPIES * DIGIT_BINS * sizeof(unsigned long long), st));
    int bits = 1;
    while (bits < 32 && (max_freq >> bits) != 0) ++bits;
    const int passes = (bits + DIGIT_BITS - 1) / DIGIT_BITS;
    const bool local4 = ((uintptr_t)f->is_local & 3) == 0, local8 = ((uintptr_t)f->is_local & 7) == 0,      // the caller's array: wide loads only if it allows them
               local16 = ((uintptr_t)f->is_local & 15) == 0;
    const int64_t sel_blocks = (n + SEL_TILE - 1) / SEL_TILE;
    uint64_t *block_tot = nullptr;
    RG_TRY(tmp.dev_n<uint64_t>((uint64_t)(sel_blocks ? sel_blocks : 1), &block_tot));
    const int64_t sel_tiles = (sel_blocks + SCAN_TILE - 1) / SCAN_TILE;
    uint64_t *tile_tot = nullptr;
    RG_TRY(tmp.dev_n<uint64_t>((uint64_t)(sel_tiles ? sel_tiles : 1), &tile_tot));
    {
        ScopedTimer tm(KG_TOPK, st);
        const unsigned grid = (unsigned)std::max<int64_t>(1, std::min<int64_t>((n + TOPK_THREADS - 1) / TOPK_THREADS, (int64_t)n_cu * 16));
        for (int p = 0; p < passes; ++p) {
            const int shift = (passes - 1 - p) * DIGIT_BITS;
            if (narrow) {
                if (local16) hipLaunchKernelGGL(digit_histogram8_kernel<true>, dim3(grid), dim3(TOPK_THREADS), 0, st, c->freq8, f->is_local, n, stp, bins);
                else hipLaunchKernelGGL(digit_histogram8_kernel<false>, dim3(grid), dim3(TOPK_THREADS), 0, st, c->freq8, f->is_local, n, stp, bins);
            } else if (local4) hipLaunchKernelGGL(digit_histogram_kernel<true>, dim3(grid), dim3(TOPK_THREADS), 0, st, c->freq, f->is_local, n, stp, shift, bins);
            else hipLaunchKernelGGL(digit_histogram_kernel<false>, dim3(grid), dim3(TOPK_THREADS), 0, st, c->freq, f->is_local, n, stp, shift, bins);
            hipLaunchKernelGGL(choose_digit_kernel, dim3(1), dim3(DIGIT_BINS), 0, st, stp, bins, shift, p == 0 ? 1 : 0, K);
        }
        if (sel_blocks > 0) {
            const dim3 sg((unsigned)sel_blocks), sb(TOPK_THREADS);
            if (narrow && local8) hipLaunchKernelGGL((select_block_totals<true, uint8_t>), sg, sb, 0, st, c->freq8, f->is_local, n, stp, block_tot);
            else if (narrow) hipLaunchKernelGGL((select_block_totals<false, uint8_t>), sg, sb, 0, st, c->freq8, f->is_local, n, stp, block_tot);
            else if (local8) hipLaunchKernelGGL((select_block_totals<true, uint32_t>), sg, sb, 0, st, c->freq, f->is_local, n, stp, block_tot);
            else hipLaunchKernelGGL((select_block_totals<false, uint32_t>), sg, sb, 0, st, c->freq, f->is_local, n, stp, block_tot);
            hipLaunchKernelGGL(select_scan_tiles, dim3((unsigned)sel_tiles), dim3(TOPK_THREADS), 0, st, block_tot, sel_blocks, tile_tot);
            hipLaunchKernelGGL(select_scan_totals, dim3(1), dim3(TOPK_THREADS), 0, st, tile_tot, sel_tiles);
        }
    }
    SelectState hs;
    {
        Readback rb(st);
        RG_TRY(rb.add(&hs, stp, sizeof(SelectState)));
        RG_TRY(rb.wait());
    }
    c->K_eff = hs.k_eff;
    RG_TRY(c->arena.dev_n<int32_t>(c->K_eff, &c->cache_ids));
    int64_t *fill_entries = nullptr;
    RG_TRY(tmp.dev_n<int64_t>(c->K_eff ? c->K_eff : 1, &fill_entries));
    RG_TRY(c->arena.dev_n<SlotRec>((uint64_t)std::max<int64_t>(sel_blocks, 1) * (SEL_TILE / 32), &c->slot_pairs));      // whole tiles: every thread of the select pass writes its share
    if (sel_blocks > 0) {
        ScopedTimer tm(KG_TOPK, st);
        const dim3 sg((unsigned)sel_blocks), sb(TOPK_THREADS);
        if (narrow && local8)
            hipLaunchKernelGGL((select_emit_kernel<true, uint8_t>), sg, sb, 0, st, c->freq8, f->is_local, n, stp, block_tot, tile_tot, c->cache_ids, c->slot_pairs, f->row_of, fill_entries);
        else if (narrow)
            hipLaunchKernelGGL((select_emit_kernel<false, uint8_t>), sg, sb, 0, st, c->freq8, f->is_local, n, stp, block_tot, tile_tot, c->cache_ids, c->slot_pairs, f->row_of, fill_entries);
        else if (local8)
            hipLaunchKernelGGL((select_emit_kernel<true, uint32_t>), sg, sb, 0, st, c->freq, f->is_local, n, stp, block_tot, tile_tot, c->cache_ids, c->slot_pairs, f->row_of, fill_entries);
        else
            hipLaunchKernelGGL((select_emit_kernel<false, uint32_t>), sg, sb, 0, st, c->freq, f->is_local, n, stp, block_tot, tile_tot, c->cache_ids, c->slot_pairs, f->row_of, fill_entries);
    }
    RG_HIP(hipGetLastError());

    // ---- a8: VectorPull -- one bulk gather of the selected rows out of the remote table.  It streams rows while the
    // plans below are bound by dependent lookups, and neither reads what the other writes: the fill goes to the
    // library's helper stream and runs beside them.
    RG_TRY(c->arena.dev(c->K_eff * c->stride, &c->rows));
    if (tls_table_bytes_sink) tls_table_bytes_sink->store(c->K_eff * c->stride, std::memory_order_release);
    struct Forked {                                       // declared after `tmp`: on every exit the fill has ended before tmp's blocks go back
        hipStream_t side = nullptr;
        ~Forked() { if (side) (void)hipStreamSynchronize(side); }
    } forked;
    if (c->K_eff > 0) {
        hipStream_t side = nullptr;
        RG_TRY(helper_stream(&side));
        RG_HIP(hipEventRecord(c->ev_fork, st));
        RG_HIP(hipStreamWaitEvent(side, c->ev_fork, 0));
        forked.side = side;
        RowSources src{(const uint8_t *)f->local_rows, f->local_stride, (const uint8_t *)c->rows, c->stride,
                       (const uint8_t *)f->remote_rows, f->remote_stride};
        RG_TRY(launch_gather(fill_entries, (int64_t)c->K_eff, nullptr, 0, 1, src, f->row_bytes, (uint8_t *)c->rows, c->stride, side, KG_FILL));
        RG_HIP(hipEventRecord(c->ev_join, side));
    }

    // ---- a5/a9: plans, miss lists and counts for every batch of every epoch
    c->plans.resize(n_epochs);
    const RouteSources rs{f->row_of, c->slot_pairs};
    for (uint32_t e = 0; e < n_epochs; ++e) RG_TRY(build_plan(epochs[e], rs, c->arena, tmp, st, &c->plans[e]));
    if (forked.side) RG_HIP(hipStreamWaitEvent(st, c->ev_join, 0));
    RG_HIP(hipStreamSynchronize(st));
    if (forked.side) { RG_HIP(hipStreamSynchronize(forked.side)); forked.side = nullptr; }
    tmp.drained();
    return RG_OK;
}

}  // namespace rg

using namespace rg;

extern "C" rg_status rg_build_cache(const rg_schedule *const *epochs, uint32_t n_epochs, const rg_features *f, uint64_t K,
                                    const rg_allocator *a, void *stream, rg_cache **out)
{
    if (!epochs || n_epochs == 0 || !f || !out) { set_error("rg_build_cache: null argument or no epoch"); return RG_EINVAL; }
    for (uint32_t e = 0; e < n_epochs; ++e) {
        if (!epochs[e]) { set_error("rg_build_cache: epochs[%u] is null", e); return RG_EINVAL; }
        if (epochs[e]->n_nodes != epochs[0]->n_nodes) { set_error("rg_build_cache: epochs disagree on n_nodes"); return RG_EINVAL; }
    }
    if (epochs[0]->n_nodes > 0 && (!f->is_local || !f->row_of)) { set_error("rg_build_cache: null is_local / row_of"); return RG_EINVAL; }
    if (f->row_bytes == 0) { set_error("rg_build_cache: row_bytes must be > 0"); return RG_EINVAL; }
    if (f->local_stride < f->row_bytes || f->remote_stride < f->row_bytes) { set_error("rg_build_cache: a stride is smaller than row_bytes"); return RG_EINVAL; }

    rg_cache *c = new (std::nothrow) rg_cache(a);
    if (!c) { set_error("rg_build_cache: out of host memory"); return RG_ENOMEM; }
    rg_status rc = build_cache_impl(epochs, n_epochs, f, K, a, as_stream(stream), c);
    if (rc != RG_OK) {
        (void)hipStreamSynchronize(as_stream(stream));
        rg_cache_destroy(c);
        return rc;
    }
    *out = c;
    return RG_OK;
}
