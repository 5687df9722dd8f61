// a3: per-hop fan-out sampling, SAMPLE(eta(v), f) for every frontier node of
// every batch of the epoch in one launch (Sec. 2.1 node-wise sampling; Sec. 4
// par. (2)).
//
// SAMPLE keeps the f neighbours with the smallest keys key32(S_v, u) and emits
// them in row order.  One wavefront works on one row at a time (or one tile of
// a long row), one wave per workgroup.
//
// A first, thread-per-node kernel writes one record per frontier node (row
// start, degree, batch, node state S_v, sample size, tile count), so that the
// sampling waves never chase frontier -> indptr -> row or search for a node's
// batch: a wave takes 64 consecutive frontier nodes, loads their records with
// one coalesced load each, and walks them with lane broadcasts, the next
// node's first 64 neighbour IDs already in flight while the current node is
// sampled.
//
//  - deg <= f: the row is the sample; it is copied.
//  - deg <= 256: the row sits in registers (1 or 4 IDs per lane).  A threshold
//    that exactly f keys do not exceed is found by bisection on ballots, and the
//    kept IDs are compacted straight into the output with ballot/popcount
//    ranks, which preserves row order.
//  - longer rows are streamed once in 1 KB blocks aligned to cache lines, one
//    16-byte load per lane, the next block's load already in flight.  IDs whose
//    key is not above the current cut are appended (ballot ranks again, so in
//    row order) to an LDS buffer of CAP >= f + 64 IDs; when the buffer would
//    overflow it is pruned to the f smallest keys with the same search and an
//    in-place ordered compaction, which also tightens the cut.  What is left
//    after the last block is the sample.
//  - rows longer than BIG_ROW are cut into T near-equal tiles, each sampled by
//    its own wave into scratch (f IDs per tile, row order); a second small
//    launch samples the concatenation of a row's tile results, which is the
//    row's sample: the f smallest keys of the row are among the f smallest of
//    each tile.  This bounds the work of one wave whatever the degree skew.
//    Tiles are dealt out by workgroup index and done before the groups of
//    nodes, which the waves then take from a counter as they become free.
//
// No step sorts anything.  While a wave writes a sample it also marks the
// batch's reached-ID bitmaps, so frontier dedup costs no extra pass.
#include "rg_internal.h"
#include "rg_device.h"

#include <algorithm>
#include <atomic>
#include <cstdlib>

namespace rg {


constexpr int TINY_ROW = 8;              // rows of up to this many IDs that need no sampling are copied by one lane each
constexpr int BIG_ROW = 16384;           // rows longer than this are sampled tile by tile ...
constexpr int TILE_PIECE = 65536;        // ... in near-equal pieces of at most this many IDs.  (A row of 16,385 to 65,536 IDs is one tile: it is
                                         // sampled among the tile jobs, where the batches that share it meet in the caches.  Measured on the five
                                         // workloads: pieces of 16,384 cost 8 % more sampling time on the largest graph, pieces of 131,072 7 %;
                                         // tiling from 8,192 IDs on is 3 % slower there and 3 % faster on large_sparse.)
__device__ __host__ __forceinline__ int64_t tiles_of(int64_t deg) { return deg > BIG_ROW ? (deg + TILE_PIECE - 1) / TILE_PIECE : 0; }

// Per frontier node, by position: where its row starts, its degree, its batch and its stream.
struct NodeRecs {
    int64_t *row_begin;
    int32_t *deg;
    uint32_t *batch;
    uint64_t *state;      // S_v = combine(combine(S_{e,i}, hop + 1), v)
};

// Also adds up, over the frontier, what the hop will read of the adjacency: [0] the sum of the degrees (in IDs),
// [1] the part of it in rows of up to BIG_ROW IDs (the rows that are not sampled as tiles), [2] the number of rows of
// 1 .. SHORT_ROW IDs and [3] the IDs in them.  The sums are spread over DEG_SUM_SLOTS sets of four counters,
// total[4 * slot + k], which the host adds up: thousands of workgroups adding to one address would queue up behind
// each other.
constexpr int DEG_SUM_SLOTS = 64;
constexpr int DEG_SUMS = 4;
constexpr int SHORT_ROW = 64;            // rows of up to this many IDs are sampled four at a time, sixteen lanes each
__global__ void __launch_bounds__(256) node_records_kernel(const int64_t *__restrict__ indptr, const int32_t *__restrict__ frontier, int64_t n,
                                                           const int64_t *__restrict__ batch_off, uint32_t n_batches, const uint64_t *__restrict__ batch_seed,
                                                           uint32_t hop, uint32_t fanout, NodeRecs r, int32_t *__restrict__ cnt, int32_t *__restrict__ tiles,
                                                           int64_t n_nodes, unsigned long long *__restrict__ total)
{
    __shared__ unsigned long long part[DEG_SUMS][4];
    unsigned long long acc[DEG_SUMS] = {0, 0, 0, 0};
    // (a bounded grid, each workgroup striding over the frontier: the sums cost two atomics per workgroup)
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
        const int32_t v = frontier[i];
        const bool known = v >= 0 && (int64_t)v < n_nodes;      // (a seed out of range is refused by the host at the hop's readback; until then it has no row)
        const int64_t b0 = known ? indptr[v] : 0;
        const int64_t deg = known ? indptr[v + 1] - b0 : 0;
        const uint32_t b = batch_of(batch_off, n_batches, i);
        r.row_begin[i] = b0;
        r.deg[i] = (int32_t)deg;
        r.batch[i] = b;
        r.state[i] = combine(combine(batch_seed[b], (uint64_t)hop + 1u), (uint64_t)(uint32_t)v);
        cnt[i] = (int32_t)(deg < (int64_t)fanout ? deg : (int64_t)fanout);
        tiles[i] = (int32_t)tiles_of(deg);
        acc[0] += (unsigned long long)deg;
        if (deg <= (int64_t)BIG_ROW) acc[1] += (unsigned long long)deg;
        if (deg > 0 && deg <= (int64_t)SHORT_ROW) { acc[2] += 1; acc[3] += (unsigned long long)deg; }
    }
#pragma unroll
    for (int k = 0; k < DEG_SUMS; ++k) {
        for (int o = 32; o > 0; o >>= 1) acc[k] += __shfl_down(acc[k], o, 64);
        if ((threadIdx.x & 63) == 0) part[k][threadIdx.x >> 6] = acc[k];
    }
    __syncthreads();
    if (threadIdx.x < DEG_SUMS) {
        const unsigned long long a = part[threadIdx.x][0] + part[threadIdx.x][1] + part[threadIdx.x][2] + part[threadIdx.x][3];
        if (a) atomicAdd(total + DEG_SUMS * (blockIdx.x % DEG_SUM_SLOTS) + threadIdx.x, a);
    }
}

// Number of set bits of m below this lane's bit (m wave-uniform): the two mbcnt instructions.
__device__ __forceinline__ int lanes_below(unsigned long long m, int lane)
{
    (void)lane;
    return (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
}

// This lane's bit of a wave-uniform mask, as a condition the vector unit takes straight from the scalar pair.
__device__ __forceinline__ bool my_bit(unsigned long long m) { return __builtin_amdgcn_inverse_ballot_w64(m); }

// The lane mask of a predicate, taken straight from the compare.
__device__ __forceinline__ unsigned long long ballot64(bool p) { return __builtin_amdgcn_ballot_w64(p); }

// Values that are the same in every lane of the wave, pinned to scalar registers so that the
// branches and loops they steer are scalar too.
__device__ __forceinline__ int uni(int x) { return __builtin_amdgcn_readfirstlane(x); }
__device__ __forceinline__ uint32_t uni(uint32_t x) { return (uint32_t)__builtin_amdgcn_readfirstlane((int)x); }
__device__ __forceinline__ bool uni(bool x) { return __builtin_amdgcn_readfirstlane((int)x) != 0; }

__device__ __forceinline__ int64_t bcast64(int64_t x, int src_lane)
{
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)x, src_lane);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)((uint64_t)x >> 32), src_lane);
    return (int64_t)(((uint64_t)hi << 32) | lo);
}

// The lanes 0 .. n-1 (n clamped to [0, 64]) as a mask.
__device__ __forceinline__ unsigned long long low_lanes(int n)
{
    return n >= 64 ? ~0ull : (n <= 0 ? 0ull : (1ull << n) - 1ull);
}

// Lane masks instead of per-lane booleans: a mask is one compare (ballot of a single comparison)
// and everything after it -- AND with the valid lanes, population counts, comparisons with f --
// is scalar work that the vector unit never sees.

// A threshold that exactly `keep` of the keys held in registers do not exceed.  k[e] is valid in
// the lanes of vm[e]; `total` >= keep keys are valid in all.  Search on the key value: the
// keep-th smallest key stays inside [lo, lo + 2^(bit+1)), and the search stops as soon as the
// number of keys below the bracket's upper end is exactly `keep` -- after about log2(total)
// bits for spread-out keys, 32 at most (keys are distinct).  Two bits are decided per step: the three
// inner quarter points are compared at once (independent compares and counts), which halves the
// number of dependent compare -> count -> decide chains a wave has to sit through; the outcome is
// that of two halving steps.  `upper` is a bound no valid key exceeds (the cut the keys were
// collected under, else 2^32 - 1): the search starts at its leading bit instead of bit 31.
template <int E>
__device__ __forceinline__ uint32_t kth_key_threshold(const uint32_t (&k)[E], const unsigned long long (&vm)[E], int keep, int total,
                                                      uint32_t upper = 0xFFFFFFFFu)
{
    keep = uni(keep);
    uint32_t lo = 0;
    int below_hi = uni(total);
    int bit = uni(31 - __clz((int)(upper | 1u)));
    while (below_hi != keep && bit >= 1) {
        const uint32_t q = 1u << (bit - 1);
        const uint32_t t1 = lo | q, t2 = lo | (q << 1), t3 = t2 | q;
        int c1 = 0, c2 = 0, c3 = 0;
#pragma unroll
        for (int e = 0; e < E; ++e) {
            c1 += __popcll(ballot64(k[e] < t1) & vm[e]);
            c2 += __popcll(ballot64(k[e] < t2) & vm[e]);
            c3 += __popcll(ballot64(k[e] < t3) & vm[e]);
        }
        if (c1 >= keep) below_hi = c1;                           // first quarter
        else if (c2 >= keep) { lo = t1; below_hi = c2; }
        else if (c3 >= keep) { lo = t2; below_hi = c3; }
        else lo = t3;                                            // last quarter: the count below its upper end is unchanged
        bit -= 2;
    }
    if (below_hi != keep && bit == 0) {                          // a single bit left
        const uint32_t trial = lo | 1u;
        int below = 0;
#pragma unroll
        for (int e = 0; e < E; ++e) below += __popcll(ballot64(k[e] < trial) & vm[e]);
        if (below < keep) lo = trial; else below_hi = below;
        bit = -1;
    }
    return lo + (uint32_t)((((uint64_t)1) << (bit + 1)) - 1u);
}

// Row of f < len <= 64 * E IDs held in registers (u[e] of lane l is row[e * 64 + l]),
// sampled and written to out in row order.  buf: scratch of at least 64 entries (used when E > 1).
template <int E, int MARK>
__device__ __forceinline__ void sample_registers(const uint32_t (&u)[E], int len, int f, uint32_t lo, uint32_t hi, int lane, uint32_t *buf,
                                                 int32_t *__restrict__ out, const ReachedOfBatch &reached_b)
{
    len = uni(len); f = uni(f); lo = uni(lo); hi = uni(hi);
    uint32_t k[E];
    unsigned long long vm[E];
#pragma unroll
    for (int e = 0; e < E; ++e) {
        vm[e] = low_lanes(len - e * 64);
        k[e] = key32(lo, hi, u[e]);
    }
    uint32_t cut = 0;
    bool have_cut = false;
    if (E > 1) {
        // As for long rows, a cut guessed from the key distribution first: about lambda of the row's keys lie below
        // lambda / len.  If between f and 64 do, the threshold is searched among those alone, one key per lane and
        // from the guessed cut's leading bit down, instead of among all E registers from bit 31; the f smallest keys of the
        // row are among them, so the result is the same.  Otherwise (or for rows too short to guess) the search below.
        const float lambda = (float)f + 4.0f * __fsqrt_rn((float)f) + 8.0f;
        if (uni(lambda * 2.0f <= (float)len)) {
            const uint32_t guessed = uni((uint32_t)(lambda / (float)len * 4294967296.0f));
            unsigned long long m[E];
            int total = 0;
#pragma unroll
            for (int e = 0; e < E; ++e) {
                m[e] = ballot64(k[e] <= guessed) & vm[e];
                total += __popcll(m[e]);
            }
            if (total >= f && total <= 64) {
                int base = 0;
#pragma unroll
                for (int e = 0; e < E; ++e) {
                    if (my_bit(m[e])) buf[base + lanes_below(m[e], lane)] = k[e];
                    base += __popcll(m[e]);
                }
                __syncthreads();
                const uint32_t ck[1] = {lane < total ? buf[lane] : 0u};
                const unsigned long long cvm[1] = {low_lanes(total)};
                cut = kth_key_threshold<1>(ck, cvm, f, total, guessed);
                if (cut > guessed) cut = guessed;      // (the search may answer with the end of its bracket: keys above the guess are no candidates)
                have_cut = true;
                __syncthreads();      // the scratch is free again
            }
        }
    }
    if (!have_cut) cut = kth_key_threshold<E>(k, vm, f, len);
    int base = 0;
#pragma unroll
    for (int e = 0; e < E; ++e) {
        const unsigned long long m = ballot64(k[e] <= cut) & vm[e];
        if (e * 64 + lane < len && k[e] <= cut) {
            out[base + lanes_below(m, lane)] = (int32_t)u[e];
            mark_reached<MARK>(reached_b, u[e]);
        }
        base += __popcll(m);
    }
}

// Keeps the `keep` smallest-key entries of buf[0..cnt), order preserved; returns a threshold that
// exactly those entries' keys do not exceed.
// Precondition: cnt > keep >= 1, cnt <= CAP.
template <int CAP>
__device__ __forceinline__ uint32_t prune_buffer(uint32_t *buf, int cnt, int keep, uint32_t lo, uint32_t hi, int lane, uint32_t upper)
{
    constexpr int E = CAP / 64;
    cnt = uni(cnt); keep = uni(keep); lo = uni(lo); hi = uni(hi);
    uint32_t u[E], k[E];
    unsigned long long vm[E];
#pragma unroll
    for (int e = 0; e < E; ++e) {
        const int idx = e * 64 + lane;
        vm[e] = low_lanes(cnt - e * 64);
        u[e] = idx < cnt ? buf[idx] : 0u;
        k[e] = key32(lo, hi, u[e]);
    }
    const uint32_t cut = uni(kth_key_threshold<E>(k, vm, keep, cnt, uni(upper)));
    __syncthreads();          // every lane has read its entries before any is overwritten
    int base = 0;
#pragma unroll
    for (int e = 0; e < E; ++e) {
        const unsigned long long m = ballot64(k[e] <= cut) & vm[e];
        if (e * 64 + lane < cnt && k[e] <= cut) buf[base + lanes_below(m, lane)] = u[e];
        base += __popcll(m);
    }
    __syncthreads();
    return cut;
}

// State of the candidate buffer while a long row streams by.
struct Stream {
    int cnt;          // entries in the buffer (wave-uniform)
    bool open;        // no cut yet: every ID is a candidate
    uint32_t cut;     // candidates must have key <= cut once !open
};

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// A block is up to 256 consecutive IDs of the row; lane l holds IDs 4l .. 4l+3 of the block (one
// 16-byte load), so row order is lane-major and ID e of a lane is valid in the lanes of vm[e].
// Appends the block's candidates to the buffer in row order.  If they do not fit, the buffer is
// pruned first (which tightens the cut and may drop some of them); if they still do not fit, the
// block goes in four quarters of 64 consecutive IDs.
// MAYBE_OPEN = false: the caller knows a cut is in force (s.open is false), which takes the test out of the loop.
template <int CAP, bool MAYBE_OPEN = true>
__device__ __forceinline__ void append_block(const uint32_t (&u)[4], const uint32_t (&k)[4], const unsigned long long (&vm)[4], int f, uint32_t lo,
                                             uint32_t hi, int lane, uint32_t *buf, Stream &s)
{
    f = uni(f); lo = uni(lo); hi = uni(hi);
    s.cnt = uni(s.cnt); s.open = MAYBE_OPEN ? uni(s.open) : false; s.cut = uni(s.cut);
    unsigned long long m[4];
    int total = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        m[e] = (MAYBE_OPEN && s.open) ? vm[e] : (ballot64(k[e] <= s.cut) & vm[e]);
        total += __popcll(m[e]);
    }
    if (total == 0) return;
    if (s.cnt + total > CAP && s.cnt > f) {
        s.cut = prune_buffer<CAP>(buf, s.cnt, f, lo, hi, lane, ((MAYBE_OPEN && s.open) ? 0xFFFFFFFFu : s.cut));
        s.cnt = f;
        s.open = false;
        total = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            m[e] &= ballot64(k[e] <= s.cut);
            total += __popcll(m[e]);
        }
        if (total == 0) return;
    }
    if (s.cnt + total <= CAP) {
        const unsigned long long any = m[0] | m[1] | m[2] | m[3];
        if (__popcll(any) == total) {
            // The usual event: no lane holds two candidates, so lane order is row order: one rank, one store.
            if (my_bit(any)) {
                const uint32_t v = my_bit(m[0]) ? u[0] : my_bit(m[1]) ? u[1] : my_bit(m[2]) ? u[2] : u[3];
                buf[s.cnt + lanes_below(any, lane)] = v;
            }
            s.cnt += total;
            return;
        }
        int rank = s.cnt;
#pragma unroll
        for (int e = 0; e < 4; ++e) rank += lanes_below(m[e], lane);
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (my_bit(m[e])) buf[rank++] = u[e];
        s.cnt += total;
        return;
    }
    for (int q = 0; q < 4; ++q) {             // lanes 16q .. 16q+15 hold 64 consecutive IDs
        if (s.cnt > CAP - 64) {
            s.cut = prune_buffer<CAP>(buf, s.cnt, f, lo, hi, lane, ((MAYBE_OPEN && s.open) ? 0xFFFFFFFFu : s.cut));
            s.cnt = f;
            s.open = false;
        }
        const unsigned long long quarter = 0xFFFFull << (16 * q);
        unsigned long long mq[4];
        int rank = s.cnt, sub = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            mq[e] = m[e] & quarter;
            if (!(MAYBE_OPEN && s.open)) mq[e] &= ballot64(k[e] <= s.cut);
            rank += lanes_below(mq[e], lane);
            sub += __popcll(mq[e]);
        }
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (my_bit(mq[e])) buf[rank++] = u[e];
        s.cnt += sub;
    }
}

// IDs p[4 * lane .. 4 * lane + 3] of a block of which `left` (> 0) IDs lie inside the row; p is 16-byte aligned.
__device__ __forceinline__ u32x4 load_block(const int32_t *__restrict__ p, int left, int lane)
{
    const int j = 4 * lane;
    if (left >= 256 || j + 3 < left) return *reinterpret_cast<const u32x4 *>(p + j);
    u32x4 r = {0u, 0u, 0u, 0u};
    if (j < left) r.x = (uint32_t)p[j];
    if (j + 1 < left) r.y = (uint32_t)p[j + 1];
    if (j + 2 < left) r.z = (uint32_t)p[j + 2];
    return r;
}

// Valid lanes of ID e of a block that holds `count` IDs: 4 * lane + e < count.
__device__ __forceinline__ unsigned long long block_lanes(int count, int e) { return low_lanes((count - e + 3) >> 2); }

// A long row is read as its head (the IDs in front of the first 128-byte boundary, fewer than 32) and aligned blocks.
__device__ __forceinline__ int row_head(const int32_t *row, int len)
{
    const int head = (32 - (int)(((uintptr_t)row >> 2) & 31)) & 31;
    return head > len ? len : head;
}
// What a row of len > 64 IDs needs besides its leading 64, fetched ahead of the row's turn: for len <= 256 the IDs
// row[64 + lane], row[128 + lane], row[192 + lane] (x, y, z; 0 past the end), for longer rows the first aligned block.
__device__ __forceinline__ u32x4 row_ahead(const int32_t *__restrict__ row, int len, int lane)
{
    len = uni(len);
    if (len <= 256) {
        u32x4 r = {0u, 0u, 0u, 0u};
        if (64 + lane < len) r.x = (uint32_t)row[64 + lane];
        if (128 + lane < len) r.y = (uint32_t)row[128 + lane];
        if (192 + lane < len) r.z = (uint32_t)row[192 + lane];
        return r;
    }
    const int head = uni(row_head(row, len));
    return load_block(row + head, len - head, lane);
}

template <int CAP, bool FULL, bool MAYBE_OPEN = true>
__device__ __forceinline__ void stream_block(const u32x4 &blk, int count, int f, uint32_t lo, uint32_t hi, int lane, uint32_t *buf, Stream &s)
{
    count = uni(count); f = uni(f); lo = uni(lo); hi = uni(hi);
    const uint32_t u[4] = {blk.x, blk.y, blk.z, blk.w};
    uint32_t k[4];
    unsigned long long vm[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        k[e] = key32(lo, hi, u[e]);
        vm[e] = FULL ? ~0ull : block_lanes(count, e);
    }
    append_block<CAP, MAYBE_OPEN>(u, k, vm, f, lo, hi, lane, buf, s);
}

// A full block while a cut is in force, the common outcomes only: no candidate, or candidates that fit the buffer.
// Returns false, with nothing done, when they do not fit; the caller then takes the block through append_block.
template <int CAP>
__device__ __forceinline__ bool stream_full_block_fast(const u32x4 &blk, uint32_t lo, uint32_t hi, int lane, uint32_t *buf, Stream &s)
{
    const uint32_t u[4] = {blk.x, blk.y, blk.z, blk.w};
    const uint32_t cut = uni(s.cut);
    s.cnt = uni(s.cnt);
    unsigned long long m[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) m[e] = ballot64(key32(lo, hi, u[e]) <= cut);
    const unsigned long long any = m[0] | m[1] | m[2] | m[3];
    if (any == 0ull) return true;
    const int total = __popcll(m[0]) + __popcll(m[1]) + __popcll(m[2]) + __popcll(m[3]);
    if (s.cnt + total > CAP) return false;
    if (__popcll(any) == total) {
        if (my_bit(any)) {
            const uint32_t v = my_bit(m[0]) ? u[0] : my_bit(m[1]) ? u[1] : my_bit(m[2]) ? u[2] : u[3];
            buf[s.cnt + lanes_below(any, lane)] = v;
        }
    } else {
        int rank = s.cnt;
#pragma unroll
        for (int e = 0; e < 4; ++e) rank += lanes_below(m[e], lane);
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (my_bit(m[e])) buf[rank++] = u[e];
    }
    s.cnt += total;
    return true;
}

// Row of len > 256 IDs streamed once; on return buf[0..f) is the sample in row order.  The IDs in
// front of the first 128-byte boundary go first (one per lane); from there on the row is read in
// blocks of 1 KB, one aligned 16-byte load per lane, so no two loads of a wave share a cache line,
// and the next block's load is in flight while the current block's keys are computed.
// first = row[lane] and blk0 = row_ahead(row, len, lane), loaded by the caller.
template <int CAP>
__device__ __forceinline__ void sample_long_row(const int32_t *__restrict__ row, int len, uint32_t first, int f, uint32_t lo, uint32_t hi, int lane,
                                                uint32_t *buf, const u32x4 &blk0)
{
    len = uni(len); f = uni(f); lo = uni(lo); hi = uni(hi);
    const int head = uni(row_head(row, len));
    const int32_t *p = row + head;
    const int rem = len - head;                                  // > 0: len > 256 and head < 32
    const int n_blocks = (rem + 255) >> 8;
    const uint32_t head_u = lane < head ? first : 0u;          // the head is part of the row's leading 64 IDs, which the caller holds
    // First attempt with a guessed cut.  Keys are uniform 32-bit words, so about lambda = f + 4 sqrt(f) + 8 of the
    // row's keys fall below lambda / len: streaming with that cut from the start collects the few IDs that can be in
    // the sample and skips the first cut and the prunes of the exact procedure.  The guess never changes the result:
    // every ID with a key up to the cut is kept, so if at least f turn up, the f smallest keys of the row are among
    // them; if fewer do (once in thousands of rows), the row is streamed again with the exact procedure.
    const float lambda = (float)f + 4.0f * __fsqrt_rn((float)f) + 8.0f;
    const bool can_guess = uni(lambda * 4.0f <= (float)len);
    const uint32_t guessed_cut = (uint32_t)(fminf(lambda / (float)len, 0.5f) * 4294967296.0f);
    Stream s{0, true, 0u};
    const int first_attempt = uni(can_guess ? 0 : 1);
  for (int attempt = first_attempt; attempt < 2; attempt = uni(attempt + 1)) {
    const bool guess = attempt == 0;
    s = guess ? Stream{0, false, guessed_cut} : Stream{0, true, 0u};
    u32x4 cur = attempt == first_attempt ? blk0 : load_block(p, rem, lane), nxt = {0u, 0u, 0u, 0u};
    int c0 = 0;
    const int count0 = rem < 256 ? rem : 256;
    if (!guess && head + count0 > f) {
        // The usual case: the head and the first block (up to 287 IDs, all in registers) already hold more
        // than f IDs.  Their f smallest keys give the first cut directly; only those f IDs enter the buffer.
        if (rem > 256) nxt = load_block(p + 256, rem - 256, lane);
        const uint32_t u[5] = {head_u, cur.x, cur.y, cur.z, cur.w};
        uint32_t k[5];
        unsigned long long vm[5];
        vm[0] = low_lanes(head);
#pragma unroll
        for (int e = 1; e < 5; ++e) vm[e] = block_lanes(count0, e - 1);
#pragma unroll
        for (int e = 0; e < 5; ++e) k[e] = key32(lo, hi, u[e]);
        s.cut = uni(kth_key_threshold<5>(k, vm, f, head + count0));
        s.open = false;
        s.cnt = f;
            unsigned long long m[5];
        int rank = 0;
#pragma unroll
        for (int e = 0; e < 5; ++e) m[e] = ballot64(k[e] <= s.cut) & vm[e];
        if (my_bit(m[0])) buf[lanes_below(m[0], lane)] = u[0];
        rank = __popcll(m[0]);
#pragma unroll
        for (int e = 1; e < 5; ++e) rank += lanes_below(m[e], lane);
#pragma unroll
        for (int e = 1; e < 5; ++e)
            if (my_bit(m[e])) buf[rank++] = u[e];
        cur = nxt;
        c0 = 1;
    } else if (guess && head > 0) {
        // under the guessed cut the head's candidates (at most 31, into an empty buffer) need no more than a rank
        const unsigned long long m = ballot64(key32(lo, hi, head_u) <= s.cut) & low_lanes(head);
        if (my_bit(m)) buf[lanes_below(m, lane)] = head_u;
        s.cnt = __popcll(m);
    } else if (head > 0) {
        const uint32_t u[4] = {head_u, 0u, 0u, 0u};
        const uint32_t k[4] = {key32(lo, hi, u[0]), 0u, 0u, 0u};
        const unsigned long long vm[4] = {low_lanes(head), 0ull, 0ull, 0ull};
        append_block<CAP>(u, k, vm, f, lo, hi, lane, buf, s);
    }
    if (guess && rem >= 256) {
        // The full blocks under the guessed cut, two in flight behind the one whose keys are computed: block j lives in
        // register quartet j mod 3 and the loop is unrolled by three, so no block is copied from one quartet to another
        // (a copy would have to wait for a load that has only just been issued).  Leaves at the first block it does not
        // take -- the partial last one, or a full one whose candidates do not fit -- which the loop below picks up.
        const int n_full = rem >> 8;
        auto load = [&](int j) {                                                                   // block j < n_blocks
            if (j < n_full) return *reinterpret_cast<const u32x4 *>(p + j * 256 + 4 * lane);
            return load_block(p + j * 256, rem - j * 256, lane);
        };
        u32x4 r0 = cur, r1 = {0u, 0u, 0u, 0u}, r2 = {0u, 0u, 0u, 0u};
        if (1 < n_blocks) r1 = load(1);
        int c = 0;
        for (;;) {
            if (c + 2 < n_blocks) r2 = load(c + 2);
            if (!stream_full_block_fast<CAP>(r0, lo, hi, lane, buf, s)) break;
            c = uni(c + 1);
            if (c >= n_full) break;
            if (c + 2 < n_blocks) r0 = load(c + 2);
            if (!stream_full_block_fast<CAP>(r1, lo, hi, lane, buf, s)) break;
            c = uni(c + 1);
            if (c >= n_full) break;
            if (c + 2 < n_blocks) r1 = load(c + 2);
            if (!stream_full_block_fast<CAP>(r2, lo, hi, lane, buf, s)) break;
            c = uni(c + 1);
            if (c >= n_full) break;
        }
        c0 = c;
        const int which = c % 3;
        cur = which == 0 ? r0 : which == 1 ? r1 : r2;            // (unused when c == n_blocks)
    }
    for (int c = uni(c0); c < n_blocks; c = uni(c + 1)) {
        const int left = uni(rem - c * 256);                     // IDs left, this block included
        if (left > 256) nxt = load_block(p + (c + 1) * 256, left - 256, lane);
        if (left >= 256) {
            if (guess) stream_block<CAP, true, false>(cur, 256, f, lo, hi, lane, buf, s);
            else stream_block<CAP, true, true>(cur, 256, f, lo, hi, lane, buf, s);
        } else stream_block<CAP, false>(cur, left, f, lo, hi, lane, buf, s);
        cur = nxt;
    }
    __syncthreads();
    if (s.cnt >= f) break;                                       // (always, in the exact attempt: len > f)
  }
    if (s.cnt > f) {
        const uint32_t upper = s.open ? 0xFFFFFFFFu : s.cut;
        if (CAP > 64 && s.cnt <= 64) (void)prune_buffer<64>(buf, s.cnt, f, lo, hi, lane, upper);     // the usual case after a guessed cut: one ID per lane
        else (void)prune_buffer<CAP>(buf, s.cnt, f, lo, hi, lane, upper);
    }
}

// SAMPLE of a row of len > f IDs into out (row order), marking the sampled IDs as MARK says.
// `first` holds row[lane] for lane < len; ahead = row_ahead(row, len, lane) when len > 64 (unused otherwise).
template <int CAP, int MARK>
__device__ __forceinline__ void sample_row(const int32_t *__restrict__ row, int len, uint32_t first, const u32x4 &ahead, int f, uint32_t lo, uint32_t hi,
                                           int lane, uint32_t *buf, int32_t *__restrict__ out, const ReachedOfBatch &reached_b)
{
    if (len <= 64) {
        const uint32_t u[1] = {first};
        sample_registers<1, MARK>(u, len, f, lo, hi, lane, buf, out, reached_b);
    } else if (len <= 256) {
        const uint32_t u[4] = {first, ahead.x, ahead.y, ahead.z};
        sample_registers<4, MARK>(u, len, f, lo, hi, lane, buf, out, reached_b);
    } else {
        sample_long_row<CAP>(row, len, first, f, lo, hi, lane, buf, ahead);
        for (int j = lane; j < f; j += 64) {
            const uint32_t u = buf[j];
            out[j] = (int32_t)u;
            mark_reached<MARK>(reached_b, u);
        }
        __syncthreads();      // the buffer is reused by the wave's next row
    }
}

// ---------------------------------------------------------------- rows of up to SHORT_ROW IDs, four at a time
// A wave that samples one short row at a time spends its time waiting: a row of 30 IDs is one load and a few dozen
// instructions, and the next row's load cannot start much earlier than this row's ends.  Here a wave takes 64
// consecutive frontier nodes, lists the ones with 1 .. SHORT_ROW neighbours -- shortest first, so that rows of a
// round are of a kind -- and samples four of them at once, one per row of sixteen lanes (lane l of a row holds IDs
// l, l + 16, l + 32, l + 48 of it), with the next four rows' IDs already on their way.  The f smallest keys of a
// row: for rows of up to 16 IDs (one key per lane) by rank -- every key is compared with every other key of its row as
// the register rotates through the sixteen lanes (DPP row rotation, no LDS), and the IDs whose key has fewer than f
// smaller keys are the sample; for longer rows by the same bisection on the key value as everywhere else, the four
// rows searching side by side, each lane counting its own row's sixteen bits of every lane mask.  Output positions
// come from the lane masks, in row order, as in the other kernels.
struct ShortRec {
    int64_t row_begin, out;
    uint64_t state;
    int32_t deg;
    uint32_t batch;
};

template <int R> __device__ __forceinline__ uint32_t rotate16(uint32_t x)      // the value R lanes away within the lane's row of sixteen
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x120 + R, 0xF, 0xF, false);
}

// The number of keys of the lane's row of sixteen lanes (one key per lane) that are smaller than this lane's.
__device__ __forceinline__ int count_smaller16(uint32_t k)
{
    int cnt = 0;
#define RG_ROT(R) cnt += rotate16<R>(k) < k ? 1 : 0;
    RG_ROT(1) RG_ROT(2) RG_ROT(3) RG_ROT(4) RG_ROT(5) RG_ROT(6) RG_ROT(7) RG_ROT(8)
    RG_ROT(9) RG_ROT(10) RG_ROT(11) RG_ROT(12) RG_ROT(13) RG_ROT(14) RG_ROT(15)
#undef RG_ROT
    return cnt;
}

// This lane's row's sixteen bits of a lane mask, counted.
__device__ __forceinline__ int popc_of_my_row(unsigned long long m, int lane) { return __popc((uint32_t)(m >> (lane & 48)) & 0xFFFFu); }

// For each row of sixteen lanes on its own: the largest key value `cut` such that exactly f of the row's keys do not
// exceed it.  k[e], e < E: the row's keys, a missing one stands as 0xFFFFFFFF; deg (> f in the rows that search, same
// in all lanes of a row): how many there are; rows with searching == false ride along and get an arbitrary answer.
// Bit by bit from the top, as kth_key_threshold does for a whole wave: the f-th smallest key stays inside
// [lo, lo + 2^(bit+1)), and a row is done as soon as exactly f keys lie below the bracket's upper end -- for keys
// spread over 32 bits after about log2(deg) + 2 steps; the loop ends when every row is done.
template <int E>
__device__ __forceinline__ uint32_t kth_key_threshold_rows(const uint32_t (&k)[4], int f, int deg, bool searching, int lane)
{
    uint32_t lo = 0, cut = 0xFFFFFFFFu;
    int below_hi = deg;
    bool done = !searching;
    for (int bit = 31; bit >= 0; --bit) {
        if (ballot64(!done) == 0ull) break;
        const uint32_t t = lo | (1u << bit);
        int c = 0;
#pragma unroll
        for (int e = 0; e < E; ++e) c += popc_of_my_row(ballot64(k[e] < t), lane);
        if (!done) {
            if (c >= f) below_hi = c; else lo = t;
            cut = lo | ((1u << bit) - 1u);
            done = below_hi == f;
        }
    }
    return cut;
}

// The listed short rows (recs[0 .. count), shortest first; LDS) sampled four per round.  All 64 lanes call it.
template <int MARK>
__device__ __forceinline__ void sample_short_rows(const ShortRec *recs, int count, const int32_t *__restrict__ indices, int f,
                                                  int32_t *__restrict__ samp_nbr, const ReachedMaps &reached, int lane)
{
    const int l16 = lane & 15, sg = lane >> 4;
    const int n_it = (count + 3) >> 2;
    // this lane's row of the round, and its IDs (0 where the row has none)
    auto fetch = [&](int it, ShortRec &r, uint32_t (&u)[4]) {
        const int slot = it * 4 + sg;
        r = slot < count ? recs[slot] : ShortRec{0, 0, 0, 0, 0};
        const int32_t *row = indices + r.row_begin;
#pragma unroll
        for (int e = 0; e < 4; ++e) u[e] = l16 + 16 * e < r.deg ? (uint32_t)row[l16 + 16 * e] : 0u;
    };
    ShortRec r, r_next;
    uint32_t u[4], u_next[4];
    fetch(0, r, u);
    for (int it = 0; it < n_it; ++it) {
        if (it + 1 < n_it) fetch(it + 1, r_next, u_next);
        const int deg = r.deg;
        bool sel[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) sel[e] = l16 + 16 * e < deg;
        const bool searching = deg > f;
        if (ballot64(searching) != 0ull) {                       // some row of the round is longer than the fan-out
            const uint32_t slo = (uint32_t)r.state, shi = (uint32_t)(r.state >> 32);
            uint32_t k[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) k[e] = sel[e] ? key32(slo, shi, u[e]) : 0xFFFFFFFFu;     // (a missing key's stand-in is never counted as smaller than anything)
            if (ballot64(searching && deg > 16) == 0ull) {       // one key per lane: by rank
                const int smaller = count_smaller16(k[0]);
                if (searching) sel[0] = sel[0] && smaller < f;
            } else {
                uint32_t cut;
                if (ballot64(searching && deg > 48) != 0ull) cut = kth_key_threshold_rows<4>(k, f, deg, searching, lane);
                else if (ballot64(searching && deg > 32) != 0ull) cut = kth_key_threshold_rows<3>(k, f, deg, searching, lane);
                else cut = kth_key_threshold_rows<2>(k, f, deg, searching, lane);
                if (searching) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) sel[e] = sel[e] && k[e] <= cut;
                }
            }
        }
        // row order is ID 0 .. 15 (e = 0), 16 .. 31 (e = 1), ...: a selected ID's place is the number of selected IDs before it
        const ReachedOfBatch reached_b = reached_of<MARK>(reached, r.batch);
        int32_t *out = samp_nbr + r.out;
        int base = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint32_t m16 = (uint32_t)(ballot64(sel[e]) >> (lane & 48)) & 0xFFFFu;       // the selected lanes of this lane's row
            if (sel[e]) {
                out[base + __popc(m16 & ((1u << l16) - 1u))] = (int32_t)u[e];
                mark_reached<MARK>(reached_b, u[e]);
            }
            base += __popc(m16);
        }
        r = r_next;
#pragma unroll
        for (int e = 0; e < 4; ++e) u[e] = u_next[e];
    }
}

// Where a lane's short row goes in the list: shortest rows first, by the number of IDs per lane ((deg - 1) / 16), lane
// order within a kind.  mine: this lane has a row of 1 .. SHORT_ROW IDs.  All 64 lanes call it.
__device__ __forceinline__ int short_row_slot(bool mine, int deg, int lane)
{
    const int kind = mine ? (deg - 1) >> 4 : -1;
    int at = 0;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        const unsigned long long m = ballot64(kind == c);
        if (c < kind) at += __popcll(m);
        else if (c == kind) at += lanes_below(m, lane);
    }
    return at;
}

// Per tile job j: the frontier position i whose row it belongs to (tile_off[i] <= j < tile_off[i + 1]), where its piece of
// the row starts in `indices`, how long it is (near-equal pieces, each longer than 2 * RG_MAX_FANOUT) and the node's
// stream S_v.  Written by the nodes that have tiles, so that a wave finds everything about its piece in one round of
// loads instead of a search through tile_off and a second round for the node's record.
struct TileRecs {
    int64_t *node;
    int64_t *begin;
    int32_t *len;
    uint64_t *state;
};
// One thread per tile job: its node is the frontier position i with tile_off[i] <= j < tile_off[i + 1].
__global__ void tile_records_kernel(const int64_t *__restrict__ tile_off, const int64_t *__restrict__ row_begin, const int32_t *__restrict__ deg,
                                    const uint64_t *__restrict__ state, int64_t n, int64_t n_tiles, TileRecs r)
{
    const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= n_tiles) return;
    int64_t lo = 0, hi = n;                    // invariant: tile_off[lo] <= j < tile_off[hi]   (tile_off[0] = 0, tile_off[n] = n_tiles)
    while (hi - lo > 1) {
        const int64_t mid = (lo + hi) >> 1;
        if (tile_off[mid] <= j) lo = mid; else hi = mid;
    }
    const int64_t i = lo;
    const int64_t d = deg[i];
    const int64_t T = tiles_of(d);            // the count tile_off was summed from
    const int64_t t = j - tile_off[i];
    const int64_t first_pos = t * d / T, last_pos = (t + 1) * d / T;
    r.node[j] = i;
    r.begin[j] = row_begin[i] + first_pos;
    r.len[j] = (int32_t)(last_pos - first_pos);
    r.state[j] = state[i];
}

// Tile jobs grouped by the piece of adjacency they read.  A hub's row is in the frontier of most batches, so the same
// piece is read once per batch; in frontier order those reads lie a whole batch apart and every one of them comes
// from HBM.  Handed out in an order in which the jobs of a piece follow each other, they run at about the same time
// and all but the first are served by the caches.  Grouping, not sorting: a job's bucket is a hash of its piece's
// start (pieces are thousands of IDs apart), jobs are counted per bucket, the counts prefix-summed, and every job
// takes the next place of its bucket (in whatever order the adds arrive: a job's result goes to the job's own
// place, so the order changes nothing but the timing).
__device__ __forceinline__ uint32_t tile_bucket(int64_t begin, int bits)
{
    return ((uint32_t)((uint64_t)begin >> 12) * 0x9E3779B1u) >> (32 - bits);
}
// rank[j] = how many jobs of j's bucket came before it (by arrival); cnt[b] ends as the bucket's size
__global__ void tile_bucket_count_kernel(const int64_t *__restrict__ begin, int64_t n_tiles, int bits, int32_t *__restrict__ cnt, int32_t *__restrict__ rank)
{
    const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j < n_tiles) rank[j] = atomicAdd(&cnt[tile_bucket(begin[j], bits)], 1);
}
__global__ void tile_bucket_place_kernel(const int64_t *__restrict__ begin, int64_t n_tiles, int bits, const int64_t *__restrict__ off,
                                         const int32_t *__restrict__ rank, int32_t *__restrict__ order)
{
    const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j < n_tiles) order[off[tile_bucket(begin[j], bits)] + rank[j]] = (int32_t)j;
}

struct HopArgs {
    const int32_t *indices;
    const int32_t *frontier; int64_t n_frontier;
    int64_t n_full_groups, n_units;                                    // set by launch_hop: see there
    int min_deg;                                                       // rows of up to this many IDs are not sampled one per wave ...
    int short_inline;                                                  // ... but four at a time: 1 = by sample_kernel<.., true>, a group's short rows first; 0 = by sample_short_kernel
    NodeRecs rec;
    uint32_t fanout;
    const int64_t *samp_off; int32_t *samp_nbr;
    const int64_t *tile_off; TileRecs tile; int64_t n_tiles; int32_t *tile_out;      // tile j writes tile_out[j * fanout ..)
    int merge_span;                                                    // tiles a wave of sample_merge_kernel looks at per round
    const int32_t *tile_order;                                         // the k-th tile job to hand out, or NULL: job k
    ReachedMaps reached;
    unsigned long long *next_work;                                     // work items are handed out in order through this counter
};

// The next unclaimed work item (lane 0 asks, every lane gets the answer).
__device__ __forceinline__ int64_t grab_work(unsigned long long *counter, int lane)
{
    unsigned long long v = 0;
    if (lane == 0) v = atomicAdd(counter, 1ull);
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)v);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(v >> 32));
    return (int64_t)(((uint64_t)hi << 32) | lo);
}

// The work of a hop: n_tiles tiles of long rows (done first, so the longest-running work starts first) and the groups
// of 64 consecutive frontier nodes.
// SHORT_INLINE: each group's rows of up to SHORT_ROW IDs are sampled four at a time before its other rows (an
// instantiation of its own: the code costs the streaming loop a few registers).
template <int CAP, int MARK, bool SHORT_INLINE>
__global__ void __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(CAP <= 256 ? 7 : 1))) sample_kernel(HopArgs a)
{
    __shared__ uint32_t buf[CAP];
    __shared__ ShortRec short_recs[SHORT_INLINE ? 64 : 1];
    const int lane = threadIdx.x;
    const int f = (int)a.fanout;
    // Tiles first, dealt out in turn (workgroup k takes tiles k, k + grid, ...): they are all of about the same
    // length, the whole grid is resident (see launch_hop), and with the next tile known in advance its record is
    // fetched while the current one is streamed -- no wave waits for a counter or a record between tiles.
    {
        // Workgroup g runs on XCD g mod 8 (workgroups are dealt out to the XCDs in turn), and every XCD has an L2 of its
        // own: in each round XCD x takes a contiguous eighth of the round's jobs, so the jobs of a piece -- neighbours
        // in the grouped order -- meet in one L2 instead of being spread over all eight.
        int64_t k = blockIdx.x;
        if (a.tile_order && (gridDim.x & 7u) == 0) k = (int64_t)(blockIdx.x & 7u) * (gridDim.x >> 3) + (blockIdx.x >> 3);
        int64_t w = 0, nb = 0; int nl = 0; uint64_t nS = 0;
        if (k < a.n_tiles) { w = a.tile_order ? a.tile_order[k] : k; nb = a.tile.begin[w]; nl = a.tile.len[w]; nS = a.tile.state[w]; }
        while (k < a.n_tiles) {
            const int32_t *row = a.indices + nb;
            const int len = nl;
            const uint64_t S = nS;
            const int64_t w_now = w;
            const uint32_t first = (uint32_t)row[lane];
            const u32x4 ahead = row_ahead(row, len, lane);
            k += gridDim.x;
            if (k < a.n_tiles) { w = a.tile_order ? a.tile_order[k] : k; nb = a.tile.begin[w]; nl = a.tile.len[w]; nS = a.tile.state[w]; }
            sample_row<CAP, MARK_NONE>(row, len, first, ahead, f, (uint32_t)S, (uint32_t)(S >> 32), lane, buf, a.tile_out + w_now * f,
                                       ReachedOfBatch{nullptr, nullptr});
        }
    }
    // Then the groups of 64 consecutive frontier nodes, taken as waves become free, so that uneven rows do not leave
    // part of the chip idle at the end -- and for the same reason the launch's last nodes come in groups of 16 (a group
    // of 64 nodes with long rows is a sizeable part of a launch's whole duration); every wave leaves once the counter
    // has passed the last group.
    for (int64_t w = grab_work(a.next_work, lane); w < a.n_units; w = grab_work(a.next_work, lane)) {
        const bool full = w < a.n_full_groups;                  // 64 nodes, or 16 of the launch's last nodes
        const int64_t i_lane = (full ? w << 6 : (a.n_full_groups << 6) + ((w - a.n_full_groups) << 4)) + lane;
        const bool in = (full || lane < 16) && i_lane < a.n_frontier;
        const int64_t rb_lane = in ? a.rec.row_begin[i_lane] : 0;
        const int deg_lane = in ? a.rec.deg[i_lane] : 0;
        const uint32_t b_lane = in ? a.rec.batch[i_lane] : 0u;
        const int64_t S_lane = in ? (int64_t)a.rec.state[i_lane] : 0;
        const int64_t out_lane = in ? a.samp_off[i_lane] : 0;
        if (SHORT_INLINE) {
            // the group's rows of up to SHORT_ROW IDs first, four at a time (their marks and scattered little reads then
            // run beside the streaming of the other waves' long rows)
            // A row of at most TINY_ROW IDs that is no longer than the fan-out is its own sample: its node's lane copies
            // and marks it, 64 rows at a time, four IDs of each in flight (on a graph whose typical row has two or three
            // IDs these are nine rows in ten, and four at a time is sixteen rounds for what is one or two here).
            const bool tiny = in && deg_lane > 0 && deg_lane <= f && deg_lane <= TINY_ROW;
            if (ballot64(tiny) != 0ull) {
                const int32_t *row = a.indices + rb_lane;
                int32_t *out = a.samp_nbr + out_lane;
                const ReachedOfBatch reached_b = reached_of<MARK>(a.reached, b_lane);
                for (int j0 = 0; ballot64(tiny && j0 < deg_lane) != 0ull; j0 += 4) {
                    int32_t u[4] = {0, 0, 0, 0};
#pragma unroll
                    for (int k = 0; k < 4; ++k)
                        if (tiny && j0 + k < deg_lane) u[k] = row[j0 + k];
#pragma unroll
                    for (int k = 0; k < 4; ++k)
                        if (tiny && j0 + k < deg_lane) { out[j0 + k] = u[k]; mark_reached<MARK>(reached_b, (uint32_t)u[k]); }
                }
            }
            const bool mine = in && !tiny && deg_lane > 0 && deg_lane <= SHORT_ROW;
            const int count = __popcll(ballot64(mine));
            if (count != 0) {
                const int at = short_row_slot(mine, deg_lane, lane);
                __syncthreads();
                if (mine) short_recs[at] = ShortRec{rb_lane, out_lane, (uint64_t)S_lane, deg_lane, b_lane};
                __syncthreads();
                sample_short_rows<MARK>(short_recs, count, a.indices, f, a.samp_nbr, a.reached, lane);
            }
        }
        unsigned long long todo = ballot64(deg_lane > a.min_deg && deg_lane <= BIG_ROW);
        if (todo == 0ull) continue;
        // the first node's leading 64 IDs; from then on the next node's are fetched while the current one is sampled
        int l = __builtin_amdgcn_readfirstlane(__ffsll((long long)todo) - 1);
        int64_t rb = bcast64(rb_lane, l);
        int deg = __builtin_amdgcn_readlane(deg_lane, l);
        uint32_t first = lane < deg ? (uint32_t)a.indices[rb + lane] : 0u;
        u32x4 ahead = {0u, 0u, 0u, 0u};
        if (deg > 64 && deg > f) ahead = row_ahead(a.indices + rb, deg, lane);
        while (todo != 0ull) {
            todo &= todo - 1ull;
            const int cl = l, cdeg = deg;
            const int64_t crb = rb;
            const uint32_t cfirst = first;
            const u32x4 cahead = ahead;
            if (todo != 0ull) {
                l = __builtin_amdgcn_readfirstlane(__ffsll((long long)todo) - 1);
                rb = bcast64(rb_lane, l);
                deg = __builtin_amdgcn_readlane(deg_lane, l);
                first = lane < deg ? (uint32_t)a.indices[rb + lane] : 0u;
                if (deg > 64 && deg > f) ahead = row_ahead(a.indices + rb, deg, lane);
            }
            const uint32_t b = (uint32_t)__builtin_amdgcn_readlane((int)b_lane, cl);
            const ReachedOfBatch reached_b = reached_of<MARK>(a.reached, b);
            const int32_t *row = a.indices + crb;
            int32_t *out = a.samp_nbr + bcast64(out_lane, cl);
            if (cdeg <= f) {                  // the whole row is the sample
                if (lane < cdeg) { out[lane] = (int32_t)cfirst; mark_reached<MARK>(reached_b, cfirst); }
                for (int j = 64 + lane; j < cdeg; j += 64) {
                    const int32_t u = row[j];
                    out[j] = u;
                    mark_reached<MARK>(reached_b, (uint32_t)u);
                }
            } else {
                const uint64_t S = (uint64_t)bcast64(S_lane, cl);
                sample_row<CAP, MARK>(row, cdeg, cfirst, cahead, f, (uint32_t)S, (uint32_t)(S >> 32), lane, buf, out, reached_b);
            }
        }
    }
}

// A long row's concatenated tile results (T * f IDs, row order, all distinct) are sampled into the final output by
// the wave that finds the row's first tile.  A wave looks at 64 tiles at once, a lane each (hub rows have hundreds of
// tiles, so first tiles are few: walking the tiles one per wave-iteration cost two dependent loads per tile), and
// then takes the rows whose first tiles it found one after the other.  a.merge_span <= 64 tiles per look: fewer
// where the launch has too few tiles to give every wave 64 of them (rows of two or three tiles would queue up).
template <int CAP, int MARK>
__global__ void __launch_bounds__(64) sample_merge_kernel(HopArgs a)
{
    __shared__ uint32_t buf[CAP];
    const int lane = threadIdx.x;
    const int f = (int)a.fanout;
    const int span = a.merge_span;
    for (int64_t base = (int64_t)blockIdx.x * span; base < a.n_tiles; base += (int64_t)gridDim.x * span) {
        int64_t i_lane = -1;
        if (lane < span && base + lane < a.n_tiles) {
            const int64_t i = a.tile.node[base + lane];
            if (a.tile_off[i] == base + lane) i_lane = i;
        }
        unsigned long long firsts = ballot64(i_lane >= 0);
        while (firsts != 0ull) {
            const int l = __builtin_amdgcn_readfirstlane(__ffsll((long long)firsts) - 1);
            firsts &= firsts - 1ull;
            const int64_t i = bcast64(i_lane, l);
            const int64_t w = base + l;
            const int64_t T = a.tile_off[i + 1] - w;
            const uint32_t b = a.rec.batch[i];
            const uint64_t S = a.rec.state[i];
            const int32_t *row = a.tile_out + w * f;
            const int len = (int)(T * f);
            u32x4 ahead = {0u, 0u, 0u, 0u};
            if (len > 64) ahead = row_ahead(row, len, lane);
            sample_row<CAP, MARK>(row, len, lane < len ? (uint32_t)row[lane] : 0u, ahead, f, (uint32_t)S, (uint32_t)(S >> 32), lane, buf,
                                  a.samp_nbr + a.samp_off[i], reached_of<MARK>(a.reached, b));
        }
    }
}


struct ShortArgs {
    const int32_t *indices;
    int64_t n_frontier;
    NodeRecs rec;
    uint32_t fanout;
    const int64_t *samp_off; int32_t *samp_nbr;
    ReachedMaps reached;
};

template <int MARK>
__global__ void __launch_bounds__(64) sample_short_kernel(ShortArgs a)
{
    __shared__ ShortRec recs[64];
    const int lane = threadIdx.x;
    const int64_t n_groups = (a.n_frontier + 63) >> 6;
    for (int64_t w = blockIdx.x; w < n_groups; w += gridDim.x) {
        const int64_t i_lane = (w << 6) + lane;
        const int deg_lane = i_lane < a.n_frontier ? a.rec.deg[i_lane] : 0;
        const bool mine = deg_lane > 0 && deg_lane <= SHORT_ROW;
        const int count = __popcll(ballot64(mine));
        if (count == 0) continue;
        const int at = short_row_slot(mine, deg_lane, lane);
        __syncthreads();                                            // the previous group's records have been read by every lane
        if (mine) recs[at] = ShortRec{a.rec.row_begin[i_lane], a.samp_off[i_lane], a.rec.state[i_lane], deg_lane, a.rec.batch[i_lane]};
        __syncthreads();
        sample_short_rows<MARK>(recs, count, a.indices, (int)a.fanout, a.samp_nbr, a.reached, lane);
    }
}

template <int MARK>
static rg_status launch_short(const ShortArgs &a, int n_cu, hipStream_t st)
{
    const int64_t n_groups = (a.n_frontier + 63) >> 6;
    const unsigned grid = (unsigned)std::max<int64_t>(1, std::min<int64_t>(n_groups, (int64_t)n_cu * 32));
    hipLaunchKernelGGL((sample_short_kernel<MARK>), dim3(grid), dim3(64), 0, st, a);
    return RG_OK;
}

// Every workgroup of the sampling launch must be resident from the start (tiles are dealt out by workgroup index), so
// the grid is what the chip holds of this kernel, or the amount of work if that is less.
template <int CAP, int MARK>
static rg_status launch_hop(const HopArgs &args, int n_cu, unsigned merge_grid, bool fine_tail, bool fine_if_few, hipStream_t st)
{
    HopArgs a = args;
    static std::atomic<int> asked[2] = {{0}, {0}};      // the same answer every time; asked once (schedules may be built from several threads)
    const int which = a.short_inline ? 1 : 0;
    int per_cu = asked[which].load(std::memory_order_relaxed);
    if (per_cu == 0) {
        int v = 0;
        if (which) RG_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&v, sample_kernel<CAP, MARK, true>, 64, 0));
        else RG_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&v, sample_kernel<CAP, MARK, false>, 64, 0));
        per_cu = v > 0 ? v : 1;
        asked[which].store(per_cu, std::memory_order_relaxed);
    }
    // Groups of 64 nodes, except that with fine_tail the last 128 nodes per resident wave (and always what is left of
    // the frontier after the last whole group) are handed out 16 at a time.
    const int64_t resident = (int64_t)n_cu * per_cu;
    int64_t tail_nodes = fine_tail ? std::min<int64_t>(a.n_frontier, resident * 128) : 0;
    if (fine_if_few && a.n_frontier < resident * 64) tail_nodes = a.n_frontier;       // fewer groups of 64 than waves: sixteens throughout
    a.n_full_groups = (a.n_frontier - tail_nodes) / 64;
    a.n_units = a.n_full_groups + (a.n_frontier - a.n_full_groups * 64 + 15) / 16;
    const int64_t n_work = a.n_tiles + a.n_units;
    const unsigned grid = (unsigned)std::max<int64_t>(1, std::min<int64_t>(n_work, resident));
    if (which) hipLaunchKernelGGL((sample_kernel<CAP, MARK, true>), dim3(grid), dim3(64), 0, st, a);
    else hipLaunchKernelGGL((sample_kernel<CAP, MARK, false>), dim3(grid), dim3(64), 0, st, a);
    if (a.n_tiles > 0) hipLaunchKernelGGL((sample_merge_kernel<CAP, MARK>), dim3(merge_grid), dim3(64), 0, st, a);
    return RG_OK;
}

// The O(f) sampler: one lane per sampled edge.  A node with deg <= f copies its row; otherwise lane t reads the
// row at its drawn position (rg_device.h) and nothing else of the row.  Lanes of a workgroup are dealt to
// (node, draw) pairs: 256 / f nodes per round when f < 256, one node per round otherwise.
constexpr int POS_THREADS = 256;
template <int MARK>
__global__ void __launch_bounds__(POS_THREADS) sample_positions_kernel(const int32_t *__restrict__ indices, NodeRecs rec, int64_t n_cur, uint32_t f,
                                                                       const int64_t *__restrict__ samp_off, int32_t *__restrict__ samp_nbr,
                                                                       ReachedMaps reached)
{
    const uint32_t per_round = f >= POS_THREADS ? 1u : POS_THREADS / f;       // nodes per workgroup round
    const uint32_t sub = f >= POS_THREADS ? 0u : threadIdx.x / f;              // this lane's node within the round
    const uint32_t t0 = f >= POS_THREADS ? threadIdx.x : threadIdx.x - sub * f;
    const uint32_t step = f >= POS_THREADS ? POS_THREADS : f;                  // a lane's next draw of the same node
    if (sub >= per_round) return;
    for (int64_t i = (int64_t)blockIdx.x * per_round + sub; i < n_cur; i += (int64_t)gridDim.x * per_round) {
        const uint32_t deg = (uint32_t)rec.deg[i];
        const uint32_t cnt = deg < f ? deg : f;
        if (t0 >= cnt) continue;
        const int32_t *row = indices + rec.row_begin[i];
        const uint64_t S = rec.state[i];
        int32_t *out = samp_nbr + samp_off[i];
        const ReachedOfBatch reached_b = reached_of<MARK>(reached, rec.batch[i]);
        for (uint32_t t = t0; t < cnt; t += step) {
            const uint32_t p = deg <= f ? t : draw_position(deg, t, S);
            const int32_t u = row[p];
            out[t] = u;
            mark_reached<MARK>(reached_b, (uint32_t)u);
        }
    }
}

// Samples hop `hop` of every batch: fills cur.samp_off / samp_nbr / n_samples and marks the reached-ID bitmaps.
// also_read_dev (or NULL): one more device value copied to *also_read_host behind the hop's own readback; if it
// comes back non-zero the hop stops there (the caller is about to refuse its input).
// Where `maps` allows the reached map's byte form, the hop marks into whichever form suits it (see below; the byte
// map is allocated, clear, by the first hop that wants it) and *marked_bytes says which, so that the frontier pass
// reads the right one.
rg_status sample_hop(const rg_graph *g, HopData &cur, uint32_t beta, const uint64_t *batch_seed, uint32_t hop, uint32_t fanout,
                     uint32_t sampler, ReachedForms &maps, int prefer_bytes, bool *marked_bytes, Arena &keep, Arena &tmp, int n_cu,
                     hipStream_t st, const unsigned long long *also_read_dev, unsigned long long *also_read_host)
{
    const int64_t n_cur = cur.off_host[beta];
    int32_t *cnt = nullptr, *tiles = nullptr;
    int64_t *tile_off = nullptr;
    NodeRecs rec{nullptr, nullptr, nullptr, nullptr};
    RG_TRY(tmp.dev_n<int32_t>((uint64_t)n_cur, &cnt));
    RG_TRY(tmp.dev_n<int32_t>((uint64_t)n_cur, &tiles));
    RG_TRY(tmp.dev_n<int64_t>((uint64_t)n_cur + 1, &tile_off));
    RG_TRY(tmp.dev_n<int64_t>((uint64_t)n_cur, &rec.row_begin));
    RG_TRY(tmp.dev_n<int32_t>((uint64_t)n_cur, &rec.deg));
    RG_TRY(tmp.dev_n<uint32_t>((uint64_t)n_cur, &rec.batch));
    RG_TRY(tmp.dev_n<uint64_t>((uint64_t)n_cur, &rec.state));
    RG_TRY(keep.dev_n<int64_t>((uint64_t)n_cur + 1, &cur.samp_off));
    unsigned long long sums[DEG_SUMS] = {0, 0, 0, 0}, *sum_deg_dev = nullptr;       // see node_records_kernel
    unsigned long long sum_parts[DEG_SUMS * DEG_SUM_SLOTS];
    RG_TRY(tmp.dev_n<unsigned long long>(DEG_SUMS * DEG_SUM_SLOTS, &sum_deg_dev));
    RG_HIP(hipMemsetAsync(sum_deg_dev, 0, sizeof(sum_parts), st));
    {
        ScopedTimer tm(KG_OFFSETS, st);
        hipLaunchKernelGGL(node_records_kernel, dim3((unsigned)std::max<int64_t>(1, std::min<int64_t>((n_cur + 255) / 256, (int64_t)n_cu * 64))), dim3(256), 0, st, g->indptr, cur.ids, n_cur, cur.off_dev, beta,
                           batch_seed, hop, fanout, rec, cnt, tiles, (int64_t)g->n_nodes, sum_deg_dev);
        RG_TRY(scan_i32_to_i64(cnt, cur.samp_off, n_cur, tmp, st));
        RG_TRY(scan_i32_to_i64(tiles, tile_off, n_cur, tmp, st));
    }
    int64_t n_tiles = 0;
    // (the byte-marking kernels exist for fan-outs up to 192: the two smaller candidate buffers)
    const bool can_bytes = maps.bytes_allowed && (sampler == RG_SAMPLER_POSITIONS || fanout + 64 <= 256);
    {
        Readback rb(st);
        RG_TRY(rb.add(sum_parts, sum_deg_dev, sizeof(sum_parts)));
        RG_TRY(rb.add(&cur.n_samples, cur.samp_off + n_cur, sizeof(int64_t)));
        RG_TRY(rb.add(&n_tiles, tile_off + n_cur, sizeof(int64_t)));
        if (also_read_dev) RG_TRY(rb.add(also_read_host, also_read_dev, sizeof(unsigned long long)));     // a value the caller wants behind the same wait
        RG_TRY(rb.wait());
        for (int k = 0; k < DEG_SUM_SLOTS; ++k)
            for (int q = 0; q < DEG_SUMS; ++q) sums[q] += sum_parts[DEG_SUMS * k + q];
        if (also_read_dev && *also_read_host != 0) return RG_OK;        // the caller refuses the build: nothing more to launch
    }
    // Which form of the reached map this hop marks.  A byte store is several times cheaper than an atomic OR, but the
    // byte map is 8 times the size and its scattered stores reach memory as whole lines; that pays where marks are a
    // large part of the hop's traffic (rows mostly no longer than the fan-out: one mark per ID read), and costs a
    // little where long rows are scanned for a few samples (measured: at one mark per 20 IDs read nothing is gained,
    // at one per 10 the hop is a quarter faster).  Threshold: one mark per 14 IDs read.
    const unsigned long long sum_deg = sums[0];
    const bool use_bytes = can_bytes && (prefer_bytes >= 0 ? prefer_bytes != 0 : (unsigned long long)cur.n_samples * 14ull >= sum_deg);
    if (use_bytes && !maps.bytes) {
        const uint64_t map_bytes = maps.words_per_batch * 32 * (uint64_t)beta;
        RG_TRY(tmp.dev_zeroed(map_bytes, (void **)&maps.bytes, st));       // (the caller hands it back as all-zero: the frontier passes clear what a hop marks)
    }
    *marked_bytes = use_bytes;
    // A hop that marks many times more IDs than the maps have groups reaches nearly every group: the per-mark flag
    // store (a third of the hop's scattered stores) is replaced by setting every flag once.
    const uint64_t flag_bytes = maps.words_per_batch / 8 * (uint64_t)beta;
    const bool all_flags = sampler == RG_SAMPLER_KEYS && fanout > 0 && fanout + 64 <= 256 && (uint64_t)cur.n_samples >= 16 * flag_bytes;
    if (all_flags) RG_HIP(hipMemsetAsync(maps.flags, 1, flag_bytes, st));
    const ReachedMaps reached{use_bytes ? (void *)maps.bytes : (void *)maps.words, maps.flags, maps.words_per_batch, (!use_bytes && maps.paired) ? 1u : 0u};
    tmp.free_one(cnt);
    tmp.free_one(tiles);
    RG_TRY(keep.dev_n<int32_t>((uint64_t)cur.n_samples, &cur.samp_nbr));
    if (sampler == RG_SAMPLER_POSITIONS) {
        if (fanout > 0 && n_cur > 0) {
            ScopedTimer tm(KG_SAMPLER, st);
            const int64_t per_round = fanout >= (uint32_t)POS_THREADS ? 1 : POS_THREADS / fanout;
            const unsigned grid = (unsigned)std::max<int64_t>(1, std::min<int64_t>((n_cur + per_round - 1) / per_round, (int64_t)n_cu * 64));
            if (use_bytes)
                hipLaunchKernelGGL(sample_positions_kernel<MARK_BYTES>, dim3(grid), dim3(POS_THREADS), 0, st, g->indices, rec, n_cur, fanout, cur.samp_off,
                                   cur.samp_nbr, reached);
            else
                hipLaunchKernelGGL(sample_positions_kernel<MARK_BITS>, dim3(grid), dim3(POS_THREADS), 0, st, g->indices, rec, n_cur, fanout, cur.samp_off,
                                   cur.samp_nbr, reached);
            RG_HIP(hipGetLastError());
        }
        return RG_OK;
    }
    if (fanout == 0) n_tiles = 0;             // nothing is drawn; every sample is empty
    int32_t *tile_out = nullptr;
    TileRecs tile{nullptr, nullptr, nullptr, nullptr};
    RG_TRY(tmp.dev_n<int32_t>((uint64_t)n_tiles * fanout, &tile_out));
    RG_TRY(tmp.dev_n<int64_t>((uint64_t)n_tiles, &tile.node));
    RG_TRY(tmp.dev_n<int64_t>((uint64_t)n_tiles, &tile.begin));
    RG_TRY(tmp.dev_n<int32_t>((uint64_t)n_tiles, &tile.len));
    RG_TRY(tmp.dev_n<uint64_t>((uint64_t)n_tiles, &tile.state));
    if (n_tiles > 0) {
        ScopedTimer tm(KG_OFFSETS, st);
        hipLaunchKernelGGL(tile_records_kernel, dim3((unsigned)((n_tiles + 255) / 256)), dim3(256), 0, st, tile_off, rec.row_begin, rec.deg, rec.state, n_cur, n_tiles, tile);
    }
    int32_t *tile_order = nullptr;
    bool group_tiles = n_tiles >= (int64_t)n_cu * 64 && n_tiles <= 0x7FFFFFFF;     // fewer jobs than two rounds of the resident waves: nothing to bring together
    if (const char *force = getenv("RAPIDGNN_GROUP_TILES")) group_tiles = force[0] == '1' && n_tiles > 0 && n_tiles <= 0x7FFFFFFF;     // same results either way; for tests and tuning
    if (group_tiles) {
        int bits = 12;                                    // about 32 jobs to a bucket: buckets that share pieces only widen the set in flight
        while (bits < 20 && ((int64_t)32 << bits) < n_tiles) ++bits;
        const uint64_t n_buckets = (uint64_t)1 << bits;
        int32_t *cnt = nullptr, *rank = nullptr;
        int64_t *off = nullptr;
        RG_TRY(tmp.dev_n<int32_t>(n_buckets, &cnt));
        RG_TRY(tmp.dev_n<int32_t>((uint64_t)n_tiles, &rank));
        RG_TRY(tmp.dev_n<int64_t>(n_buckets + 1, &off));
        RG_TRY(tmp.dev_n<int32_t>((uint64_t)n_tiles, &tile_order));
        ScopedTimer tm(KG_OFFSETS, st);
        RG_HIP(hipMemsetAsync(cnt, 0, n_buckets * sizeof(int32_t), st));
        const dim3 grid((unsigned)((n_tiles + 255) / 256));
        hipLaunchKernelGGL(tile_bucket_count_kernel, grid, dim3(256), 0, st, tile.begin, n_tiles, bits, cnt, rank);
        RG_TRY(scan_i32_to_i64(cnt, off, (int64_t)n_buckets, tmp, st));
        hipLaunchKernelGGL(tile_bucket_place_kernel, grid, dim3(256), 0, st, tile.begin, n_tiles, bits, off, rank, tile_order);
        RG_HIP(hipGetLastError());
    }

    if (fanout > 0 && n_cur > 0) {
        // Rows of up to SHORT_ROW IDs are sampled four at a time wherever a frontier has any: by a kernel of their own
        // where the hop marks with plain byte stores, inside the other kernel (each group's short rows first) where marks are
        // atomic ORs -- a kernel of nothing but short rows is then bound by the rate of those atomics (large_sparse: 58 M of
        // them in 2.6 ms, 22 G/s), while between the streaming of long rows they cost next to nothing.  Same samples in
        // every case; RAPIDGNN_SHORT_ROWS = 0 / 1 / 2 forces one row per wave / the kernel of their own / the inline form.
        int short_mode = sums[2] == 0 ? 0 : use_bytes ? 1 : 2;
        if (const char *force = getenv("RAPIDGNN_SHORT_ROWS")) short_mode = force[0] == '1' ? 1 : force[0] == '2' ? 2 : 0;
        const bool short_rows_apart = short_mode == 1;
        const uint32_t need = fanout + 64;
        const int mark = need > 256 ? MARK_BITS : all_flags && use_bytes ? MARK_BYTES_ALL : all_flags ? MARK_BITS_ALL : use_bytes ? MARK_BYTES : MARK_BITS;
        unsigned long long *next_work = nullptr;
        RG_TRY(tmp.dev_n<unsigned long long>(1, &next_work));
        RG_HIP(hipMemsetAsync(next_work, 0, sizeof(unsigned long long), st));
        int merge_span = 64;                              // tiles per look of a merging wave: 64 if that still occupies the chip's waves
        while (merge_span > 1 && n_tiles / merge_span < (int64_t)n_cu * 32) merge_span >>= 1;
        const unsigned merge_grid = (unsigned)std::max<int64_t>(1, std::min<int64_t>((n_tiles + merge_span - 1) / merge_span, (int64_t)n_cu * 64));
        HopArgs a{g->indices, cur.ids, n_cur, 0, 0, short_mode != 0 ? SHORT_ROW : 0, short_mode == 2 ? 1 : 0, rec, fanout, cur.samp_off, cur.samp_nbr, tile_off, tile, n_tiles, tile_out, merge_span, tile_order, reached, next_work};
        ScopedTimer tm(KG_SAMPLER, st);
        // worth it where a group is long work: rows of a thousand IDs on average, tiles aside (short rows finish a
        // group of 64 in no time, and four times the requests to the work counter then cost more than the tail does;
        // measured: Medium, 2,500 IDs per row, 4 % faster; large_sparse and partition_share, a few hundred, 1-8 % slower)
        const unsigned long long ids_here = sums[1] - (short_mode != 0 ? sums[3] : 0), rows_here = (unsigned long long)n_cur - (short_mode != 0 ? sums[2] : 0);
        const bool fine_tail = ids_here >= 1024ull * rows_here;
        // a frontier that does not give every resident wave a group of 64 (the seed hop) is split finer from rows of 256 IDs on
        const bool fine_if_few = ids_here >= 256ull * rows_here;
        if (need <= 128) {
            if (all_flags && use_bytes) RG_TRY((launch_hop<128, MARK_BYTES_ALL>(a, n_cu, merge_grid, fine_tail, fine_if_few, st)));
            else if (all_flags) RG_TRY((launch_hop<128, MARK_BITS_ALL>(a, n_cu, merge_grid, fine_tail, fine_if_few, st)));
            else if (use_bytes) RG_TRY((launch_hop<128, MARK_BYTES>(a, n_cu, merge_grid, fine_tail, fine_if_few, st)));
            else RG_TRY((launch_hop<128, MARK_BITS>(a, n_cu, merge_grid, fine_tail, fine_if_few, st)));
        } else if (need <= 256) {
            if (all_flags && use_bytes) RG_TRY((launch_hop<256, MARK_BYTES_ALL>(a, n_cu, merge_grid, fine_tail, fine_if_few, st)));
            else if (all_flags) RG_TRY((launch_hop<256, MARK_BITS_ALL>(a, n_cu, merge_grid, fine_tail, fine_if_few, st)));
            else if (use_bytes) RG_TRY((launch_hop<256, MARK_BYTES>(a, n_cu, merge_grid, fine_tail, fine_if_few, st)));
            else RG_TRY((launch_hop<256, MARK_BITS>(a, n_cu, merge_grid, fine_tail, fine_if_few, st)));
        }
        else if (need <= 512) RG_TRY((launch_hop<512, MARK_BITS>(a, n_cu, merge_grid, fine_tail, fine_if_few, st)));
        else if (need <= 1024) RG_TRY((launch_hop<1024, MARK_BITS>(a, n_cu, merge_grid, fine_tail, fine_if_few, st)));
        else RG_TRY((launch_hop<2048, MARK_BITS>(a, n_cu, merge_grid, fine_tail, fine_if_few, st)));
        RG_HIP(hipGetLastError());
        if (short_rows_apart) {
            const ShortArgs sa{g->indices, n_cur, rec, fanout, cur.samp_off, cur.samp_nbr, reached};
            switch (mark) {
            case MARK_BYTES_ALL: RG_TRY(launch_short<MARK_BYTES_ALL>(sa, n_cu, st)); break;
            case MARK_BITS_ALL: RG_TRY(launch_short<MARK_BITS_ALL>(sa, n_cu, st)); break;
            case MARK_BYTES: RG_TRY(launch_short<MARK_BYTES>(sa, n_cu, st)); break;
            default: RG_TRY(launch_short<MARK_BITS>(sa, n_cu, st)); break;
            }
            RG_HIP(hipGetLastError());
        }
    }
    return RG_OK;
}

}  // namespace rg

