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
//  - longer rows are streamed once, 256 IDs per step, the next step's loads
//    already in flight.  IDs whose key is below the current cut are appended
//    (ballot ranks again, so in row order) to an LDS buffer of CAP >= f + 64
//    IDs; when the buffer could overflow it is pruned to the f smallest keys
//    with the same search and an in-place ordered compaction, which also
//    tightens the cut.  What is left after the last step is the sample.
//  - rows longer than BIG_ROW are cut into T near-equal tiles, each sampled by
//    its own wave into scratch (f IDs per tile, row order); a second small
//    launch samples the concatenation of a row's tile results, which is the
//    row's sample: the f smallest keys of the row are among the f smallest of
//    each tile.  This bounds the work of one wave whatever the degree skew.
//
// No step sorts anything.  While a wave writes a sample it also marks the
// batch's reached-ID bitmaps, so frontier dedup costs no extra pass.
#include "rg_internal.h"
#include "rg_device.h"

#include <algorithm>

namespace rg {

constexpr int BIG_ROW = 16384;           // rows longer than this are sampled tile by tile

__device__ __host__ __forceinline__ int64_t tiles_of(int64_t deg) { return deg > BIG_ROW ? (deg + BIG_ROW - 1) / BIG_ROW : 0; }

// Per frontier node, by position: where its row starts, its degree, its batch and its stream.
struct NodeRecs {
    int64_t *row_begin;
    int32_t *deg;
    uint32_t *batch;
    uint64_t *state;      // S_v = combine(combine(S_{e,i}, hop + 1), v)
};

__global__ void node_records_kernel(const int64_t *__restrict__ indptr, const int32_t *__restrict__ frontier, int64_t n,
                                    const int64_t *__restrict__ batch_off, uint32_t n_batches, const uint64_t *__restrict__ batch_seed,
                                    uint32_t hop, uint32_t fanout, NodeRecs r, int32_t *__restrict__ cnt, int32_t *__restrict__ tiles)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const int32_t v = frontier[i];
    const int64_t b0 = indptr[v];
    const int64_t deg = indptr[v + 1] - b0;
    const uint32_t b = batch_of(batch_off, n_batches, i);
    r.row_begin[i] = b0;
    r.deg[i] = (int32_t)deg;
    r.batch[i] = b;
    r.state[i] = combine(combine(batch_seed[b], (uint64_t)hop + 1u), (uint64_t)(uint32_t)v);
    cnt[i] = (int32_t)(deg < (int64_t)fanout ? deg : (int64_t)fanout);
    tiles[i] = (int32_t)tiles_of(deg);
}

__device__ __forceinline__ int lanes_below(unsigned long long m, int lane) { return __popcll(m & ((1ull << lane) - 1ull)); }

__device__ __forceinline__ int64_t bcast64(int64_t x, int src_lane)
{
    const uint32_t lo = (uint32_t)__shfl((int)(uint32_t)x, src_lane, 64);
    const uint32_t hi = (uint32_t)__shfl((int)(uint32_t)((uint64_t)x >> 32), src_lane, 64);
    return (int64_t)(((uint64_t)hi << 32) | lo);
}

// A threshold that exactly `keep` of the keys held in registers (E per lane, `total` >= keep of
// them valid) do not exceed.  Bisection on the key value, counting with ballots: the keep-th
// smallest key stays inside [lo, lo + 2^(bit+1)), and the search stops as soon as the number of
// keys below the bracket's upper end is exactly `keep` -- after about log2(total) steps for
// spread-out keys, 32 at most (keys are distinct).
template <int E>
__device__ __forceinline__ uint32_t kth_key_threshold(const uint32_t (&k)[E], const bool (&valid)[E], int keep, int total)
{
    uint32_t lo = 0;
    int below_hi = total;
    int bit = 31;
    while (below_hi != keep) {
        const uint32_t trial = lo | (1u << bit);
        int below = 0;
#pragma unroll
        for (int e = 0; e < E; ++e) below += __popcll(__ballot(valid[e] && k[e] < trial));
        if (below < keep) lo = trial; else below_hi = below;
        --bit;
    }
    return lo + (uint32_t)((((uint64_t)1) << (bit + 1)) - 1u);
}

// Row of f < len <= 64 * E IDs held in registers (u[e] of lane l is row[e * 64 + l]),
// sampled and written to out in row order.
template <int E, bool MARK>
__device__ __forceinline__ void sample_registers(const uint32_t (&u)[E], int len, int f, uint32_t lo, uint32_t hi, int lane,
                                                 int32_t *__restrict__ out, uint32_t *__restrict__ seen_b, uint32_t *__restrict__ fresh_b)
{
    uint32_t k[E];
    bool valid[E];
#pragma unroll
    for (int e = 0; e < E; ++e) {
        valid[e] = e * 64 + lane < len;
        k[e] = key32(lo, hi, u[e]);
    }
    const uint32_t cut = kth_key_threshold<E>(k, valid, f, len);
    int base = 0;
#pragma unroll
    for (int e = 0; e < E; ++e) {
        const bool keep_it = valid[e] && k[e] <= cut;
        const unsigned long long m = __ballot(keep_it);
        if (keep_it) {
            out[base + lanes_below(m, lane)] = (int32_t)u[e];
            if (MARK) mark_reached(seen_b, fresh_b, u[e]);
        }
        base += __popcll(m);
    }
}

// Keeps the `keep` smallest-key entries of buf[0..cnt), order preserved; returns a threshold that
// exactly those entries' keys do not exceed.
// Precondition: cnt > keep >= 1, cnt <= CAP.
template <int CAP>
__device__ __forceinline__ uint32_t prune_buffer(uint32_t *buf, int cnt, int keep, uint32_t lo, uint32_t hi, int lane)
{
    constexpr int E = CAP / 64;
    uint32_t u[E], k[E];
    bool valid[E];
#pragma unroll
    for (int e = 0; e < E; ++e) {
        const int idx = e * 64 + lane;
        valid[e] = idx < cnt;
        u[e] = valid[e] ? buf[idx] : 0u;
        k[e] = key32(lo, hi, u[e]);
    }
    const uint32_t cut = kth_key_threshold<E>(k, valid, keep, cnt);
    __syncthreads();          // every lane has read its entries before any is overwritten
    int base = 0;
#pragma unroll
    for (int e = 0; e < E; ++e) {
        const bool keep_it = valid[e] && k[e] <= cut;
        const unsigned long long m = __ballot(keep_it);
        if (keep_it) buf[base + lanes_below(m, lane)] = u[e];
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

// One step of 256 IDs (cur[e] of lane l is step[e * 64 + l]); FULL: all 256 are inside the row.
template <int CAP, bool FULL>
__device__ __forceinline__ void stream_step(const uint32_t (&cur)[4], int count, int f, uint32_t lo, uint32_t hi, int lane, uint32_t *buf, Stream &s)
{
    uint32_t k[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) k[e] = key32(lo, hi, cur[e]);
    bool ok[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) ok[e] = FULL || e * 64 + lane < count;
    if (!s.open) {
        const bool any = (ok[0] && k[0] <= s.cut) || (ok[1] && k[1] <= s.cut) || (ok[2] && k[2] <= s.cut) || (ok[3] && k[3] <= s.cut);
        if (__ballot(any) == 0ull) return;
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        if (s.cnt > CAP - 64) {               // the next 64 might not fit: tighten first
            s.cut = prune_buffer<CAP>(buf, s.cnt, f, lo, hi, lane);
            s.cnt = f;
            s.open = false;
        }
        const bool pass = ok[e] && (s.open || k[e] <= s.cut);
        const unsigned long long m = __ballot(pass);
        if (pass) buf[s.cnt + lanes_below(m, lane)] = cur[e];
        s.cnt += __popcll(m);
    }
}

// Row of len > 256 IDs streamed once; `first` holds row[lane]; on return buf[0..f) is the sample in row order.
template <int CAP>
__device__ __forceinline__ void sample_long_row(const int32_t *__restrict__ row, int len, uint32_t first, int f, uint32_t lo, uint32_t hi, int lane,
                                                uint32_t *buf)
{
    Stream s{0, true, 0u};
    const int n_full = len >> 8, tail = len & 255;
    uint32_t cur[4], nxt[4] = {0u, 0u, 0u, 0u};
    cur[0] = first;
#pragma unroll
    for (int e = 1; e < 4; ++e) cur[e] = (uint32_t)row[e * 64 + lane];
    for (int c = 0; c < n_full; ++c) {
        const int32_t *p = row + (c + 1) * 256;                  // next step's loads go out before this step's keys are computed
        if (c + 1 < n_full) {
#pragma unroll
            for (int e = 0; e < 4; ++e) nxt[e] = (uint32_t)p[e * 64 + lane];
        } else if (tail) {
#pragma unroll
            for (int e = 0; e < 4; ++e) nxt[e] = e * 64 + lane < tail ? (uint32_t)p[e * 64 + lane] : 0u;
        }
        stream_step<CAP, true>(cur, 256, f, lo, hi, lane, buf, s);
#pragma unroll
        for (int e = 0; e < 4; ++e) cur[e] = nxt[e];
    }
    if (tail) stream_step<CAP, false>(cur, tail, f, lo, hi, lane, buf, s);
    __syncthreads();
    if (s.cnt > f) (void)prune_buffer<CAP>(buf, s.cnt, f, lo, hi, lane);
}

// SAMPLE of a row of len > f IDs into out (row order), marking the bitmaps when MARK.
// `first` holds row[lane] for lane < len.
template <int CAP, bool MARK>
__device__ __forceinline__ void sample_row(const int32_t *__restrict__ row, int len, uint32_t first, int f, uint32_t lo, uint32_t hi, int lane,
                                           uint32_t *buf, int32_t *__restrict__ out, uint32_t *__restrict__ seen_b, uint32_t *__restrict__ fresh_b)
{
    if (len <= 64) {
        const uint32_t u[1] = {first};
        sample_registers<1, MARK>(u, len, f, lo, hi, lane, out, seen_b, fresh_b);
    } else if (len <= 256) {
        uint32_t u[4];
        u[0] = first;
#pragma unroll
        for (int e = 1; e < 4; ++e) u[e] = e * 64 + lane < len ? (uint32_t)row[e * 64 + lane] : 0u;
        sample_registers<4, MARK>(u, len, f, lo, hi, lane, out, seen_b, fresh_b);
    } else {
        sample_long_row<CAP>(row, len, first, f, lo, hi, lane, buf);
        for (int j = lane; j < f; j += 64) {
            const uint32_t u = buf[j];
            out[j] = (int32_t)u;
            if (MARK) mark_reached(seen_b, fresh_b, u);
        }
        __syncthreads();      // the buffer is reused by the wave's next row
    }
}

struct HopArgs {
    const int32_t *indices;
    const int32_t *frontier; int64_t n_frontier;
    NodeRecs rec;
    uint32_t fanout;
    const int64_t *samp_off; int32_t *samp_nbr;
    const int64_t *tile_off; int64_t n_tiles; int32_t *tile_out;      // tile j writes tile_out[j * fanout ..)
    uint32_t *seen; uint32_t *fresh; uint64_t words_per_batch;
};

// Position i of the frontier whose tiles contain tile job j: tile_off[i] <= j < tile_off[i + 1].
__device__ __forceinline__ int64_t node_of_tile(const int64_t *__restrict__ tile_off, int64_t n, int64_t j)
{
    int64_t lo = 0, hi = n;
    while (hi - lo > 1) {
        const int64_t mid = (lo + hi) >> 1;
        if (tile_off[mid] <= j) lo = mid; else hi = mid;
    }
    return lo;
}

// Work items [0, n_tiles) are tiles of long rows (first, so the longest-running work starts first);
// item n_tiles + c is the c-th group of 64 consecutive frontier nodes.
template <int CAP>
__global__ void __launch_bounds__(64) sample_kernel(HopArgs a)
{
    __shared__ uint32_t buf[CAP];
    const int lane = threadIdx.x;
    const int f = (int)a.fanout;
    const int64_t n_groups = (a.n_frontier + 63) >> 6;
    const int64_t n_work = a.n_tiles + n_groups;
    for (int64_t w = blockIdx.x; w < n_work; w += gridDim.x) {
        if (w < a.n_tiles) {
            const int64_t i = node_of_tile(a.tile_off, a.n_frontier, w);
            const int64_t T = a.tile_off[i + 1] - a.tile_off[i], t = w - a.tile_off[i];
            const int64_t row_begin = a.rec.row_begin[i], deg = a.rec.deg[i];
            const int64_t first_pos = t * deg / T, last_pos = (t + 1) * deg / T;     // near-equal tiles, each longer than 2 * RG_MAX_FANOUT
            const uint64_t S = a.rec.state[i];
            const int32_t *row = a.indices + row_begin + first_pos;
            sample_row<CAP, false>(row, (int)(last_pos - first_pos), (uint32_t)row[lane], f, (uint32_t)S, (uint32_t)(S >> 32), lane, buf,
                                   a.tile_out + w * f, nullptr, nullptr);
            continue;
        }
        const int64_t i_lane = ((w - a.n_tiles) << 6) + lane;
        const bool in = i_lane < a.n_frontier;
        const int64_t rb_lane = in ? a.rec.row_begin[i_lane] : 0;
        const int deg_lane = in ? a.rec.deg[i_lane] : 0;
        const uint32_t b_lane = in ? a.rec.batch[i_lane] : 0u;
        const int64_t S_lane = in ? (int64_t)a.rec.state[i_lane] : 0;
        const int64_t out_lane = in ? a.samp_off[i_lane] : 0;
        unsigned long long todo = __ballot(deg_lane > 0 && deg_lane <= BIG_ROW);
        if (todo == 0ull) continue;
        // the first node's leading 64 IDs; from then on the next node's are fetched while the current one is sampled
        int l = __ffsll((long long)todo) - 1;
        int64_t rb = bcast64(rb_lane, l);
        int deg = __shfl(deg_lane, l, 64);
        uint32_t first = lane < deg ? (uint32_t)a.indices[rb + lane] : 0u;
        while (todo != 0ull) {
            todo &= todo - 1ull;
            const int cl = l, cdeg = deg;
            const int64_t crb = rb;
            const uint32_t cfirst = first;
            if (todo != 0ull) {
                l = __ffsll((long long)todo) - 1;
                rb = bcast64(rb_lane, l);
                deg = __shfl(deg_lane, l, 64);
                first = lane < deg ? (uint32_t)a.indices[rb + lane] : 0u;
            }
            const uint32_t b = (uint32_t)__shfl((int)b_lane, cl, 64);
            uint32_t *seen_b = a.seen + (uint64_t)b * a.words_per_batch;
            uint32_t *fresh_b = a.fresh + (uint64_t)b * a.words_per_batch;
            const int32_t *row = a.indices + crb;
            int32_t *out = a.samp_nbr + bcast64(out_lane, cl);
            if (cdeg <= f) {                  // the whole row is the sample
                if (lane < cdeg) { out[lane] = (int32_t)cfirst; mark_reached(seen_b, fresh_b, cfirst); }
                for (int j = 64 + lane; j < cdeg; j += 64) {
                    const int32_t u = row[j];
                    out[j] = u;
                    mark_reached(seen_b, fresh_b, (uint32_t)u);
                }
            } else {
                const uint64_t S = (uint64_t)bcast64(S_lane, cl);
                sample_row<CAP, true>(row, cdeg, cfirst, f, (uint32_t)S, (uint32_t)(S >> 32), lane, buf, out, seen_b, fresh_b);
            }
        }
    }
}

// One wave per tile job; the wave that holds a long row's first tile samples the row's
// concatenated tile results (T * f IDs, row order, all distinct) into the final output.
template <int CAP>
__global__ void __launch_bounds__(64) sample_merge_kernel(HopArgs a)
{
    __shared__ uint32_t buf[CAP];
    const int lane = threadIdx.x;
    const int f = (int)a.fanout;
    for (int64_t w = blockIdx.x; w < a.n_tiles; w += gridDim.x) {
        const int64_t i = node_of_tile(a.tile_off, a.n_frontier, w);
        if (a.tile_off[i] != w) continue;
        const int64_t T = a.tile_off[i + 1] - a.tile_off[i];
        const uint32_t b = a.rec.batch[i];
        const uint64_t S = a.rec.state[i];
        const int32_t *row = a.tile_out + w * f;
        const int len = (int)(T * f);
        sample_row<CAP, true>(row, len, lane < len ? (uint32_t)row[lane] : 0u, f, (uint32_t)S, (uint32_t)(S >> 32), lane, buf,
                              a.samp_nbr + a.samp_off[i], a.seen + (uint64_t)b * a.words_per_batch, a.fresh + (uint64_t)b * a.words_per_batch);
    }
}

template <int CAP>
static void launch_hop(const HopArgs &a, unsigned grid, unsigned merge_grid, hipStream_t st)
{
    hipLaunchKernelGGL(sample_kernel<CAP>, dim3(grid), dim3(64), 0, st, a);
    if (a.n_tiles > 0) hipLaunchKernelGGL(sample_merge_kernel<CAP>, dim3(merge_grid), dim3(64), 0, st, a);
}

// Samples hop `hop` of every batch: fills cur.samp_off / samp_nbr / n_samples and marks seen / fresh.
rg_status sample_hop(const rg_graph *g, HopData &cur, uint32_t beta, const uint64_t *batch_seed, uint32_t hop, uint32_t fanout,
                     uint32_t *seen, uint32_t *fresh, uint64_t words_per_batch, Arena &keep, Arena &tmp, int n_cu, hipStream_t st)
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
    {
        ScopedTimer tm(KG_OFFSETS, st);
        hipLaunchKernelGGL(node_records_kernel, dim3((unsigned)((n_cur + 255) / 256)), dim3(256), 0, st, g->indptr, cur.ids, n_cur, cur.off_dev, beta,
                           batch_seed, hop, fanout, rec, cnt, tiles);
        RG_TRY(scan_i32_to_i64(cnt, cur.samp_off, n_cur, tmp, st));
        RG_TRY(scan_i32_to_i64(tiles, tile_off, n_cur, tmp, st));
    }
    int64_t n_tiles = 0;
    RG_HIP(hipMemcpyAsync(&cur.n_samples, cur.samp_off + n_cur, sizeof(int64_t), hipMemcpyDeviceToHost, st));
    RG_HIP(hipMemcpyAsync(&n_tiles, tile_off + n_cur, sizeof(int64_t), hipMemcpyDeviceToHost, st));
    RG_HIP(hipStreamSynchronize(st));
    tmp.free_one(cnt);
    tmp.free_one(tiles);
    RG_TRY(keep.dev_n<int32_t>((uint64_t)cur.n_samples, &cur.samp_nbr));
    if (fanout == 0) n_tiles = 0;             // nothing is drawn; every sample is empty
    int32_t *tile_out = nullptr;
    RG_TRY(tmp.dev_n<int32_t>((uint64_t)n_tiles * fanout, &tile_out));

    if (fanout > 0 && n_cur > 0) {
        HopArgs a{g->indices, cur.ids, n_cur, rec, fanout, cur.samp_off, cur.samp_nbr, tile_off, n_tiles, tile_out, seen, fresh, words_per_batch};
        ScopedTimer tm(KG_SAMPLER, st);
        const int64_t n_work = n_tiles + (n_cur + 63) / 64;
        const unsigned grid = (unsigned)std::max<int64_t>(1, std::min<int64_t>(n_work, (int64_t)n_cu * 64));
        const unsigned merge_grid = (unsigned)std::max<int64_t>(1, std::min<int64_t>(n_tiles, (int64_t)n_cu * 64));
        const uint32_t need = fanout + 64;
        if (need <= 128) launch_hop<128>(a, grid, merge_grid, st);
        else if (need <= 256) launch_hop<256>(a, grid, merge_grid, st);
        else if (need <= 512) launch_hop<512>(a, grid, merge_grid, st);
        else if (need <= 1024) launch_hop<1024>(a, grid, merge_grid, st);
        else launch_hop<2048>(a, grid, merge_grid, st);
        RG_HIP(hipGetLastError());
    }
    return RG_OK;
}

}  // namespace rg
