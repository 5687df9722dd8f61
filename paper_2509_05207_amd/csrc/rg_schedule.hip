// rg_build_schedule: seed derivation, epoch shuffle, per-hop fan-out sampling
// and frontier construction for all batches of an epoch at once.
//
// Layout in HBM.  Batches are independent, so a hop is one launch over the
// concatenated frontiers of every batch.  Per batch the library keeps two
// bitmaps of n_nodes bits for the duration of the build: `seen` (members of
// the current frontier) and `fresh` (IDs first reached in this hop).  Reading
// the fresh bitmap in word order yields the new IDs already deduplicated and
// in ascending order, which is the canonical frontier order; no sort or hash
// table is involved and the result does not depend on the order in which
// waves mark bits.
#include "rg_internal.h"

#include <algorithm>
#include <atomic>

namespace rg {

// ---------------------------------------------------------------- hash family
// H of Sec. 3 "Seeding and reproducibility": a 64-bit multiply / xor-shift
// mixer.  Constants: floor(2^64/phi), frac(sqrt 2) * 2^64 made odd,
// frac(sqrt 3) * 2^64; the 32-bit ones are the top words of the same numbers.
constexpr uint64_t HG64 = 0x9E3779B97F4A7C15ull;
constexpr uint64_t HA64 = 0x6A09E667F3BCC909ull;
constexpr uint64_t HB64 = 0xBB67AE8584CAA73Bull;
constexpr uint32_t HG32 = 0x9E3779B9u;
constexpr uint32_t HA32 = 0x6A09E667u;
constexpr uint32_t HB32 = 0xBB67AE85u;

__host__ __device__ __forceinline__ uint64_t mix64(uint64_t x)
{
    x ^= x >> 32; x *= HA64; x ^= x >> 29; x *= HB64; x ^= x >> 32;
    return x;
}
__host__ __device__ __forceinline__ uint64_t combine(uint64_t h, uint64_t x) { return mix64(h ^ mix64(x + HG64)); }

// Key of neighbour u under a node's state (lo, hi).  For fixed state this is a
// bijection of 32-bit words, so the keys of one row never tie.
__device__ __forceinline__ uint32_t key32(uint32_t lo, uint32_t hi, uint32_t u)
{
    uint32_t x = u ^ lo;
    x *= HG32; x ^= x >> 16;
    x += hi;
    x *= HA32; x ^= x >> 15;
    x *= HB32; x ^= x >> 16;
    return x;
}

// ---------------------------------------------------------------- a1/a2: seeds, shuffle keys
__global__ void batch_seeds_kernel(uint64_t s0, uint32_t worker, uint32_t epoch, uint32_t n_batches, uint64_t *__restrict__ seeds)
{
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_batches) return;
    uint64_t h = mix64(s0 ^ HG64);
    h = combine(h, worker);
    h = combine(h, epoch);
    h = combine(h, i);
    seeds[i] = h;
}

// Shuffle: train position t gets key combine(P_e, t); the epoch's order is
// ascending (key, t).  Entries beyond T are padding that sorts last.
struct KeyPos { uint64_t key; uint64_t pos; };

__device__ __forceinline__ bool kp_less(const KeyPos &a, const KeyPos &b)
{
    return a.key < b.key || (a.key == b.key && a.pos < b.pos);
}

__global__ void shuffle_keys_kernel(uint64_t s0, uint32_t worker, uint32_t epoch, uint64_t T, uint64_t n_pad, KeyPos *__restrict__ kp)
{
    const uint64_t t = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= n_pad) return;
    uint64_t P = mix64(s0 ^ HG64);
    P = combine(P, worker);
    P = combine(P, ((uint64_t)1 << 32) + epoch);
    KeyPos x;
    if (t < T) { x.key = combine(P, t); x.pos = t; }
    else { x.key = ~0ull; x.pos = ~0ull; }
    kp[t] = x;
}

// Bitonic network.  Stages whose partner distance is < SORT_TILE/2 run in LDS.
constexpr int SORT_THREADS = 256;
constexpr int SORT_TILE = 2048;     // elements per block in the LDS kernels (32 KB of KeyPos)

__global__ void __launch_bounds__(SORT_THREADS) bitonic_global_step(KeyPos *__restrict__ kp, uint64_t n_pad, uint64_t k, uint64_t j)
{
    const uint64_t t = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;      // one compare-exchange per thread
    if (t >= n_pad / 2) return;
    const uint64_t i = ((t & ~(j - 1)) << 1) | (t & (j - 1));                // index with bit j clear
    const uint64_t l = i | j;
    const bool up = (i & k) == 0;
    KeyPos a = kp[i], b = kp[l];
    if (kp_less(b, a) == up) { kp[i] = b; kp[l] = a; }
}

// Runs, inside LDS, every stage (k, j) with k in [k_first, k_last] and j <= min(k/2, SORT_TILE/2);
// for k > SORT_TILE only the tail j = SORT_TILE/2 .. 1 of that k (k_first == k_last then).
__global__ void __launch_bounds__(SORT_THREADS) bitonic_lds_steps(KeyPos *__restrict__ kp, uint64_t k_first, uint64_t k_last)
{
    __shared__ KeyPos tile[SORT_TILE];
    const uint64_t base = (uint64_t)blockIdx.x * SORT_TILE;
    for (int e = threadIdx.x; e < SORT_TILE; e += SORT_THREADS) tile[e] = kp[base + e];
    __syncthreads();
    for (uint64_t k = k_first; k <= k_last; k <<= 1) {
        uint64_t j0 = k >> 1;
        if (j0 > SORT_TILE / 2) j0 = SORT_TILE / 2;
        for (uint64_t j = j0; j >= 1; j >>= 1) {
            for (int t = threadIdx.x; t < SORT_TILE / 2; t += SORT_THREADS) {
                const uint32_t i = (uint32_t)(((t & ~(j - 1)) << 1) | (t & (j - 1)));
                const uint32_t l = i | (uint32_t)j;
                const bool up = ((base + i) & k) == 0;
                KeyPos a = tile[i], b = tile[l];
                if (kp_less(b, a) == up) { tile[i] = b; tile[l] = a; }
            }
            __syncthreads();
        }
    }
    for (int e = threadIdx.x; e < SORT_TILE; e += SORT_THREADS) kp[base + e] = tile[e];
}

__global__ void apply_shuffle_kernel(const KeyPos *__restrict__ kp, const int32_t *__restrict__ train, uint64_t T, int32_t *__restrict__ seeds)
{
    const uint64_t t = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t < T) seeds[t] = train[kp[t].pos];
}

// ---------------------------------------------------------------- batch lookup
// Batch of flat frontier position i: the b with off[b] <= i < off[b+1].
__device__ __forceinline__ uint32_t batch_of(const int64_t *__restrict__ off, uint32_t n_batches, int64_t i)
{
    uint32_t lo = 0, hi = n_batches;          // invariant: off[lo] <= i < off[hi]
    while (hi - lo > 1) {
        const uint32_t mid = (lo + hi) >> 1;
        if (off[mid] <= i) lo = mid; else hi = mid;
    }
    return lo;
}

// ---------------------------------------------------------------- bitmaps
__global__ void mark_seeds_kernel(const int32_t *__restrict__ seeds, uint64_t T, uint32_t batch_size, uint32_t *__restrict__ seen, uint64_t words_per_batch)
{
    const uint64_t t = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= T) return;
    const uint32_t v = (uint32_t)seeds[t];
    atomicOr(&seen[(t / batch_size) * words_per_batch + (v >> 5)], 1u << (v & 31));
}

// A sampled ID is new to the batch iff its `seen` bit was clear; the wave that
// flips it also sets the `fresh` bit.  Bits are only ever set here, so the
// plain pre-check can at worst cause a redundant atomic.
__device__ __forceinline__ void mark_reached(uint32_t *__restrict__ seen_b, uint32_t *__restrict__ fresh_b, uint32_t u)
{
    const uint32_t w = u >> 5, bit = 1u << (u & 31);
    if (seen_b[w] & bit) return;
    const uint32_t old = atomicOr(&seen_b[w], bit);
    if (!(old & bit)) atomicOr(&fresh_b[w], bit);
}

// ---------------------------------------------------------------- a3: per-node sample sizes
__global__ void sample_counts_kernel(const int64_t *__restrict__ indptr, const int32_t *__restrict__ frontier, int64_t n, uint32_t fanout,
                                     int32_t *__restrict__ cnt)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const int32_t v = frontier[i];
    const int64_t deg = indptr[v + 1] - indptr[v];
    cnt[i] = (int32_t)(deg < (int64_t)fanout ? deg : (int64_t)fanout);
}

// ---------------------------------------------------------------- a3: the sampler
// One wavefront per frontier node (grid-stride over nodes), one wave per
// workgroup.  The row is streamed once, 64 neighbours per step, coalesced.
// SAMPLE keeps the `fanout` neighbours with the smallest keys.  Candidates
// (key below the current cut) are appended to an LDS buffer in row order; when
// the buffer could overflow, the exact fanout-th smallest key among them is
// found by a bitwise search on ballots and the buffer is compacted in place,
// still in row order, which also tightens the cut for the rest of the row.
// What is left after the last step is the sample, already in row order.
template <int CAP>
struct Selector {
    static constexpr int E = CAP / 64;      // buffer entries per lane

    // Keeps the `keep` smallest-key entries of buf[0..cnt), order preserved; returns the cut
    // (the keep-th smallest key).  Precondition: cnt > keep >= 1, cnt <= CAP.
    static __device__ __forceinline__ uint32_t prune(uint32_t *buf, int cnt, int keep, uint32_t lo, uint32_t hi, int lane)
    {
        uint32_t u[E], k[E];
        bool valid[E];
#pragma unroll
        for (int e = 0; e < E; ++e) {
            const int idx = e * 64 + lane;
            valid[e] = idx < cnt;
            u[e] = valid[e] ? buf[idx] : 0u;
            k[e] = key32(lo, hi, u[e]);
        }
        // largest cut with |{key < cut}| < keep  ==  the keep-th smallest key
        uint32_t cut = 0;
        for (int bit = 31; bit >= 0; --bit) {
            const uint32_t trial = cut | (1u << bit);
            int below = 0;
#pragma unroll
            for (int e = 0; e < E; ++e) below += __popcll(__ballot(valid[e] && k[e] < trial));
            if (below < keep) cut = trial;
        }
        __syncthreads();          // every lane has read its entries before any is overwritten
        int base = 0;
#pragma unroll
        for (int e = 0; e < E; ++e) {
            const bool keep_it = valid[e] && k[e] <= cut;
            const unsigned long long m = __ballot(keep_it);
            if (keep_it) buf[base + __popcll(m & ((1ull << lane) - 1ull))] = u[e];
            base += __popcll(m);
        }
        __syncthreads();
        return cut;
    }
};

template <int CAP>
__global__ void __launch_bounds__(64) sample_kernel(const int64_t *__restrict__ indptr, const int32_t *__restrict__ indices,
                                                    const int32_t *__restrict__ frontier, int64_t n_frontier,
                                                    const int64_t *__restrict__ batch_off, uint32_t n_batches,
                                                    const uint64_t *__restrict__ batch_seed, uint32_t hop, uint32_t fanout,
                                                    const int64_t *__restrict__ samp_off, int32_t *__restrict__ samp_nbr,
                                                    uint32_t *__restrict__ seen, uint32_t *__restrict__ fresh, uint64_t words_per_batch)
{
    __shared__ uint32_t buf[CAP];
    const int lane = threadIdx.x;
    const int f = (int)fanout;
    for (int64_t i = blockIdx.x; i < n_frontier; i += gridDim.x) {
        const int32_t v = frontier[i];
        const int64_t row_begin = indptr[v];
        const int64_t deg = indptr[v + 1] - row_begin;
        if (deg == 0 || f == 0) continue;
        const uint32_t b = batch_of(batch_off, n_batches, i);
        uint32_t *seen_b = seen + (uint64_t)b * words_per_batch;
        uint32_t *fresh_b = fresh + (uint64_t)b * words_per_batch;
        const int32_t *row = indices + row_begin;
        int32_t *out = samp_nbr + samp_off[i];

        if (deg <= f) {                       // the whole row is the sample
            for (int64_t j = lane; j < deg; j += 64) {
                const int32_t u = row[j];
                out[j] = u;
                mark_reached(seen_b, fresh_b, (uint32_t)u);
            }
            continue;
        }
        const uint64_t S = combine(combine(batch_seed[b], (uint64_t)hop + 1u), (uint64_t)(uint32_t)v);
        const uint32_t lo = (uint32_t)S, hi = (uint32_t)(S >> 32);

        int cnt = 0;                          // wave-uniform
        bool open = true;                     // no cut yet: everything is a candidate
        uint32_t cut = 0;
        for (int64_t base = 0; base < deg; base += 256) {
            uint32_t u[4], k[4];
            bool ok[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int64_t j = base + e * 64 + lane;
                ok[e] = j < deg;
                u[e] = ok[e] ? (uint32_t)row[j] : 0u;
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) k[e] = key32(lo, hi, u[e]);
            if (!open) {
                const bool any = (ok[0] && k[0] < cut) || (ok[1] && k[1] < cut) || (ok[2] && k[2] < cut) || (ok[3] && k[3] < cut);
                if (__ballot(any) == 0ull) continue;
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (cnt > CAP - 64) {         // the next 64 might not fit: tighten first
                    cut = Selector<CAP>::prune(buf, cnt, f, lo, hi, lane);
                    cnt = f;
                    open = false;
                }
                const bool pass = ok[e] && (open || k[e] < cut);
                const unsigned long long m = __ballot(pass);
                if (pass) buf[cnt + __popcll(m & ((1ull << lane) - 1ull))] = u[e];
                cnt += __popcll(m);
            }
        }
        __syncthreads();
        if (cnt > f) { (void)Selector<CAP>::prune(buf, cnt, f, lo, hi, lane); cnt = f; }
        for (int j = lane; j < f; j += 64) {
            const uint32_t u = buf[j];
            out[j] = (int32_t)u;
            mark_reached(seen_b, fresh_b, u);
        }
        __syncthreads();                      // buffer is reused by the next node
    }
}

// ---------------------------------------------------------------- a4: frontier from the fresh bitmap
constexpr int FR_THREADS = 256;
constexpr int FR_WORDS_PER_THREAD = 8;
constexpr int FR_CHUNK_WORDS = FR_THREADS * FR_WORDS_PER_THREAD;     // 2048 words = 65536 node IDs per block

// cnt[b * chunks + c] = number of fresh IDs of batch b in chunk c
__global__ void __launch_bounds__(FR_THREADS) fresh_count_kernel(const uint32_t *__restrict__ fresh, uint64_t words_per_batch, uint32_t chunks,
                                                                 int32_t *__restrict__ cnt)
{
    __shared__ int red[FR_THREADS / 64];
    const uint32_t c = blockIdx.x, b = blockIdx.y;
    const uint32_t *base = fresh + (uint64_t)b * words_per_batch;
    const uint64_t w0 = (uint64_t)c * FR_CHUNK_WORDS + (uint64_t)threadIdx.x * FR_WORDS_PER_THREAD;
    int n = 0;
    if (w0 < words_per_batch) {      // words_per_batch is a multiple of FR_WORDS_PER_THREAD
        const uint4 a = *reinterpret_cast<const uint4 *>(base + w0);
        const uint4 d = *reinterpret_cast<const uint4 *>(base + w0 + 4);
        n = __popc(a.x) + __popc(a.y) + __popc(a.z) + __popc(a.w) + __popc(d.x) + __popc(d.y) + __popc(d.z) + __popc(d.w);
    }
    for (int o = 32; o > 0; o >>= 1) n += __shfl_down(n, o, 64);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = n;
    __syncthreads();
    if (threadIdx.x == 0) cnt[(uint64_t)b * chunks + c] = red[0] + red[1] + red[2] + red[3];
}

// next_off[b] = cur_off[b] + (number of fresh IDs in batches < b)
__global__ void next_offsets_kernel(const int64_t *__restrict__ cur_off, const int64_t *__restrict__ fresh_scan, uint32_t n_batches, uint32_t chunks,
                                    int64_t *__restrict__ next_off)
{
    const uint32_t b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b <= n_batches) next_off[b] = cur_off[b] + fresh_scan[(uint64_t)b * chunks];
}

__global__ void copy_prefix_kernel(const int32_t *__restrict__ cur, const int64_t *__restrict__ cur_off, const int64_t *__restrict__ next_off,
                                   uint32_t n_batches, int64_t n_cur, int32_t *__restrict__ next)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_cur) return;
    const uint32_t b = batch_of(cur_off, n_batches, i);
    next[next_off[b] + (i - cur_off[b])] = cur[i];
}

// Writes the fresh IDs of (batch, chunk) in ascending order behind the batch's old frontier
// and clears the words it consumed, leaving `fresh` all-zero for the next hop.
__global__ void __launch_bounds__(FR_THREADS) fresh_emit_kernel(uint32_t *__restrict__ fresh, uint64_t words_per_batch, uint32_t chunks,
                                                                const int64_t *__restrict__ fresh_scan, const int64_t *__restrict__ cur_off,
                                                                int32_t *__restrict__ next)
{
    __shared__ int wave_tot[FR_THREADS / 64];
    const uint32_t c = blockIdx.x, b = blockIdx.y;
    const int64_t scan_here = fresh_scan[(uint64_t)b * chunks + c];
    if (fresh_scan[(uint64_t)b * chunks + c + 1] == scan_here) return;       // nothing fresh in this chunk (block-uniform)
    uint32_t *base = fresh + (uint64_t)b * words_per_batch;
    const uint64_t w0 = (uint64_t)c * FR_CHUNK_WORDS + (uint64_t)threadIdx.x * FR_WORDS_PER_THREAD;
    uint32_t w[FR_WORDS_PER_THREAD] = {0, 0, 0, 0, 0, 0, 0, 0};
    int n = 0;
    if (w0 < words_per_batch) {
        const uint4 a = *reinterpret_cast<const uint4 *>(base + w0);
        const uint4 d = *reinterpret_cast<const uint4 *>(base + w0 + 4);
        w[0] = a.x; w[1] = a.y; w[2] = a.z; w[3] = a.w; w[4] = d.x; w[5] = d.y; w[6] = d.z; w[7] = d.w;
#pragma unroll
        for (int k = 0; k < FR_WORDS_PER_THREAD; ++k) n += __popc(w[k]);
        if (n) {
            *reinterpret_cast<uint4 *>(base + w0) = make_uint4(0, 0, 0, 0);
            *reinterpret_cast<uint4 *>(base + w0 + 4) = make_uint4(0, 0, 0, 0);
        }
    }
    // exclusive scan of n over the block
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int incl = n;
    for (int d = 1; d < 64; d <<= 1) {
        const int y = __shfl_up(incl, d, 64);
        if (lane >= d) incl += y;
    }
    if (lane == 63) wave_tot[wave] = incl;
    __syncthreads();
    int before = incl - n;
    for (int k = 0; k < wave; ++k) before += wave_tot[k];
    // next_off[b] + |U_l of b| + scan - scan(b, 0)  ==  cur_off[b + 1] + scan
    int64_t pos = cur_off[b + 1] + scan_here + before;
#pragma unroll
    for (int k = 0; k < FR_WORDS_PER_THREAD; ++k) {
        uint32_t x = w[k];
        const uint32_t id0 = (uint32_t)((w0 + k) << 5);
        while (x) {
            const int bit = __ffs((int)x) - 1;
            x &= x - 1;
            next[pos++] = (int32_t)(id0 + bit);
        }
    }
}

static std::atomic<uint64_t> g_next_uid{1};

static rg_status sort_keypos(KeyPos *kp, uint64_t n_pad, hipStream_t st)
{
    // n_pad is a power of two >= SORT_TILE
    const unsigned lds_blocks = (unsigned)(n_pad / SORT_TILE);
    const unsigned g_blocks = (unsigned)((n_pad / 2 + SORT_THREADS - 1) / SORT_THREADS);
    hipLaunchKernelGGL(bitonic_lds_steps, dim3(lds_blocks), dim3(SORT_THREADS), 0, st, kp, (uint64_t)2, (uint64_t)SORT_TILE);
    for (uint64_t k = (uint64_t)SORT_TILE * 2; k <= n_pad; k <<= 1) {
        for (uint64_t j = k >> 1; j > SORT_TILE / 2; j >>= 1)
            hipLaunchKernelGGL(bitonic_global_step, dim3(g_blocks), dim3(SORT_THREADS), 0, st, kp, n_pad, k, j);
        hipLaunchKernelGGL(bitonic_lds_steps, dim3(lds_blocks), dim3(SORT_THREADS), 0, st, kp, k, k);
    }
    RG_HIP(hipGetLastError());
    return RG_OK;
}

template <int CAP>
static void launch_sampler(unsigned grid, hipStream_t st, const rg_graph *g, const int32_t *frontier, int64_t n_frontier,
                           const int64_t *batch_off, uint32_t n_batches, const uint64_t *batch_seed, uint32_t hop, uint32_t fanout,
                           const int64_t *samp_off, int32_t *samp_nbr, uint32_t *seen, uint32_t *fresh, uint64_t wpb)
{
    hipLaunchKernelGGL(sample_kernel<CAP>, dim3(grid), dim3(64), 0, st, g->indptr, g->indices, frontier, n_frontier, batch_off,
                       n_batches, batch_seed, hop, fanout, samp_off, samp_nbr, seen, fresh, wpb);
}

static rg_status build_schedule_impl(const rg_graph *g, const int32_t *train, uint64_t T, uint32_t B, const uint32_t *fanout,
                                     uint32_t L, uint64_t s0, uint32_t worker, uint32_t epoch, const rg_allocator *a, hipStream_t st, rg_schedule *s)
{
    const uint32_t beta = (uint32_t)(B ? (T + B - 1) / B : 0);
    s->n_nodes = g->n_nodes;
    s->n_batches = beta;
    s->L = L;
    s->T = T;
    s->uid = g_next_uid.fetch_add(1);
    s->hop.resize(L + 1);
    Arena tmp(a);             // build-time scratch, released when this function returns

    // ---- a1: batch seeds
    uint64_t *batch_seed = nullptr;
    RG_TRY(tmp.dev_n<uint64_t>(beta ? beta : 1, &batch_seed));
    if (beta) hipLaunchKernelGGL(batch_seeds_kernel, dim3((beta + 255) / 256), dim3(256), 0, st, s0, worker, epoch, beta, batch_seed);

    // ---- a2: shuffle and cut into batches
    HopData &h0 = s->hop[0];
    RG_TRY(s->arena.dev_n<int32_t>(T, &h0.ids));
    RG_TRY(s->arena.dev_n<int64_t>((uint64_t)beta + 1, &h0.off_dev));
    h0.off_host.resize((size_t)beta + 1);
    for (uint32_t b = 0; b <= beta; ++b) h0.off_host[b] = (int64_t)std::min<uint64_t>((uint64_t)b * B, T);
    RG_HIP(hipMemcpyAsync(h0.off_dev, h0.off_host.data(), ((size_t)beta + 1) * sizeof(int64_t), hipMemcpyHostToDevice, st));
    if (T > 0) {
        uint64_t n_pad = SORT_TILE;
        while (n_pad < T) n_pad <<= 1;
        KeyPos *kp = nullptr;
        RG_TRY(tmp.dev_n<KeyPos>(n_pad, &kp));
        {
            ScopedTimer tm(KG_SORT, st);
            hipLaunchKernelGGL(shuffle_keys_kernel, dim3((unsigned)((n_pad + 255) / 256)), dim3(256), 0, st, s0, worker, epoch, T, n_pad, kp);
            RG_TRY(sort_keypos(kp, n_pad, st));
            hipLaunchKernelGGL(apply_shuffle_kernel, dim3((unsigned)((T + 255) / 256)), dim3(256), 0, st, kp, train, T, h0.ids);
        }
        RG_HIP(hipGetLastError());
    }
    if (beta == 0) {          // no batches: every hop is an empty frontier with the single offset 0
        for (uint32_t l = 0; l < L; ++l) {
            RG_TRY(s->arena.dev_n<int64_t>(1, &s->hop[l].samp_off));
            RG_HIP(hipMemsetAsync(s->hop[l].samp_off, 0, sizeof(int64_t), st));
            RG_TRY(s->arena.dev_n<int32_t>(0, &s->hop[l].samp_nbr));
            HopData &nx = s->hop[l + 1];
            RG_TRY(s->arena.dev_n<int32_t>(0, &nx.ids));
            RG_TRY(s->arena.dev_n<int64_t>(1, &nx.off_dev));
            RG_HIP(hipMemsetAsync(nx.off_dev, 0, sizeof(int64_t), st));
            nx.off_host.assign(1, 0);
        }
    }
    if (L == 0 || beta == 0) { RG_HIP(hipStreamSynchronize(st)); return RG_OK; }

    // ---- bitmaps (n_nodes bits per batch, rounded up to whole 8-word groups)
    const uint64_t wpb = (((uint64_t)g->n_nodes + 31) / 32 + FR_WORDS_PER_THREAD - 1) / FR_WORDS_PER_THREAD * FR_WORDS_PER_THREAD;
    const uint32_t chunks = (uint32_t)((wpb + FR_CHUNK_WORDS - 1) / FR_CHUNK_WORDS);
    uint32_t *seen = nullptr, *fresh = nullptr;
    RG_TRY(tmp.dev_n<uint32_t>(wpb * beta, &seen));
    RG_TRY(tmp.dev_n<uint32_t>(wpb * beta, &fresh));
    RG_HIP(hipMemsetAsync(seen, 0, wpb * beta * sizeof(uint32_t), st));
    RG_HIP(hipMemsetAsync(fresh, 0, wpb * beta * sizeof(uint32_t), st));
    {
        ScopedTimer tm(KG_FRONTIER, st);
        hipLaunchKernelGGL(mark_seeds_kernel, dim3((unsigned)((T + 255) / 256)), dim3(256), 0, st, h0.ids, T, B, seen, wpb);
    }
    int32_t *fresh_cnt = nullptr;
    int64_t *fresh_scan = nullptr;
    const uint64_t n_cells = (uint64_t)beta * chunks;
    RG_TRY(tmp.dev_n<int32_t>(n_cells, &fresh_cnt));
    RG_TRY(tmp.dev_n<int64_t>(n_cells + 1, &fresh_scan));

    int dev = 0, n_cu = 256;
    RG_HIP(hipGetDevice(&dev));
    RG_HIP(hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev));

    for (uint32_t l = 0; l < L; ++l) {
        HopData &cur = s->hop[l];
        HopData &nxt = s->hop[l + 1];
        const int64_t n_cur = cur.off_host[beta];
        const uint32_t f = fanout[l];

        // sample sizes -> offsets
        int32_t *cnt = nullptr;
        RG_TRY(tmp.dev_n<int32_t>((uint64_t)n_cur, &cnt));
        RG_TRY(s->arena.dev_n<int64_t>((uint64_t)n_cur + 1, &cur.samp_off));
        {
            ScopedTimer tm(KG_OFFSETS, st);
            hipLaunchKernelGGL(sample_counts_kernel, dim3((unsigned)((n_cur + 255) / 256)), dim3(256), 0, st, g->indptr, cur.ids, n_cur, f, cnt);
            RG_TRY(scan_i32_to_i64(cnt, cur.samp_off, n_cur, tmp, st));
        }
        RG_HIP(hipMemcpyAsync(&cur.n_samples, cur.samp_off + n_cur, sizeof(int64_t), hipMemcpyDeviceToHost, st));
        RG_HIP(hipStreamSynchronize(st));
        tmp.free_one(cnt);
        RG_TRY(s->arena.dev_n<int32_t>((uint64_t)cur.n_samples, &cur.samp_nbr));

        // the sampler, marking reached IDs as it writes them
        {
            ScopedTimer tm(KG_SAMPLER, st);
            const unsigned grid = (unsigned)std::min<int64_t>(n_cur, (int64_t)n_cu * 64);
            const uint32_t need = f + 64;
            if (need <= 128) launch_sampler<128>(grid, st, g, cur.ids, n_cur, cur.off_dev, beta, batch_seed, l, f, cur.samp_off, cur.samp_nbr, seen, fresh, wpb);
            else if (need <= 256) launch_sampler<256>(grid, st, g, cur.ids, n_cur, cur.off_dev, beta, batch_seed, l, f, cur.samp_off, cur.samp_nbr, seen, fresh, wpb);
            else if (need <= 512) launch_sampler<512>(grid, st, g, cur.ids, n_cur, cur.off_dev, beta, batch_seed, l, f, cur.samp_off, cur.samp_nbr, seen, fresh, wpb);
            else if (need <= 1024) launch_sampler<1024>(grid, st, g, cur.ids, n_cur, cur.off_dev, beta, batch_seed, l, f, cur.samp_off, cur.samp_nbr, seen, fresh, wpb);
            else launch_sampler<2048>(grid, st, g, cur.ids, n_cur, cur.off_dev, beta, batch_seed, l, f, cur.samp_off, cur.samp_nbr, seen, fresh, wpb);
            RG_HIP(hipGetLastError());
        }

        // fresh IDs per (batch, chunk) -> positions -> next frontier
        RG_TRY(s->arena.dev_n<int64_t>((uint64_t)beta + 1, &nxt.off_dev));
        {
            ScopedTimer tm(KG_FRONTIER, st);
            hipLaunchKernelGGL(fresh_count_kernel, dim3(chunks, beta), dim3(FR_THREADS), 0, st, fresh, wpb, chunks, fresh_cnt);
            RG_TRY(scan_i32_to_i64(fresh_cnt, fresh_scan, (int64_t)n_cells, tmp, st));
            hipLaunchKernelGGL(next_offsets_kernel, dim3((beta + 1 + 255) / 256), dim3(256), 0, st, cur.off_dev, fresh_scan, beta, chunks, nxt.off_dev);
        }
        nxt.off_host.resize((size_t)beta + 1);
        RG_HIP(hipMemcpyAsync(nxt.off_host.data(), nxt.off_dev, ((size_t)beta + 1) * sizeof(int64_t), hipMemcpyDeviceToHost, st));
        RG_HIP(hipStreamSynchronize(st));
        const int64_t n_next = nxt.off_host[beta];
        RG_TRY(s->arena.dev_n<int32_t>((uint64_t)n_next, &nxt.ids));
        {
            ScopedTimer tm(KG_FRONTIER, st);
            hipLaunchKernelGGL(copy_prefix_kernel, dim3((unsigned)((n_cur + 255) / 256)), dim3(256), 0, st, cur.ids, cur.off_dev, nxt.off_dev, beta, n_cur, nxt.ids);
            hipLaunchKernelGGL(fresh_emit_kernel, dim3(chunks, beta), dim3(FR_THREADS), 0, st, fresh, wpb, chunks, fresh_scan, cur.off_dev, nxt.ids);
        }
        RG_HIP(hipGetLastError());
    }
    RG_HIP(hipStreamSynchronize(st));
    return RG_OK;
}

}  // namespace rg

using namespace rg;

extern "C" rg_status rg_build_schedule(const rg_graph *g, const int32_t *train_nodes, uint64_t T, uint32_t batch_size,
                                       const uint32_t *fanout, uint32_t L, uint64_t s0, uint32_t worker, uint32_t epoch,
                                       const rg_allocator *a, void *stream, rg_schedule **out)
{
    if (!g || !out) { set_error("rg_build_schedule: null graph or output pointer"); return RG_EINVAL; }
    if (g->n_nodes < 0 || g->n_nodes >= ((int64_t)1 << 31)) { set_error("rg_build_schedule: n_nodes %lld outside [0, 2^31)", (long long)g->n_nodes); return RG_ERANGE; }
    if (!g->indptr) { set_error("rg_build_schedule: null indptr"); return RG_EINVAL; }
    if (T > 0 && !train_nodes) { set_error("rg_build_schedule: null train_nodes with T > 0"); return RG_EINVAL; }
    if (T > 0 && batch_size == 0) { set_error("rg_build_schedule: batch_size must be > 0"); return RG_EINVAL; }
    if (T > 0 && g->n_nodes == 0) { set_error("rg_build_schedule: train nodes given for an empty graph"); return RG_EINVAL; }
    if (L > RG_MAX_HOPS) { set_error("rg_build_schedule: L = %u exceeds RG_MAX_HOPS = %u", L, RG_MAX_HOPS); return RG_ERANGE; }
    if (L > 0 && !fanout) { set_error("rg_build_schedule: null fanout with L > 0"); return RG_EINVAL; }
    for (uint32_t l = 0; l < L; ++l)
        if (fanout[l] > RG_MAX_FANOUT) { set_error("rg_build_schedule: fanout[%u] = %u exceeds RG_MAX_FANOUT = %u", l, fanout[l], RG_MAX_FANOUT); return RG_ERANGE; }
    if (T > 0 && (T + batch_size - 1) / batch_size > 0xFFFFFFFFull / 2) { set_error("rg_build_schedule: too many batches"); return RG_ERANGE; }

    rg_schedule *s = new (std::nothrow) rg_schedule(a);
    if (!s) { set_error("rg_build_schedule: out of host memory"); return RG_ENOMEM; }
    rg_status rc = build_schedule_impl(g, train_nodes, T, batch_size, fanout, L, s0, worker, epoch, a, as_stream(stream), s);
    if (rc != RG_OK) {
        (void)hipStreamSynchronize(as_stream(stream));
        delete s;
        return rc;
    }
    *out = s;
    return RG_OK;
}
