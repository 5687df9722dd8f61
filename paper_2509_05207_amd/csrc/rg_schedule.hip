// rg_build_schedule: seed derivation, epoch shuffle, per-hop fan-out sampling
// (rg_sampler.hip) and frontier construction for all batches of an epoch.
//
// Layout in HBM.  Batches are independent, so a hop is one launch over the
// concatenated frontiers of every batch.  Per batch the library keeps two
// bitmaps of n_nodes bits for the duration of the build: `seen` (members of
// the current frontier) and `reached` (IDs sampled in this hop).  Reading
// reached & ~seen in word order yields the new IDs already deduplicated and in
// ascending order, which is the canonical frontier order; no sort or hash
// table is involved and the result does not depend on the order in which
// waves mark bits.
#include "rg_internal.h"
#include "rg_device.h"

#include <cstdlib>

#include <algorithm>
#include <atomic>

namespace rg {

rg_status sample_hop(const rg_graph *g, HopData &cur, uint32_t beta, const uint64_t *batch_seed, uint32_t hop, uint32_t fanout, uint32_t sampler,
                     ReachedForms &maps, int prefer_bytes, bool *marked_bytes, Arena &keep, Arena &tmp, int n_cu, hipStream_t st,
                     const unsigned long long *also_read_dev, unsigned long long *also_read_host);

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

// Shuffle: train position t gets key combine(P_e, t); the epoch's order is ascending (key, t).
//
// The keys are hash values, so their top bits spread them evenly: the positions are dealt into buckets by the top
// bits of their keys (a count, a prefix sum, a scatter), and one workgroup per bucket then places each of its
// bucket's entries by rank -- the number of entries of the bucket that precede it in (key, t) order -- which for a
// hundred-odd entries per bucket is less work than any sorting network and takes a bucket of any size (its entries
// pass through LDS a tile at a time).  Four launches and a prefix sum, whatever T.
struct KeyPos { uint64_t key; uint64_t pos; };

__device__ __forceinline__ bool kp_less(const KeyPos &a, const KeyPos &b)
{
    return a.key < b.key || (a.key == b.key && a.pos < b.pos);
}

__device__ __forceinline__ uint64_t shuffle_key(uint64_t s0, uint32_t worker, uint32_t epoch, uint64_t t)
{
    uint64_t P = mix64(s0 ^ HG64);
    P = combine(P, worker);
    P = combine(P, ((uint64_t)1 << 32) + epoch);
    return combine(P, t);
}
__device__ __forceinline__ uint32_t bucket_of_key(uint64_t key, uint32_t bucket_bits) { return bucket_bits ? (uint32_t)(key >> (64u - bucket_bits)) : 0u; }

__global__ void shuffle_count_kernel(uint64_t s0, uint32_t worker, uint32_t epoch, uint64_t T, uint32_t bucket_bits, int32_t *__restrict__ bucket_cnt)
{
    const uint64_t t = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t < T) atomicAdd(&bucket_cnt[bucket_of_key(shuffle_key(s0, worker, epoch, t), bucket_bits)], 1);
}

// bucket_cnt is counted down again, so every slot of a bucket is handed out once; the order inside a bucket is
// whatever the atomics give, the ranks below do not depend on it.
__global__ void shuffle_scatter_kernel(uint64_t s0, uint32_t worker, uint32_t epoch, uint64_t T, uint32_t bucket_bits,
                                       const int64_t *__restrict__ bucket_off, int32_t *__restrict__ bucket_cnt, KeyPos *__restrict__ kp)
{
    const uint64_t t = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= T) return;
    const uint64_t key = shuffle_key(s0, worker, epoch, t);
    const uint32_t b = bucket_of_key(key, bucket_bits);
    const int32_t left = atomicSub(&bucket_cnt[b], 1);                 // count .. 1
    kp[bucket_off[b] + left - 1] = KeyPos{key, t};
}

constexpr int RANK_THREADS = 256;
constexpr int RANK_TILE = 1024;      // entries of a bucket in LDS at a time (16 KB)

// One workgroup per bucket: seeds[first + rank(x)] = train[x.pos] for every entry x of the bucket.
__global__ void __launch_bounds__(RANK_THREADS) shuffle_rank_kernel(const KeyPos *__restrict__ kp, const int64_t *__restrict__ bucket_off,
                                                                    const int32_t *__restrict__ train, int32_t *__restrict__ seeds)
{
    __shared__ KeyPos tile[RANK_TILE];
    const int64_t first = bucket_off[blockIdx.x], n = bucket_off[blockIdx.x + 1] - first;
    for (int64_t e0 = 0; e0 < n; e0 += RANK_THREADS) {                 // the entries this round's threads place (uniform trip count)
        const int64_t e = e0 + threadIdx.x;
        const bool have = e < n;
        KeyPos mine = have ? kp[first + e] : KeyPos{0, 0};
        int64_t rank = 0;
        for (int64_t j0 = 0; j0 < n; j0 += RANK_TILE) {
            const int m = (int)(n - j0 < RANK_TILE ? n - j0 : RANK_TILE);
            __syncthreads();                                           // the previous tile has been read by everyone
            for (int j = threadIdx.x; j < m; j += RANK_THREADS) tile[j] = kp[first + j0 + j];
            __syncthreads();
            if (have)
                for (int j = 0; j < m; ++j) rank += kp_less(tile[j], mine) ? 1 : 0;
        }
        if (have) seeds[first + rank] = train[mine.pos];
    }
}

// The precondition on train_nodes, checked on the device: *n_bad += the IDs outside [0, n_nodes) and the IDs that
// occurred before (`once`: a bit per node ID, clear on entry).  Until the host has seen the count (at the build's
// first readback), the kernels that index by a seed's value skip values out of range.
__global__ void check_train_kernel(const int32_t *__restrict__ train, uint64_t T, int64_t n_nodes, uint32_t *__restrict__ once,
                                   unsigned long long *__restrict__ n_bad)
{
    const uint64_t t = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    bool bad = false;
    if (t < T) {
        const int64_t v = train[t];
        if (v < 0 || v >= n_nodes) bad = true;
        else bad = (atomicOr(&once[v >> 5], 1u << (v & 31)) >> (v & 31)) & 1u;
    }
    const unsigned long long m = __ballot(bad);
    if (m != 0ull && (threadIdx.x & 63) == 0) atomicAdd(n_bad, (unsigned long long)__popcll(m));
}

// paired: `seen` points at the first group's `seen` half of the paired records (see paired_word)
__global__ void mark_seeds_kernel(const int32_t *__restrict__ seeds, uint64_t T, uint32_t batch_size, uint32_t *__restrict__ seen,
                                  uint8_t *__restrict__ seen_flags, uint64_t words_per_batch, int64_t n_nodes, int paired)
{
    const uint64_t t = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= T) return;
    const uint32_t v = (uint32_t)seeds[t];
    if ((int64_t)v >= n_nodes) return;          // (refused by the host as soon as it has read check_train_kernel's count)
    const uint64_t word = (t / batch_size) * words_per_batch + (v >> 5);
    atomicOr(&seen[paired ? paired_word(word) : word], 1u << (v & 31));
    if (seen_flags) seen_flags[word >> 3] = 1;          // (NULL in the large-graph form: see clear_listed_seen_kernel)
}

// ---------------------------------------------------------------- a6 (first half): freq(v) of the epoch as column sums
// After the last hop a batch's `seen` bitmap is exactly its input set N_i^e, so freq(v) = in how many batches' bitmaps
// bit v is set: the sum of a column of a bit matrix of n_batches rows.  A thread owns one word position (32 node IDs)
// and adds the batches' words into 16 bit-sliced counters (plane k holds bit k of all 32 counts; adding a word is a
// ripple of AND/XOR through the planes), so the whole tally reads every bitmap once, coalesced, and has no atomics.
constexpr int FREQ_PLANES = 16;          // counts up to 65,535 batches
__global__ void epoch_freq_kernel(const uint32_t *__restrict__ seen, uint64_t words_per_batch, uint32_t n_batches, int64_t n_nodes,
                                  uint32_t *__restrict__ freq)
{
    const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= words_per_batch) return;
    uint32_t plane[FREQ_PLANES];
#pragma unroll
    for (int k = 0; k < FREQ_PLANES; ++k) plane[k] = 0;
    for (uint32_t b = 0; b < n_batches; ++b) {
        uint32_t carry = seen[(uint64_t)b * words_per_batch + i];
#pragma unroll
        for (int k = 0; k < FREQ_PLANES; ++k) {
            const uint32_t t = plane[k] & carry;
            plane[k] ^= carry;
            carry = t;
        }
    }
    const int64_t v0 = (int64_t)(i << 5);
#pragma unroll 4
    for (int j = 0; j < 32; ++j) {
        uint32_t c = 0;
#pragma unroll
        for (int k = 0; k < FREQ_PLANES; ++k) c |= ((plane[k] >> j) & 1u) << k;
        if (v0 + j < n_nodes) freq[v0 + j] = c;
    }
}

// ---------------------------------------------------------------- a4: frontier from the fresh bitmap
constexpr int FR_THREADS = 256;
constexpr int FR_WORDS_PER_THREAD = 8;
constexpr int FR_CHUNK_WORDS = FR_THREADS * FR_WORDS_PER_THREAD;     // 2048 words = 65536 node IDs per block

// The reached bits of one group of 256 IDs (eight words).  BYTES: from the byte map, where every ID has a byte that
// is 0 or 1: four such bytes in a dword d become four bits by one multiply ((d * 0x00204081) >> 21 puts byte k's bit
// at position k; the partial products below bit 21 sum to less than 2^17, so nothing carries in).
template <bool BYTES>
__device__ __forceinline__ void load_reached_group(const void *reached, uint64_t at, uint32_t (&r)[8])
{
    if (!BYTES) {
        const uint32_t *p = static_cast<const uint32_t *>(reached) + at;
        const uint4 r0 = *reinterpret_cast<const uint4 *>(p), r1 = *reinterpret_cast<const uint4 *>(p + 4);
        r[0] = r0.x; r[1] = r0.y; r[2] = r0.z; r[3] = r0.w; r[4] = r1.x; r[5] = r1.y; r[6] = r1.z; r[7] = r1.w;
    } else {
        const uint4 *p = reinterpret_cast<const uint4 *>(static_cast<const uint8_t *>(reached) + (at << 5));       // 256 bytes
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const uint4 a = p[2 * k], b = p[2 * k + 1];
            const uint32_t d[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
            uint32_t w = 0;
#pragma unroll
            for (int q = 0; q < 8; ++q) w |= ((d[q] * 0x00204081u >> 21) & 0xFu) << (4 * q);
            r[k] = w;
        }
    }
}
template <bool BYTES>
__device__ __forceinline__ void clear_reached_group(void *reached, uint64_t at)
{
    if (!BYTES) {
        uint32_t *p = static_cast<uint32_t *>(reached) + at;
        *reinterpret_cast<uint4 *>(p) = make_uint4(0, 0, 0, 0);
        *reinterpret_cast<uint4 *>(p + 4) = make_uint4(0, 0, 0, 0);
    } else {
        uint4 *p = reinterpret_cast<uint4 *>(static_cast<uint8_t *>(reached) + (at << 5));
#pragma unroll
        for (int k = 0; k < 16; ++k) p[k] = make_uint4(0, 0, 0, 0);
    }
}

// cnt[b * chunks + c] = number of fresh IDs (reached and not yet seen) of batch b in chunk c
template <bool BYTES>
__global__ void __launch_bounds__(FR_THREADS) fresh_count_kernel(const void *__restrict__ reached, const uint8_t *__restrict__ flags,
                                                                 const uint32_t *__restrict__ seen, uint64_t words_per_batch, uint32_t chunks,
                                                                 int32_t *__restrict__ cnt)
{
    __shared__ int red[FR_THREADS / 64];
    const uint32_t c = blockIdx.x, b = blockIdx.y;
    const uint64_t w0 = (uint64_t)c * FR_CHUNK_WORDS + (uint64_t)threadIdx.x * FR_WORDS_PER_THREAD;
    int n = 0;
    if (w0 < words_per_batch) {      // words_per_batch is a multiple of FR_WORDS_PER_THREAD; a thread's words are one flag's group
        const uint64_t at = (uint64_t)b * words_per_batch + w0;
        if (flags[at >> 3]) {        // on big graphs most groups were not reached: neither map is read there
            uint32_t r[8];
            load_reached_group<BYTES>(reached, at, r);
            const uint4 s0 = *reinterpret_cast<const uint4 *>(seen + at), s1 = *reinterpret_cast<const uint4 *>(seen + at + 4);
            n = __popc(r[0] & ~s0.x) + __popc(r[1] & ~s0.y) + __popc(r[2] & ~s0.z) + __popc(r[3] & ~s0.w) +
                __popc(r[4] & ~s1.x) + __popc(r[5] & ~s1.y) + __popc(r[6] & ~s1.z) + __popc(r[7] & ~s1.w);
        }
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

// Writes the fresh IDs of (batch, chunk) in ascending order behind the batch's old frontier, adds
// the reached IDs to `seen` and clears `reached` for the next hop.
template <bool BYTES>
__global__ void __launch_bounds__(FR_THREADS) fresh_emit_kernel(void *__restrict__ reached, uint8_t *__restrict__ flags, uint32_t *__restrict__ seen,
                                                                uint8_t *__restrict__ seen_flags, uint64_t words_per_batch, uint32_t chunks, const int64_t *__restrict__ fresh_scan,
                                                                const int64_t *__restrict__ cur_off, int32_t *__restrict__ next)
{
    __shared__ int wave_tot[FR_THREADS / 64];
    const uint32_t c = blockIdx.x, b = blockIdx.y;
    const int64_t scan_here = fresh_scan[(uint64_t)b * chunks + c];
    const bool any_fresh = fresh_scan[(uint64_t)b * chunks + c + 1] != scan_here;      // block-uniform
    const uint64_t w0 = (uint64_t)c * FR_CHUNK_WORDS + (uint64_t)threadIdx.x * FR_WORDS_PER_THREAD;
    uint32_t w[FR_WORDS_PER_THREAD] = {0, 0, 0, 0, 0, 0, 0, 0};
    int n = 0;
    if (w0 < words_per_batch) {
        const uint64_t at = (uint64_t)b * words_per_batch + w0;
        if (flags[at >> 3]) {
            uint32_t r[8];
            load_reached_group<BYTES>(reached, at, r);
            const uint4 s0 = *reinterpret_cast<const uint4 *>(seen + at), s1 = *reinterpret_cast<const uint4 *>(seen + at + 4);
            w[0] = r[0] & ~s0.x; w[1] = r[1] & ~s0.y; w[2] = r[2] & ~s0.z; w[3] = r[3] & ~s0.w;
            w[4] = r[4] & ~s1.x; w[5] = r[5] & ~s1.y; w[6] = r[6] & ~s1.z; w[7] = r[7] & ~s1.w;
#pragma unroll
            for (int k = 0; k < FR_WORDS_PER_THREAD; ++k) n += __popc(w[k]);
            if (n) {
                *reinterpret_cast<uint4 *>(seen + at) = make_uint4(s0.x | r[0], s0.y | r[1], s0.z | r[2], s0.w | r[3]);
                *reinterpret_cast<uint4 *>(seen + at + 4) = make_uint4(s1.x | r[4], s1.y | r[5], s1.z | r[6], s1.w | r[7]);
                seen_flags[at >> 3] = 1;
            }
            clear_reached_group<BYTES>(reached, at);
            flags[at >> 3] = 0;
        }
    }
    if (!any_fresh) return;
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

// The same two passes for graphs so large that almost every group of a batch's bitmap is untouched (10^8 nodes:
// a batch reaches a few 10^4 IDs out of 3.5 M words).  A thread owns eight consecutive groups, i.e. one 8-byte
// load of flags; a cell is 16,384 words, so the grid is eight times smaller and an untouched cell costs one
// flag load per thread.  The few flagged groups of a wave's 512 are first listed (in ascending order, through
// LDS) and then dealt out one per lane, so that their loads are all in flight at once instead of one after
// another in the lane that happens to own them.  Flagged groups are read twice (count, then emit): they are few,
// but each read lands in a memory page of its own, which is what these passes cost -- so here a group's words of
// `reached` and of `seen` share one 64-byte record (see paired_word) and a visit is one scattered access, not two.
constexpr int FRS_GROUPS = 8;                                            // groups per thread (a multiple of eight; 16 and 32 measure the same)
constexpr int FRS_FLAG_WORDS = FRS_GROUPS / 8;                           // their flags, as 8-byte words
constexpr int FRS_WORDS_PER_THREAD = FR_WORDS_PER_THREAD * FRS_GROUPS;   // words_per_batch is a multiple of this
constexpr int FRS_CHUNK_WORDS = FR_THREADS * FRS_WORDS_PER_THREAD;
constexpr int FRS_WAVE_GROUPS = 64 * FRS_GROUPS;                         // groups per wave
constexpr int FRS_ROUNDS = FRS_GROUPS;                                   // a lane takes at most this many listed groups

struct FrsFlags { unsigned long long w[FRS_FLAG_WORDS]; };

__device__ __forceinline__ FrsFlags load_frs_flags(const uint8_t *flags, uint64_t first_group, bool inside)
{
    FrsFlags f;
#pragma unroll
    for (int k = 0; k < FRS_FLAG_WORDS; ++k) f.w[k] = inside ? reinterpret_cast<const unsigned long long *>(flags + first_group)[k] : 0ull;
    return f;
}

__device__ __forceinline__ void clear_frs_flags(uint8_t *flags, uint64_t first_group, const FrsFlags &f)
{
#pragma unroll
    for (int k = 0; k < FRS_FLAG_WORDS; ++k)
        if (f.w[k] != 0ull) reinterpret_cast<unsigned long long *>(flags + first_group)[k] = 0ull;
}

// The large-graph passes work on paired records (see paired_word): `reached` points at the records, `seen` eight
// words further on, and `at` is a group's first word in the records (twice its word in a map of its own).
__device__ __forceinline__ int fresh_in_group(const uint32_t *__restrict__ reached, const uint32_t *__restrict__ seen, uint64_t at, uint32_t (&w)[8])
{
    const uint4 r0 = *reinterpret_cast<const uint4 *>(reached + at), r1 = *reinterpret_cast<const uint4 *>(reached + at + 4);
    const uint4 s0 = *reinterpret_cast<const uint4 *>(seen + at), s1 = *reinterpret_cast<const uint4 *>(seen + at + 4);
    w[0] = r0.x & ~s0.x; w[1] = r0.y & ~s0.y; w[2] = r0.z & ~s0.z; w[3] = r0.w & ~s0.w;
    w[4] = r1.x & ~s1.x; w[5] = r1.y & ~s1.y; w[6] = r1.z & ~s1.z; w[7] = r1.w & ~s1.w;
    int n = 0;
#pragma unroll
    for (int k = 0; k < 8; ++k) n += __popc(w[k]);
    return n;
}

// Lists the wave's flagged groups in ascending order: list[0 .. total) holds their indices within the wave's 512
// (lane * 8 + g).  fl: this lane's eight flag bytes.  Returns total (wave-uniform).  Ends with a block barrier.
__device__ __forceinline__ int list_flagged_groups(const FrsFlags &fl, uint16_t *list /* this wave's [FRS_WAVE_GROUPS] */)
{
    const int lane = threadIdx.x & 63;
    // one bit per flagged group of this lane: a byte is non-zero iff, after OR-folding it onto its lowest bit, that bit is set
    unsigned long long x[FRS_FLAG_WORDS];
    int nf = 0;
#pragma unroll
    for (int k = 0; k < FRS_FLAG_WORDS; ++k) {
        unsigned long long y = fl.w[k];
        y |= y >> 4; y |= y >> 2; y |= y >> 1;
        x[k] = y & 0x0101010101010101ull;
        nf += __popcll(x[k]);
    }
    int incl = nf;
    for (int d = 1; d < 64; d <<= 1) {
        const int y = __shfl_up(incl, d, 64);
        if (lane >= d) incl += y;
    }
    const int total = __shfl(incl, 63, 64);
    int at = incl - nf;
#pragma unroll
    for (int g = 0; g < FRS_GROUPS; ++g)
        if ((x[g >> 3] >> (8 * (g & 7))) & 1ull) list[at++] = (uint16_t)(lane * FRS_GROUPS + g);
    __syncthreads();
    return total;
}

__global__ void __launch_bounds__(FR_THREADS) fresh_count_sparse_kernel(const uint32_t *__restrict__ reached, const uint8_t *__restrict__ flags,
                                                                        const uint32_t *__restrict__ seen, uint64_t words_per_batch,
                                                                        uint32_t chunks, int32_t *__restrict__ cnt)
{
    __shared__ uint16_t lists[FR_THREADS / 64][FRS_WAVE_GROUPS];
    __shared__ int red[FR_THREADS / 64];
    const uint32_t c = blockIdx.x, b = blockIdx.y;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint64_t w0 = (uint64_t)c * FRS_CHUNK_WORDS + (uint64_t)threadIdx.x * FRS_WORDS_PER_THREAD;
    const uint64_t at = (uint64_t)b * words_per_batch + w0;
    const FrsFlags fl = load_frs_flags(flags, at >> 3, w0 < words_per_batch);
    const int total = list_flagged_groups(fl, lists[wave]);
    const uint64_t wave_at = (uint64_t)b * words_per_batch + (uint64_t)c * FRS_CHUNK_WORDS + (uint64_t)wave * (FRS_WAVE_GROUPS * FR_WORDS_PER_THREAD);
    int n = 0;
    for (int i = lane; i < total; i += 64) {
        uint32_t w[8];
        n += fresh_in_group(reached, seen, 2 * (wave_at + (uint64_t)lists[wave][i] * FR_WORDS_PER_THREAD), w);
    }
    for (int o = 32; o > 0; o >>= 1) n += __shfl_down(n, o, 64);
    if (lane == 0) red[wave] = n;
    __syncthreads();
    if (threadIdx.x == 0) cnt[(uint64_t)b * chunks + c] = red[0] + red[1] + red[2] + red[3];
}

__global__ void __launch_bounds__(FR_THREADS) fresh_emit_sparse_kernel(uint32_t *__restrict__ reached, uint8_t *__restrict__ flags,
                                                                       uint32_t *__restrict__ seen, uint8_t *__restrict__ seen_flags,
                                                                       uint64_t words_per_batch, uint32_t chunks,
                                                                       const int64_t *__restrict__ fresh_scan, const int64_t *__restrict__ cur_off,
                                                                       int32_t *__restrict__ next, int keep_seen)
{
    // keep_seen == 0 (the last hop): nothing reads `seen` again, so the fresh IDs are not added to it
    __shared__ uint16_t lists[FR_THREADS / 64][FRS_WAVE_GROUPS];
    __shared__ int wave_tot[FR_THREADS / 64];
    const uint32_t c = blockIdx.x, b = blockIdx.y;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t scan_here = fresh_scan[(uint64_t)b * chunks + c];
    const bool any_fresh = fresh_scan[(uint64_t)b * chunks + c + 1] != scan_here;      // block-uniform
    const uint64_t w0 = (uint64_t)c * FRS_CHUNK_WORDS + (uint64_t)threadIdx.x * FRS_WORDS_PER_THREAD;
    const uint64_t at = (uint64_t)b * words_per_batch + w0;
    const FrsFlags fl = load_frs_flags(flags, at >> 3, w0 < words_per_batch);
    const int total = list_flagged_groups(fl, lists[wave]);
    const uint64_t wave_w0 = (uint64_t)c * FRS_CHUNK_WORDS + (uint64_t)wave * (FRS_WAVE_GROUPS * FR_WORDS_PER_THREAD);   // first word of the wave's groups within the batch
    const uint64_t wave_at = (uint64_t)b * words_per_batch + wave_w0;
    // first round of loads: how many fresh IDs each listed group holds, and from that where each group's IDs go
    int before[FRS_ROUNDS];            // fresh IDs of the wave's listed groups in front of this lane's group of round r
    uint32_t w_first[8] = {0, 0, 0, 0, 0, 0, 0, 0};       // the fresh words of the first round's group (nearly always the only round): kept for the second pass
    int n_first = 0;
    int carry = 0;
    if (any_fresh) {
#pragma unroll
        for (int r = 0; r < FRS_ROUNDS; ++r) {
            before[r] = 0;
            if (r * 64 < total) {                                       // wave-uniform
                const int i = r * 64 + lane;
                int n = 0;
                if (i < total) {
                    uint32_t w[8];
                    n = fresh_in_group(reached, seen, 2 * (wave_at + (uint64_t)lists[wave][i] * FR_WORDS_PER_THREAD), w);
                    if (r == 0) {
                        n_first = n;
#pragma unroll
                        for (int k = 0; k < 8; ++k) w_first[k] = w[k];
                    }
                }
                int incl = n;
                for (int d = 1; d < 64; d <<= 1) {
                    const int y = __shfl_up(incl, d, 64);
                    if (lane >= d) incl += y;
                }
                before[r] = carry + incl - n;
                carry += __shfl(incl, 63, 64);
            }
        }
    }
    if (lane == 0) wave_tot[wave] = carry;
    __syncthreads();
    int64_t base = cur_off[b + 1] + scan_here;
    for (int k = 0; k < wave; ++k) base += wave_tot[k];
    // second round: write the fresh IDs in ascending order, add them to `seen`, clear `reached`
#pragma unroll
    for (int r = 0; r < FRS_ROUNDS; ++r) {
        const int i = r * 64 + lane;
        if (i < total) {
            const uint32_t grp = lists[wave][i];
            const uint64_t ag = wave_at + (uint64_t)grp * FR_WORDS_PER_THREAD;
            if (any_fresh) {
                uint32_t w[8];
                int ng;
                if (r == 0) {
                    ng = n_first;
#pragma unroll
                    for (int k = 0; k < 8; ++k) w[k] = w_first[k];
                } else ng = fresh_in_group(reached, seen, 2 * ag, w);
                if (ng) {
                    int64_t pos = base + before[r];
#pragma unroll
                    for (int k = 0; k < 8; ++k) {
                        uint32_t x = w[k];
                        if (x) {
                            const uint32_t id0 = (uint32_t)((wave_w0 + (uint64_t)grp * FR_WORDS_PER_THREAD + k) << 5);
                            if (keep_seen) seen[2 * ag + k] |= x;
                            while (x) {
                                const int bit = __ffs((int)x) - 1;
                                x &= x - 1;
                                next[pos++] = (int32_t)(id0 + bit);
                            }
                        }
                    }
                    if (keep_seen && seen_flags) seen_flags[ag >> 3] = 1;
                }
            }
            *reinterpret_cast<uint4 *>(reached + 2 * ag) = make_uint4(0, 0, 0, 0);
            *reinterpret_cast<uint4 *>(reached + 2 * ag + 4) = make_uint4(0, 0, 0, 0);
        }
    }
    clear_frs_flags(flags, at >> 3, fl);
}

// *n += the non-zero 8-byte words of p[0 .. n_words): the check behind RAPIDGNN_CHECK_ZERO_MAPS
__global__ void count_nonzero_kernel(const unsigned long long *__restrict__ p, uint64_t n_words, unsigned long long *__restrict__ n)
{
    unsigned long long mine = 0;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_words; i += (uint64_t)gridDim.x * blockDim.x) mine += p[i] != 0ull;
    for (int o = 32; o > 0; o >>= 1) mine += __shfl_down(mine, o, 64);
    if ((threadIdx.x & 63) == 0 && mine) atomicAdd(n, mine);
}

// After the last hop: `seen` back to all-zero by clearing only the groups that hold bits (seen_flags), so that the
// bitmap can serve the next build without a memset of the whole map.  A thread owns eight groups.
__global__ void __launch_bounds__(FR_THREADS) clear_seen_kernel(uint32_t *__restrict__ seen, uint8_t *__restrict__ seen_flags, uint64_t n_flag_words, int paired)
{
    const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_flag_words) return;
    const unsigned long long fl = reinterpret_cast<const unsigned long long *>(seen_flags)[i];
    if (fl == 0ull) return;
#pragma unroll
    for (int g = 0; g < 8; ++g)
        if ((fl >> (8 * g)) & 0xFFull) {
            uint32_t *p = seen + (i * 8 + g) * (FR_WORDS_PER_THREAD << paired);
            *reinterpret_cast<uint4 *>(p) = make_uint4(0, 0, 0, 0);
            *reinterpret_cast<uint4 *>(p + 4) = make_uint4(0, 0, 0, 0);
        }
    reinterpret_cast<unsigned long long *>(seen_flags)[i] = 0ull;
}

// The large-graph form keeps no flags for `seen`: the IDs that were ever added to it are the frontier in front of the
// last hop (the last hop's own new IDs are not added), so their groups' `seen` halves of the paired records are
// cleared by walking that list -- one scattered 32-byte store per listed ID instead of a flag store per group in
// every emit pass plus a pass over all flags.
__global__ void clear_listed_seen_kernel(const int32_t *__restrict__ ids, const int64_t *__restrict__ off, uint32_t n_batches, int64_t n,
                                         uint64_t words_per_batch, uint32_t *__restrict__ seen /* the first record's `seen` half */)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const uint32_t b = batch_of(off, n_batches, i);
    const uint64_t word = (uint64_t)b * words_per_batch + ((uint32_t)ids[i] >> 5);
    uint32_t *p = seen + paired_word(word & ~(uint64_t)7);
    *reinterpret_cast<uint4 *>(p) = make_uint4(0, 0, 0, 0);
    *reinterpret_cast<uint4 *>(p + 4) = make_uint4(0, 0, 0, 0);
}

std::atomic<uint64_t> g_next_schedule_uid{1};        // also taken by schedules loaded from a file

static rg_status build_schedule_impl(const rg_graph *g, const int32_t *train, uint64_t T, uint32_t B, const uint32_t *fanout,
                                     uint32_t L, uint64_t s0, uint32_t worker, uint32_t epoch, uint32_t sampler, const rg_allocator *a, hipStream_t st, rg_schedule *s)
{
    const uint32_t beta = (uint32_t)(B ? (T + B - 1) / B : 0);
    s->n_nodes = g->n_nodes;
    s->n_batches = beta;
    s->L = L;
    s->T = T;
    s->uid = g_next_schedule_uid.fetch_add(1);
    s->hop.resize(L + 1);
    Arena tmp(a, st);         // build-time scratch, released (behind a drained stream) when this function returns

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
    unsigned long long *n_bad_train = nullptr, n_bad_host = 0;
    RG_TRY(tmp.dev_n<unsigned long long>(1, &n_bad_train));
    RG_HIP(hipMemsetAsync(n_bad_train, 0, sizeof(unsigned long long), st));
    if (T > 0) {
        uint32_t *once = nullptr;
        const uint64_t once_words = ((uint64_t)g->n_nodes + 31) / 32;
        RG_TRY(tmp.dev_n<uint32_t>(once_words, &once));
        RG_HIP(hipMemsetAsync(once, 0, once_words * sizeof(uint32_t), st));
        hipLaunchKernelGGL(check_train_kernel, dim3((unsigned)((T + 255) / 256)), dim3(256), 0, st, train, T, (int64_t)g->n_nodes, once, n_bad_train);
    }
    auto refuse_bad_train = [&]() -> rg_status {
        if (n_bad_host == 0) return RG_OK;
        set_error("rg_build_schedule: %llu of the %llu train nodes are outside [0, n_nodes) or repeated", n_bad_host, (unsigned long long)T);
        return RG_EINVAL;
    };
    if (T > 0) {
        // about a hundred positions per bucket, a power of two of buckets
        uint32_t bucket_bits = 0;
        while (bucket_bits < 20 && ((uint64_t)128 << bucket_bits) < T) ++bucket_bits;
        const uint64_t n_buckets = (uint64_t)1 << bucket_bits;
        KeyPos *kp = nullptr;
        int32_t *bucket_cnt = nullptr;
        int64_t *bucket_off = nullptr;
        RG_TRY(tmp.dev_n<KeyPos>(T, &kp));
        RG_TRY(tmp.dev_n<int32_t>(n_buckets, &bucket_cnt));
        RG_TRY(tmp.dev_n<int64_t>(n_buckets + 1, &bucket_off));
        RG_HIP(hipMemsetAsync(bucket_cnt, 0, n_buckets * sizeof(int32_t), st));
        {
            ScopedTimer tm(KG_SORT, st);
            const unsigned blocks = (unsigned)((T + 255) / 256);
            hipLaunchKernelGGL(shuffle_count_kernel, dim3(blocks), dim3(256), 0, st, s0, worker, epoch, T, bucket_bits, bucket_cnt);
            RG_TRY(scan_i32_to_i64(bucket_cnt, bucket_off, (int64_t)n_buckets, tmp, st));
            hipLaunchKernelGGL(shuffle_scatter_kernel, dim3(blocks), dim3(256), 0, st, s0, worker, epoch, T, bucket_bits, bucket_off, bucket_cnt, kp);
            hipLaunchKernelGGL(shuffle_rank_kernel, dim3((unsigned)n_buckets), dim3(RANK_THREADS), 0, st, kp, bucket_off, train, h0.ids);
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
    if (L == 0 || beta == 0) {
        Readback rb(st);
        RG_TRY(rb.add(&n_bad_host, n_bad_train, sizeof(n_bad_host)));
        RG_TRY(rb.wait());
        tmp.drained();
        return refuse_bad_train();
    }

    // ---- bitmaps (n_nodes bits per batch, rounded up to whole 8-word groups)
    const uint64_t wpb = (((uint64_t)g->n_nodes + 31) / 32 + FRS_WORDS_PER_THREAD - 1) / FRS_WORDS_PER_THREAD * FRS_WORDS_PER_THREAD;
    bool sparse_maps = wpb >= ((uint64_t)1 << 18);                           // 8.4 M nodes and up: a batch leaves most groups untouched
    if (const char *force = getenv("RAPIDGNN_SPARSE_FRONTIER")) sparse_maps = force[0] == '1';   // same results either way; for tests and tuning
    const uint32_t chunk_words = sparse_maps ? FRS_CHUNK_WORDS : FR_CHUNK_WORDS;
    const uint32_t chunks = (uint32_t)((wpb + chunk_words - 1) / chunk_words);
    // `reached` always as a bit per ID; where a byte per ID stays within the last-level cache's size (256 MB) a hop
    // may mark that form instead (sample_hop decides, and allocates it at the first such hop).  Both start out clear
    // and every hop's frontier pass clears what the hop marked.
    bool byte_map = !sparse_maps && wpb * 32 * (uint64_t)beta <= ((uint64_t)256 << 20);
    int prefer_bytes = -1;                             // -1: by the hop's own figures
    if (const char *force = getenv("RAPIDGNN_BYTE_MAPS")) {     // same results either way; for tests and tuning
        prefer_bytes = force[0] == '1';
        byte_map = prefer_bytes && !sparse_maps;
    }
    // The maps come from the pool of all-zero blocks and go back to it: every hop's frontier pass clears what the hop
    // marked in `reached` and its flags, and `seen` is cleared at the end group by group (seen_flags says which), so a
    // build clears what it touched, not n_batches * n_nodes bits (2 GB a map on a graph of 10^8 nodes).
    uint32_t *seen = nullptr, *reached_words = nullptr;
    uint8_t *reached_flags = nullptr;                  // one byte per group of 256 IDs of `reached`
    uint8_t *seen_flags = nullptr;                     // the same for `seen`: groups that hold any bit
    const uint64_t n_groups = wpb / FR_WORDS_PER_THREAD * beta;          // (a multiple of eight: wpb is a multiple of 64)
    uint32_t *paired = nullptr;                        // the large-graph form: both maps in one array of records (see paired_word)
    if (sparse_maps) {
        RG_TRY(tmp.dev_zeroed(2 * wpb * beta * sizeof(uint32_t), (void **)&paired, st));
        reached_words = paired;
        seen = paired + FR_WORDS_PER_THREAD;
    } else {
        RG_TRY(tmp.dev_zeroed(wpb * beta * sizeof(uint32_t), (void **)&seen, st));
        RG_TRY(tmp.dev_zeroed(wpb * beta * sizeof(uint32_t), (void **)&reached_words, st));
    }
    RG_TRY(tmp.dev_zeroed(n_groups, (void **)&reached_flags, st));
    if (!sparse_maps) RG_TRY(tmp.dev_zeroed(n_groups, (void **)&seen_flags, st));
    if (const char *check = getenv("RAPIDGNN_CHECK_ZERO_MAPS"); check && check[0] == '1') {
        // for tests: the maps, wherever they came from, really hold nothing but zeros (the pool of all-zero blocks keeps its promise)
        unsigned long long *n_dev = nullptr, n_host = 0;
        RG_TRY(tmp.dev_n<unsigned long long>(1, &n_dev));
        RG_HIP(hipMemsetAsync(n_dev, 0, sizeof(unsigned long long), st));
        const struct { const void *p; uint64_t bytes; } parts[4] = {{paired ? nullptr : seen, paired ? 0 : wpb * beta * 4}, {reached_words, wpb * beta * (paired ? 8u : 4u)},
                                                                    {reached_flags, n_groups}, {seen_flags, seen_flags ? n_groups : 0}};
        for (const auto &part : parts)
            if (part.bytes)
                hipLaunchKernelGGL(count_nonzero_kernel, dim3(1024), dim3(256), 0, st, (const unsigned long long *)part.p, part.bytes / 8, n_dev);
        Readback rb(st);
        RG_TRY(rb.add(&n_host, n_dev, sizeof(n_host)));
        RG_TRY(rb.wait());
        if (n_host != 0) { set_error("rg_build_schedule: %llu words of the per-batch maps are not zero at the start of the build", n_host); return RG_EHIP; }
    }
    ReachedForms maps{reached_words, nullptr, reached_flags, wpb, byte_map, paired != nullptr};
    {
        ScopedTimer tm(KG_FRONTIER, st);
        hipLaunchKernelGGL(mark_seeds_kernel, dim3((unsigned)((T + 255) / 256)), dim3(256), 0, st, h0.ids, T, B, seen, seen_flags, wpb, (int64_t)g->n_nodes, sparse_maps ? 1 : 0);
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

        // a3: the samples of this hop; sampled IDs are marked in `reached` as they are written
        bool marked_bytes = false;
        RG_TRY(sample_hop(g, cur, beta, batch_seed, l, fanout[l], sampler, maps, prefer_bytes, &marked_bytes, s->arena, tmp, n_cu, st,
                          l == 0 ? n_bad_train : nullptr, &n_bad_host));
        if (l == 0) RG_TRY(refuse_bad_train());
        void *reached = marked_bytes ? (void *)maps.bytes : (void *)reached_words;

        // a4: fresh IDs per (batch, chunk) -> positions -> next frontier
        RG_TRY(s->arena.dev_n<int64_t>((uint64_t)beta + 1, &nxt.off_dev));
        {
            ScopedTimer tm(KG_FRONTIER, st);
            if (sparse_maps)
                hipLaunchKernelGGL(fresh_count_sparse_kernel, dim3(chunks, beta), dim3(FR_THREADS), 0, st, reached_words, reached_flags, seen, wpb, chunks, fresh_cnt);
            else if (marked_bytes)
                hipLaunchKernelGGL(fresh_count_kernel<true>, dim3(chunks, beta), dim3(FR_THREADS), 0, st, reached, reached_flags, seen, wpb, chunks, fresh_cnt);
            else
                hipLaunchKernelGGL(fresh_count_kernel<false>, dim3(chunks, beta), dim3(FR_THREADS), 0, st, reached, reached_flags, seen, wpb, chunks, fresh_cnt);
            RG_TRY(scan_i32_to_i64(fresh_cnt, fresh_scan, (int64_t)n_cells, tmp, st));
            hipLaunchKernelGGL(next_offsets_kernel, dim3((beta + 1 + 255) / 256), dim3(256), 0, st, cur.off_dev, fresh_scan, beta, chunks, nxt.off_dev);
        }
        nxt.off_host.resize((size_t)beta + 1);
        {
            Readback rb(st);
            RG_TRY(rb.add(nxt.off_host.data(), nxt.off_dev, ((size_t)beta + 1) * sizeof(int64_t)));
            RG_TRY(rb.wait());
        }
        const int64_t n_next = nxt.off_host[beta];
        RG_TRY(s->arena.dev_n<int32_t>((uint64_t)n_next, &nxt.ids));
        {
            ScopedTimer tm(KG_FRONTIER, st);
            hipLaunchKernelGGL(copy_prefix_kernel, dim3((unsigned)((n_cur + 255) / 256)), dim3(256), 0, st, cur.ids, cur.off_dev, nxt.off_dev, beta, n_cur, nxt.ids);
            if (sparse_maps)
                hipLaunchKernelGGL(fresh_emit_sparse_kernel, dim3(chunks, beta), dim3(FR_THREADS), 0, st, reached_words, reached_flags, seen, seen_flags, wpb, chunks, fresh_scan, cur.off_dev, nxt.ids, l + 1 < L ? 1 : 0);
            else if (marked_bytes)
                hipLaunchKernelGGL(fresh_emit_kernel<true>, dim3(chunks, beta), dim3(FR_THREADS), 0, st, reached, reached_flags, seen, seen_flags, wpb, chunks, fresh_scan, cur.off_dev, nxt.ids);
            else
                hipLaunchKernelGGL(fresh_emit_kernel<false>, dim3(chunks, beta), dim3(FR_THREADS), 0, st, reached, reached_flags, seen, seen_flags, wpb, chunks, fresh_scan, cur.off_dev, nxt.ids);
        }
        RG_HIP(hipGetLastError());
    }
    // a6, first half: where the bitmaps are smaller than the lists of input nodes, the epoch's frequencies come from them
    if (!sparse_maps && beta < (1u << FREQ_PLANES) && wpb * (uint64_t)beta <= (uint64_t)s->hop[L].off_host[beta]) {
        RG_TRY(s->arena.dev_n<uint32_t>((uint64_t)g->n_nodes, &s->epoch_freq));
        ScopedTimer tm(KG_HIST, st);
        hipLaunchKernelGGL(epoch_freq_kernel, dim3((unsigned)((wpb + 255) / 256)), dim3(256), 0, st, seen, wpb, beta, (int64_t)g->n_nodes, s->epoch_freq);
        RG_HIP(hipGetLastError());
    }
    {
        // `seen` back to all-zero.  Clearing the flagged groups alone costs about eight times as much per group as a
        // fill costs per group of the whole map (scattered 32-byte stores against a streaming fill), and a group is
        // flagged by at least one input node: the fill wins unless fewer than an eighth of the groups can be flagged.
        ScopedTimer tm(KG_FRONTIER, st);
        if (paired) {
            const HopData &added = s->hop[L > 0 ? L - 1 : 0];          // every ID that was added to `seen`
            const int64_t listed = beta ? added.off_host[beta] : 0;
            if ((uint64_t)listed > n_groups / 4) {                    // (the fill covers both halves of the records)
                RG_HIP(hipMemsetAsync(paired, 0, 2 * n_groups * FR_WORDS_PER_THREAD * sizeof(uint32_t), st));
            } else if (listed > 0) {
                hipLaunchKernelGGL(clear_listed_seen_kernel, dim3((unsigned)((listed + 255) / 256)), dim3(256), 0, st, added.ids, added.off_dev, beta, listed, wpb, seen);
                RG_HIP(hipGetLastError());
            }
        } else {
            const uint64_t listed = L > 0 ? (uint64_t)s->hop[L].off_host[beta] : T;
            if (listed > n_groups / 8) {
                RG_HIP(hipMemsetAsync(seen, 0, n_groups * FR_WORDS_PER_THREAD * sizeof(uint32_t), st));
                RG_HIP(hipMemsetAsync(seen_flags, 0, n_groups, st));
            } else {
                hipLaunchKernelGGL(clear_seen_kernel, dim3((unsigned)((n_groups / 8 + FR_THREADS - 1) / FR_THREADS)), dim3(FR_THREADS), 0, st, seen, seen_flags, n_groups / 8, 0);
                RG_HIP(hipGetLastError());
            }
        }
    }
    RG_HIP(hipStreamSynchronize(st));
    tmp.drained();
    // every map is all-zero again and nothing writes them any more
    if (paired) tmp.free_zeroed(paired);
    else { tmp.free_zeroed(seen); tmp.free_zeroed(reached_words); }
    if (seen_flags) tmp.free_zeroed(seen_flags);
    tmp.free_zeroed(reached_flags);
    if (maps.bytes) tmp.free_zeroed(maps.bytes);
    return RG_OK;
}

}  // namespace rg

using namespace rg;

extern "C" rg_status rg_build_schedule(const rg_graph *g, const int32_t *train_nodes, uint64_t T, uint32_t batch_size,
                                       const uint32_t *fanout, uint32_t L, uint64_t s0, uint32_t worker, uint32_t epoch,
                                       const rg_allocator *a, void *stream, rg_schedule **out)
{
    return rg_build_schedule_with(g, train_nodes, T, batch_size, fanout, L, s0, worker, epoch, RG_SAMPLER_KEYS, a, stream, out);
}

extern "C" rg_status rg_build_schedule_with(const rg_graph *g, const int32_t *train_nodes, uint64_t T, uint32_t batch_size,
                                            const uint32_t *fanout, uint32_t L, uint64_t s0, uint32_t worker, uint32_t epoch,
                                            uint32_t sampler, const rg_allocator *a, void *stream, rg_schedule **out)
{
    if (sampler != RG_SAMPLER_KEYS && sampler != RG_SAMPLER_POSITIONS) { set_error("rg_build_schedule: unknown sampler %u", sampler); return RG_EINVAL; }
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
    if (T > 0 && (T + batch_size - 1) / batch_size > RG_MAX_BATCHES) {
        set_error("rg_build_schedule: %llu batches exceed RG_MAX_BATCHES = %u", (unsigned long long)((T + batch_size - 1) / batch_size), RG_MAX_BATCHES);
        return RG_ERANGE;
    }

    rg_schedule *s = new (std::nothrow) rg_schedule(a);
    if (!s) { set_error("rg_build_schedule: out of host memory"); return RG_ENOMEM; }
    rg_status rc = build_schedule_impl(g, train_nodes, T, batch_size, fanout, L, s0, worker, epoch, sampler, a, as_stream(stream), s);
    if (rc != RG_OK) {
        (void)hipStreamSynchronize(as_stream(stream));
        delete s;
        return rc;
    }
    *out = s;
    return RG_OK;
}
