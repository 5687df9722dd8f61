// Device-side helpers shared by the schedule kernels: the hash family, the
// batch lookup and the per-batch reached-ID bitmaps.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

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

// ---------------------------------------------------------------- drawn positions (the O(f) sampler)
// Position p_t of draw t among the deg > f slots of a row, for a node state s; p_0, p_1, ... are distinct.
//   deg <= 64: selection without replacement.  Draw k takes r_k = floor(u_k * (deg - k)), u_k the top 32 bits of
//              mix64(s + (k + 1) G) read as a fraction, and picks the r_k-th slot not picked by draws 0 .. k-1.
//              The lane of draw t replays draws 0 .. t over a 64-bit mask of taken slots.
//   deg > 64:  p_t = pi_s(t), pi_s a permutation of [0, deg): an alternating Feistel network on
//              n = bitlen(deg - 1) bits (left part n - n/2 bits, right part n/2 bits, six rounds, round value =
//              top 32 bits of mix64((s ^ other part) + (r + 1) G)), walked along its cycle until the value is
//              below deg.  The walk ends: the cycle through t comes back to t < deg.
__device__ __forceinline__ uint32_t draw32(uint64_t s, uint32_t k) { return (uint32_t)(mix64(s + (uint64_t)(k + 1u) * HG64) >> 32); }

__device__ __forceinline__ uint32_t feistel(uint32_t x, uint32_t n_bits, uint64_t s)
{
    const uint32_t hb = n_bits >> 1, ha = n_bits - hb;
    const uint32_t mask_a = (1u << ha) - 1u, mask_b = (1u << hb) - 1u;        // n_bits <= 31: both parts below 32 bits
    uint32_t a = x >> hb, b = x & mask_b;
#pragma unroll
    for (uint32_t r = 0; r < 6; ++r) {
        if ((r & 1u) == 0) a ^= (uint32_t)(mix64((s ^ (uint64_t)b) + (uint64_t)(r + 1u) * HG64) >> 32) & mask_a;
        else               b ^= (uint32_t)(mix64((s ^ (uint64_t)a) + (uint64_t)(r + 1u) * HG64) >> 32) & mask_b;
    }
    return (a << hb) | b;
}

// The r-th (from 0) set bit of m; m has more than r set bits.
__device__ __forceinline__ uint32_t nth_set_bit(uint64_t m, uint32_t r)
{
    uint32_t p = 0;
#pragma unroll
    for (uint32_t w = 32; w >= 1; w >>= 1) {
        const uint32_t c = (uint32_t)__popcll((m >> p) & ((1ull << w) - 1ull));
        if (r >= c) { r -= c; p += w; }
    }
    return p;
}

// Requires 1 <= deg, t < deg.
__device__ __forceinline__ uint32_t draw_position(uint32_t deg, uint32_t t, uint64_t s)
{
    if (deg <= 64u) {
        const uint64_t all = deg == 64u ? ~0ull : (1ull << deg) - 1ull;
        uint64_t taken = 0;
        uint32_t p = 0;
        for (uint32_t k = 0; k <= t; ++k) {
            const uint32_t r = __umulhi(draw32(s, k), deg - k);
            p = nth_set_bit(all & ~taken, r);
            taken |= 1ull << p;
        }
        return p;
    }
    const uint32_t n_bits = 32u - (uint32_t)__clz((int)(deg - 1u));
    uint32_t x = feistel(t, n_bits, s);
    while (x >= deg) x = feistel(x, n_bits, s);
    return x;
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

// ---------------------------------------------------------------- reached-ID maps
// Every sampled ID is marked in the batch's `reached` map; which of the reached IDs are new to the batch is decided
// afterwards, group by group, against the batch's `seen` bitmap.  The map comes in two forms.  As a byte per node ID,
// where a mark is a plain store of 1: nothing is read, nothing is atomic, and the memory system takes three to five
// times as many of them per second as of the other form -- but the map is eight times as large and its scattered
// stores reach memory as whole lines.  As a bit per node ID, where a mark is an atomic OR without return value.  The
// wave waits for neither; a hop uses the form that suits its traffic (see sample_hop).  Beside the map there is one
// flag byte per 256 IDs: the frontier passes read the flags and touch only the flagged groups, which on a graph of
// 10^8 nodes is a few per cent of the map.
// What a kernel does with a sampled ID (a template argument).  MARK_BYTES_ALL, MARK_BITS_ALL: the same forms without
// the flag store, for a hop that reaches nearly every group anyway; its caller sets every flag instead.
constexpr int MARK_NONE = 0, MARK_BITS = 1, MARK_BYTES = 2, MARK_BYTES_ALL = 3, MARK_BITS_ALL = 4;
struct ReachedForms {             // host side: the forms a schedule build holds
    uint32_t *words;              // [n_batches * words_per_batch]
    uint8_t *bytes;               // [n_batches * words_per_batch * 32]; NULL until the first hop that wants it
    uint8_t *flags;               // [n_batches * words_per_batch / 8]
    uint64_t words_per_batch;     // a multiple of 8
    bool bytes_allowed;           // the byte form is small enough to be worth having
    bool paired;                  // `words` holds a 64-byte record per group of 256 IDs: the group's eight words of `reached`,
                                  // then its eight words of `seen` (see paired_word)
};
struct ReachedMaps {              // the form one hop marks
    void *map;
    uint8_t *flags;
    uint64_t words_per_batch;
    uint32_t paired;              // 1: the bit form in paired records
};
struct ReachedOfBatch {
    void *map;
    uint8_t *flags;
    uint32_t paired;
};
// On graphs of 10^8 nodes a batch touches a few per cent of its groups, so the frontier passes read a group's words
// of `reached` and of `seen` from two unrelated places each time.  Paired, both lie in one 64-byte record: word w of
// a map that would hold both arrays apart is word paired_word(w) of the records (`seen`: eight words further on).
__host__ __device__ __forceinline__ uint64_t paired_word(uint64_t w) { return ((w >> 3) << 4) | (w & 7); }
template <int MARK>
__device__ __forceinline__ ReachedOfBatch reached_of(const ReachedMaps &m, uint32_t batch)
{
    const uint64_t step = (MARK == MARK_BYTES || MARK == MARK_BYTES_ALL) ? m.words_per_batch << 5 : m.words_per_batch << (2 + m.paired);       // bytes per batch
    return ReachedOfBatch{static_cast<uint8_t *>(m.map) + (uint64_t)batch * step, m.flags + (uint64_t)batch * (m.words_per_batch >> 3), m.paired};
}
template <int MARK>
__device__ __forceinline__ void mark_reached(const ReachedOfBatch &r, uint32_t u)
{
    if (MARK == MARK_NONE) return;
    if (MARK == MARK_BYTES_ALL) { static_cast<uint8_t *>(r.map)[u] = 1; return; }
    if (MARK == MARK_BYTES) static_cast<uint8_t *>(r.map)[u] = 1;
    else {
        const uint32_t w = u >> 5;
        (void)__hip_atomic_fetch_or(static_cast<uint32_t *>(r.map) + (r.paired ? (((w >> 3) << 4) | (w & 7)) : w), 1u << (u & 31), __ATOMIC_RELAXED,
                                    __HIP_MEMORY_SCOPE_AGENT);
    }
    if (MARK != MARK_BITS_ALL) r.flags[u >> 8] = 1;
}

}  // namespace rg
