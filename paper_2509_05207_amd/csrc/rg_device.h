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

// ---------------------------------------------------------------- reached-ID bitmaps
// Every sampled ID sets its bit in the batch's `reached` bitmap.  The OR needs no return value, so
// the wave never waits for it; which of the reached IDs are new to the batch is decided afterwards,
// word by word, against the batch's `seen` bitmap.
__device__ __forceinline__ void mark_reached(uint32_t *__restrict__ reached_b, uint32_t u)
{
    (void)__hip_atomic_fetch_or(&reached_b[u >> 5], 1u << (u & 31), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

}  // namespace rg
