// Micro-benchmarks behind figures quoted beside the library's kernels: what the memory system gives for the access
// patterns alone.  Built and run by `python -m paper_2509_05207_amd.microbench`; not part of librapidgnn_hip.so.
//   mb_copy    a plain streaming copy (16-byte loads and stores, four or eight per thread in flight)
//   mb_fill    stores alone (16-byte, plain or nontemporal) and mb_read, loads alone: the one-directional rates a copy's
//              two halves are held to
//   mb_marks   the sampler's marking traffic alone: atomic ORs into per-batch bitmaps against byte stores into
//              per-batch byte maps, each with the flag byte per 256 IDs
//   mb_stream  the sampler's row reads alone: one wave per frontier node streams the node's adjacency row in aligned
//              1 KB blocks with the next block in flight, computes the key of every ID and keeps the minimum
// Every function returns the average milliseconds per launch (negative: a HIP error).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../csrc/rg_device.h"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <int U>
__global__ void __launch_bounds__(256) copy_kernel(const u32x4 *__restrict__ a, u32x4 *__restrict__ b, size_t n)
{
    const size_t nt = (size_t)gridDim.x * 256;
    for (size_t base = (size_t)blockIdx.x * 256 + threadIdx.x; base < n; base += nt * U) {
        u32x4 v[U];
#pragma unroll
        for (int k = 0; k < U; ++k) { const size_t i = base + k * nt; if (i < n) v[k] = a[i]; }
#pragma unroll
        for (int k = 0; k < U; ++k) { const size_t i = base + k * nt; if (i < n) b[i] = v[k]; }
    }
}

template <bool NT>
__global__ void __launch_bounds__(256) fill_kernel(u32x4 *__restrict__ b, size_t n, uint32_t x)
{
    const size_t nt = (size_t)gridDim.x * 256;
    const u32x4 v = {x, x + 1u, x + 2u, x + 3u};
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += nt) {
        if (NT) __builtin_nontemporal_store(v, b + i);
        else b[i] = v;
    }
}

__global__ void __launch_bounds__(256) read_kernel(const u32x4 *__restrict__ a, size_t n, uint32_t *__restrict__ out)
{
    const size_t nt = (size_t)gridDim.x * 256;
    uint32_t acc = 0;
    for (size_t base = (size_t)blockIdx.x * 256 + threadIdx.x; base < n; base += nt * 4) {
        u32x4 v[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) { const size_t i = base + k * nt; v[k] = i < n ? a[i] : u32x4{0u, 0u, 0u, 0u}; }
#pragma unroll
        for (int k = 0; k < 4; ++k) acc ^= v[k].x ^ v[k].y ^ v[k].z ^ v[k].w;
    }
    if (acc == 0x12345678u) out[0] = acc;        // keeps the loads alive; practically never stores
}

// IDs with a power-law bias (popular nodes are hit often, like sampled neighbours); consecutive marks share a batch.
template <int MODE>
__global__ void marks_kernel(uint32_t *words, uint8_t *flags, uint8_t *bytes, uint64_t wpb, uint32_t n_nodes, uint32_t n_batches, uint64_t n)
{
    const uint64_t step = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += step) {
        const uint64_t h = rg::mix64(i + 1);
        const float x = (float)((uint32_t)(h >> 40)) * (1.0f / 16777216.0f);
        uint32_t u = (uint32_t)((double)n_nodes * x * x * x);
        if (u >= n_nodes) u = n_nodes - 1;
        u = (uint32_t)(((uint64_t)u * 2654435761ull) % n_nodes);
        const uint32_t b = (uint32_t)((i * n_batches) / n);
        if (MODE == 0) (void)__hip_atomic_fetch_or(&words[(uint64_t)b * wpb + (u >> 5)], 1u << (u & 31), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        else bytes[(uint64_t)b * (wpb << 5) + u] = 1;
        flags[(uint64_t)b * (wpb >> 3) + (u >> 8)] = 1;
    }
}

__device__ __forceinline__ int64_t lane_value64(int64_t x, int l)
{
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)x, l), hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)((uint64_t)x >> 32), l);
    return (int64_t)(((uint64_t)hi << 32) | lo);
}

// HASH = false: XOR of the IDs instead of their keys (the loads alone)
template <bool HASH>
__global__ void __launch_bounds__(64) stream_kernel(const int32_t *__restrict__ indices, const int64_t *__restrict__ row_begin, const int32_t *__restrict__ deg,
                                                    int64_t n, uint32_t *__restrict__ out)
{
    const int lane = threadIdx.x;
    const int64_t n_groups = (n + 63) >> 6;
    for (int64_t g = blockIdx.x; g < n_groups; g += gridDim.x) {
        const int64_t i_lane = (g << 6) + lane;
        const bool in = i_lane < n;
        const int64_t rb_lane = in ? row_begin[i_lane] : 0;
        const int deg_lane = in ? deg[i_lane] : 0;
        unsigned long long todo = __ballot(deg_lane > 0);
        uint32_t mine = 0;
        while (todo) {
            const int l = __builtin_amdgcn_readfirstlane(__ffsll((long long)todo) - 1);
            todo &= todo - 1;
            const int64_t rb = lane_value64(rb_lane, l);
            const int len = __builtin_amdgcn_readlane(deg_lane, l);
            const int32_t *row = indices + rb;
            const uint32_t lo = (uint32_t)rb * 2654435761u, hi = (uint32_t)len;
            uint32_t acc = HASH ? 0xFFFFFFFFu : 0u;
            auto use1 = [&](uint32_t u) { if (HASH) { const uint32_t k = rg::key32(lo, hi, u); acc = k < acc ? k : acc; } else acc ^= u; };
            int head = (32 - (int)(((uintptr_t)row >> 2) & 31)) & 31;
            if (head > len) head = len;
            if (lane < head) use1((uint32_t)row[lane]);
            const int32_t *p = row + head;
            const int rem = len - head, n_blocks = (rem + 255) >> 8;
            auto load = [&](int c) -> u32x4 {
                const int left = rem - c * 256, j = 4 * lane;
                const int32_t *q = p + c * 256;
                if (left >= 256 || j + 3 < left) return *reinterpret_cast<const u32x4 *>(q + j);
                u32x4 r = {0u, 0u, 0u, 0u};
                if (j < left) r.x = (uint32_t)q[j];
                if (j + 1 < left) r.y = (uint32_t)q[j + 1];
                if (j + 2 < left) r.z = (uint32_t)q[j + 2];
                return r;
            };
            u32x4 cur = {0u, 0u, 0u, 0u}, nxt = {0u, 0u, 0u, 0u};
            if (n_blocks > 0) cur = load(0);
            for (int c = 0; c < n_blocks; ++c) {
                if (c + 1 < n_blocks) nxt = load(c + 1);
                use1(cur.x); use1(cur.y); use1(cur.z); use1(cur.w);
                cur = nxt;
            }
            for (int o = 32; o > 0; o >>= 1) { const uint32_t y = __shfl_xor(acc, o, 64); acc = HASH ? (y < acc ? y : acc) : (acc ^ y); }
            if (lane == l) mine = acc;
        }
        if (in) out[i_lane] = mine;
    }
}

template <typename F>
float timed(F launch, int iters)
{
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return -1.f;
    launch();
    if (hipDeviceSynchronize() != hipSuccess) return -2.f;
    (void)hipEventRecord(e0, 0);
    for (int i = 0; i < iters; ++i) launch();
    (void)hipEventRecord(e1, 0);
    if (hipEventSynchronize(e1) != hipSuccess || hipGetLastError() != hipSuccess) return -3.f;
    float ms = 0;
    (void)hipEventElapsedTime(&ms, e0, e1);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    return ms / iters;
}

}  // namespace

extern "C" {

// a, b: device buffers of `bytes` bytes (a multiple of 16); unroll 4 or 8
float mb_copy(const void *a, void *b, uint64_t bytes, int unroll, int grid, int iters)
{
    const size_t n = bytes / 16;
    if (unroll == 8) return timed([&] { hipLaunchKernelGGL(copy_kernel<8>, dim3(grid), dim3(256), 0, 0, (const u32x4 *)a, (u32x4 *)b, n); }, iters);
    return timed([&] { hipLaunchKernelGGL(copy_kernel<4>, dim3(grid), dim3(256), 0, 0, (const u32x4 *)a, (u32x4 *)b, n); }, iters);
}

// b: device buffer of `bytes` bytes (a multiple of 16); nontemporal != 0: stores that bypass the caches
float mb_fill(void *b, uint64_t bytes, int nontemporal, int grid, int iters)
{
    const size_t n = bytes / 16;
    if (nontemporal) return timed([&] { hipLaunchKernelGGL(fill_kernel<true>, dim3(grid), dim3(256), 0, 0, (u32x4 *)b, n, 7u); }, iters);
    return timed([&] { hipLaunchKernelGGL(fill_kernel<false>, dim3(grid), dim3(256), 0, 0, (u32x4 *)b, n, 7u); }, iters);
}

// a: device buffer of `bytes` bytes (a multiple of 16); out: one uint32
float mb_read(const void *a, uint64_t bytes, void *out, int grid, int iters)
{
    const size_t n = bytes / 16;
    return timed([&] { hipLaunchKernelGGL(read_kernel, dim3(grid), dim3(256), 0, 0, (const u32x4 *)a, n, (uint32_t *)out); }, iters);
}

// words: n_batches * wpb uint32; flags: n_batches * wpb / 8 bytes; bytes: n_batches * wpb * 32 bytes; wpb = words per batch,
// a multiple of 8 with wpb * 32 >= n_nodes.  mode 0: atomic OR + flag, 1: byte store + flag.
float mb_marks(void *words, void *flags, void *bytes, uint64_t wpb, uint32_t n_nodes, uint32_t n_batches, uint64_t n_marks, int mode, int iters)
{
    if (wpb * 32 < n_nodes || n_batches == 0 || n_nodes == 0) return -4.f;
    if (mode == 0) return timed([&] { hipLaunchKernelGGL(marks_kernel<0>, dim3(8192), dim3(256), 0, 0, (uint32_t *)words, (uint8_t *)flags, (uint8_t *)bytes, wpb, n_nodes, n_batches, n_marks); }, iters);
    return timed([&] { hipLaunchKernelGGL(marks_kernel<1>, dim3(8192), dim3(256), 0, 0, (uint32_t *)words, (uint8_t *)flags, (uint8_t *)bytes, wpb, n_nodes, n_batches, n_marks); }, iters);
}

// row_begin[i], deg[i]: the adjacency row of frontier node i inside `indices` (device arrays of n entries; every row inside
// the indices array, which must start on a 128-byte boundary); out: n uint32
float mb_stream(const int32_t *indices, const int64_t *row_begin, const int32_t *deg, int64_t n, uint32_t *out, int hash, int grid, int iters)
{
    if (hash) return timed([&] { hipLaunchKernelGGL(stream_kernel<true>, dim3(grid), dim3(64), 0, 0, indices, row_begin, deg, n, out); }, iters);
    return timed([&] { hipLaunchKernelGGL(stream_kernel<false>, dim3(grid), dim3(64), 0, 0, indices, row_begin, deg, n, out); }, iters);
}

}  // extern "C"
