// Computation blocks (Sec. 4 par. (8): the sampled subgraph handed to the trainer).
//
// Block of hop l, batch b: destinations U_l of the batch, sources U_{l+1} of the batch (destination j is
// source j, since U_{l+1} starts with U_l), edges = the hop's samples.  What is computed here is the
// relabelling src_pos[k] = position of samp_nbr[k] in the batch's U_{l+1}; with samp_off it is the
// block's CSR in block-local indices, and the gathered feature block is already in source order.
//
// Method: a position table of n_nodes int32 per batch, filled by scattering j -> table[U_{l+1}[j]] and
// read back once per sampled edge.  Only entries written for the same batch are ever read (every
// sampled ID is in U_{l+1}), so the table is never cleared.  Batches are processed in groups sized to a
// workspace limit: with 288 GB of HBM one group usually covers the epoch.
#include "rg_internal.h"

#include <algorithm>

namespace rg {

constexpr int BLK_THREADS = 256;
constexpr int BLK_GRID_X = 32;          // workgroups per batch; each walks its share with a grid stride

// table[g][U_{l+1,b}[j]] = j for batch b = b_lo + g
__global__ void __launch_bounds__(BLK_THREADS) block_positions_kernel(const int32_t *__restrict__ ids, const int64_t *__restrict__ off, uint32_t b_lo,
                                                                      int64_t n_nodes, int32_t *__restrict__ table)
{
    const uint32_t g = blockIdx.y, b = b_lo + g;
    const int64_t u0 = off[b], n = off[b + 1] - u0;
    int32_t *t = table + (uint64_t)g * (uint64_t)n_nodes;
    for (int64_t j = (int64_t)blockIdx.x * BLK_THREADS + threadIdx.x; j < n; j += (int64_t)gridDim.x * BLK_THREADS)
    {
        const uint32_t v = (uint32_t)ids[u0 + j];
        if (v < (uint64_t)n_nodes) t[v] = (int32_t)j;
    }
}

// src_pos[k] = table[g][samp_nbr[k]] for the samples of batch b = b_lo + g
__global__ void __launch_bounds__(BLK_THREADS) block_relabel_kernel(const int32_t *__restrict__ samp_nbr, const int64_t *__restrict__ samp_off,
                                                                    const int64_t *__restrict__ off, uint32_t b_lo, int64_t n_nodes,
                                                                    const int32_t *__restrict__ table, int32_t *__restrict__ src_pos)
{
    const uint32_t g = blockIdx.y, b = b_lo + g;
    const int64_t k0 = samp_off[off[b]], k1 = samp_off[off[b + 1]];
    const int32_t *t = table + (uint64_t)g * (uint64_t)n_nodes;
    for (int64_t k = k0 + (int64_t)blockIdx.x * BLK_THREADS + threadIdx.x; k < k1; k += (int64_t)gridDim.x * BLK_THREADS) {
        const uint32_t u = (uint32_t)samp_nbr[k];
        src_pos[k] = u < (uint64_t)n_nodes ? t[u] : -1;
    }
}

}  // namespace rg

using namespace rg;

extern "C" {

rg_status rg_schedule_build_blocks(rg_schedule *s, uint64_t workspace_limit_bytes, void *stream)
{
    if (!s) { set_error("rg_schedule_build_blocks: null schedule"); return RG_EINVAL; }
    if (s->blocks_built) return RG_OK;
    hipStream_t st = as_stream(stream);
    const uint64_t per_batch = (uint64_t)std::max<int64_t>(s->n_nodes, 1) * sizeof(int32_t);
    if (workspace_limit_bytes == 0) workspace_limit_bytes = (uint64_t)4 << 30;
    const uint32_t group = (uint32_t)std::max<uint64_t>(1, std::min<uint64_t>(s->n_batches, workspace_limit_bytes / per_batch));
    Arena tmp(s->arena.allocator(), st);     // scratch from the allocator the schedule was built with
    int32_t *table = nullptr;
    if (s->n_batches > 0) RG_TRY(tmp.dev((uint64_t)group * per_batch, (void **)&table));
    for (uint32_t l = 0; l < s->L; ++l)           // every allocation before the first launch: no early return with kernels in flight
        if (!s->hop[l].src_pos) RG_TRY(s->arena.dev_n<int32_t>((uint64_t)s->hop[l].n_samples, &s->hop[l].src_pos));
    for (uint32_t l = 0; l < s->L; ++l) {
        HopData &h = s->hop[l];
        const HopData &nx = s->hop[l + 1];
        if (h.n_samples == 0) continue;
        ScopedTimer tm(KG_BLOCKS, st);
        for (uint32_t b_lo = 0; b_lo < s->n_batches; b_lo += group) {
            const uint32_t nb = std::min(group, s->n_batches - b_lo);
            hipLaunchKernelGGL(block_positions_kernel, dim3(BLK_GRID_X, nb), dim3(BLK_THREADS), 0, st, nx.ids, nx.off_dev, b_lo, s->n_nodes, table);
            hipLaunchKernelGGL(block_relabel_kernel, dim3(BLK_GRID_X, nb), dim3(BLK_THREADS), 0, st, h.samp_nbr, h.samp_off, h.off_dev, b_lo,
                               s->n_nodes, table, h.src_pos);
        }
    }
    RG_HIP(hipGetLastError());
    RG_HIP(hipStreamSynchronize(st));            // the table is released below
    tmp.drained();
    s->blocks_built = true;
    return RG_OK;
}

rg_status rg_schedule_block(const rg_schedule *s, uint32_t hop, const int32_t **src_pos_dev)
{
    if (!s) { set_error("rg_schedule_block: null schedule"); return RG_EINVAL; }
    if (hop >= s->L) { set_error("rg_schedule_block: hop %u >= L = %u", hop, s->L); return RG_ERANGE; }
    if (!s->blocks_built) { set_error("rg_schedule_block: call rg_schedule_build_blocks first"); return RG_EINVAL; }
    if (src_pos_dev) *src_pos_dev = s->hop[hop].src_pos;
    return RG_OK;
}

}  // extern "C"
