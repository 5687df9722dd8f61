/*
 * rapidgnn.h -- C ABI of the MI355X (gfx950) data-path library for RapidGNN
 * (arXiv 2509.05207): deterministic seeded K-hop fan-out sampling of a whole
 * epoch's mini-batch schedule, the access-frequency tally and TopHot selection
 * that build the steady feature cache, and the per-batch feature-block gather.
 *
 * Conventions
 *  - Every function returns rg_status (0 = RG_OK, negative = error).  On error
 *    nothing is written through output handle pointers, and rg_last_error()
 *    describes the failure (thread-local, valid until the next call on this
 *    thread).  No exception crosses this boundary.
 *  - "dev" pointers are device (HBM) addresses on the current HIP device;
 *    "host" pointers are ordinary host addresses; "dev-visible" means either
 *    device memory or pinned host memory (hipHostMalloc) that kernels can read.
 *  - Node IDs are int32 (0 <= id < n_nodes < 2^31); row offsets and flat
 *    positions are int64; counts are uint32/uint64.  Epoch, batch, hop and
 *    worker indices are zero-based (the paper's text counts from 1).
 *  - The caller owns every input buffer and the gather output buffer.  Inputs
 *    are borrowed: the graph and train nodes only during rg_build_schedule;
 *    the rg_features arrays during rg_build_cache and every rg_gather_batch.
 *    Handles (rg_schedule, rg_cache) are owned by the library and released by
 *    the matching *_destroy, through the allocator they were created with.
 *  - Kernels are enqueued on the caller's hipStream_t (passed as void*; NULL =
 *    the default stream).  The build calls return after the stream has
 *    drained (they need sizes on the host); rg_gather_batch is asynchronous
 *    when it is served from a cache's prepared plan.
 */
#ifndef RAPIDGNN_H
#define RAPIDGNN_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t rg_status;
#define RG_OK        0
#define RG_EINVAL   (-1)   /* bad argument (null pointer, zero batch size, ...) */
#define RG_ENOMEM   (-2)   /* an allocation failed */
#define RG_EHIP     (-3)   /* a HIP runtime call failed */
#define RG_ERANGE   (-4)   /* a size is beyond a documented limit, or an output buffer is too small */
#define RG_EIO      (-5)   /* a schedule file cannot be opened, read or written, or its contents are not a schedule */

#define RG_MAX_HOPS    8u      /* L <= 8 */
#define RG_MAX_FANOUT  1984u   /* every fanout[l] <= 1984 */
#define RG_MAX_BATCHES 65535u  /* ceil(T / batch_size) <= 65535 batches per epoch */

const char *rg_last_error(void);

/* Optional allocator: lets the host framework own all memory (e.g. a caching
 * allocator).  kind 1 = device memory, kind 0 = pinned host memory.  alloc
 * returns NULL on failure.  Passing a NULL rg_allocator* selects
 * hipMalloc / hipHostMalloc. */
typedef struct rg_allocator {
    void *(*alloc)(uint64_t bytes, int kind, void *ctx);
    void (*free)(void *p, int kind, void *ctx);
    void *ctx;
} rg_allocator;

/* CSR adjacency the sampler reads (the graph structure this worker's sampler
 * sees, Sec. 2.3).  Precondition: within each row the
 * neighbour IDs are strictly ascending (sorted, duplicate free) and in
 * [0, n_nodes); rg_graph_validate checks it. */
typedef struct rg_graph {
    int64_t n_nodes;
    const int64_t *indptr;    /* dev, [n_nodes + 1], indptr[0] = 0, non-decreasing */
    const int32_t *indices;   /* dev, [indptr[n_nodes]] */
} rg_graph;

/* Checks the precondition above on the device.  *n_bad (host) receives the
 * number of violations (rows that decrease, neighbour out of range, indptr
 * decreasing); RG_OK is returned whenever the check itself ran. */
rg_status rg_graph_validate(const rg_graph *g, void *stream, uint64_t *n_bad);

typedef struct rg_schedule rg_schedule;
typedef struct rg_cache rg_cache;

/*
 * rg_build_schedule -- one epoch of the precomputed schedule (Alg. 1 step 1;
 * Sec. 3 "Offline enumeration and cache construction"; Sec. 4 par. (1)-(3)).
 *
 * Derives the per-batch seeds s_{e,i}^{(w)} = H(s0, worker, epoch, i)
 * (Sec. 3 "Seeding and reproducibility"), shuffles train_nodes with the
 * epoch's stream and cuts them into beta = ceil(T / batch_size) batches (the
 * last one may be partial), then for every batch runs the K-hop uniform
 * fan-out sampler: at hop l every node of the frontier U_l is sampled with
 * SAMPLE(eta(v), fanout[l]) (uniform, without replacement, min(deg, fanout[l])
 * neighbours, emitted in row order; fanout[0] applies to the seeds), and
 * U_{l+1} = U_l followed by the newly reached IDs in ascending order.  The
 * batch's input-node set N_i^e is U_L.  The result is a pure function of the
 * arguments: it does not depend on launch shape or timing.
 *
 *   g            graph (struct on host, arrays on device)
 *   train_nodes  dev, [T], distinct node IDs in [0, n_nodes); checked on the device, RG_EINVAL otherwise
 *   batch_size   > 0 (unless T == 0); ceil(T / batch_size) <= RG_MAX_BATCHES, RG_ERANGE otherwise
 *   fanout       host, [L]; L <= RG_MAX_HOPS, fanout[l] <= RG_MAX_FANOUT; L may be 0
 *   a            allocator or NULL
 *   out          receives the handle
 * Scratch, for the duration of the call: a bitmap of n_batches * n_nodes bits and
 * a map of the IDs a hop reaches, n_batches * n_nodes bytes if that is at most
 * 2 GiB (marks are then plain stores), else as many bits (marks are atomic ORs).
 * Environment: RAPIDGNN_SPARSE_FRONTIER=1 / 0 forces / forbids the frontier
 * passes tuned for graphs of 10^7 nodes and more (default: chosen from
 * n_nodes); RAPIDGNN_BYTE_MAPS=1 / 0 forces / forbids the byte form of the
 * reached map (never used together with those passes); RAPIDGNN_SHORT_ROWS=0 / 1 / 2
 * makes rows of up to 64 IDs be sampled one per wave / four at a time by a kernel
 * of their own / four at a time inside the main kernel (default: 1 in hops that
 * mark with byte stores, 2 in the others); RAPIDGNN_GROUP_TILES=1 / 0 forces /
 * forbids handing out the pieces of rows above 16,384 IDs grouped by the piece
 * they read, so that batches that share a row meet in the caches (default: from
 * 16,384 pieces on).  The result is the same in every case.  The maps are drawn from a pool of blocks known to be
 * all-zero and handed back to it after the build has cleared what it touched;
 * RAPIDGNN_CHECK_ZERO_MAPS=1 makes every build verify that on the device first.
 */
rg_status rg_build_schedule(const rg_graph *g, const int32_t *train_nodes, uint64_t T,
                            uint32_t batch_size, const uint32_t *fanout, uint32_t L,
                            uint64_t s0, uint32_t worker, uint32_t epoch,
                            const rg_allocator *a, void *stream, rg_schedule **out);

/* The same with a choice of SAMPLE's procedure.  The paper fixes the law of
 * SAMPLE (uniform, without replacement; Prop. 1(a)), not how it is drawn:
 *   RG_SAMPLER_KEYS       the f neighbours with the smallest hash keys, emitted
 *                         in row order; reads every row in full (O(deg)).
 *                         This is what rg_build_schedule uses.
 *   RG_SAMPLER_POSITIONS  f distinct positions of the row are drawn from the
 *                         node's state (selection without replacement for rows
 *                         up to 64, a keyed permutation of [0, deg) beyond) and
 *                         only those are read (O(f)); emitted in draw order.
 * Seeds, shuffle, frontier rule, counts and every other contract are the same;
 * the two procedures give different (equally distributed) samples.
 * RG_EINVAL for any other value. */
#define RG_SAMPLER_KEYS       0u
#define RG_SAMPLER_POSITIONS  1u
rg_status rg_build_schedule_with(const rg_graph *g, const int32_t *train_nodes, uint64_t T,
                                 uint32_t batch_size, const uint32_t *fanout, uint32_t L,
                                 uint64_t s0, uint32_t worker, uint32_t epoch, uint32_t sampler,
                                 const rg_allocator *a, void *stream, rg_schedule **out);

/* Read-only views ("metadata blocks": ordered batches, arrays N_i^e, offsets;
 * Sec. 4 par. (3)).  Device pointers stay valid until rg_schedule_destroy. */
rg_status rg_schedule_info(const rg_schedule *s, uint32_t *n_batches, uint32_t *L, int64_t *n_nodes);

/* Frontier U_hop of every batch, concatenated; hop in [0, L]; hop 0 = the
 * shuffled seeds, hop L = the input-node sets N_i^e.  batch_off has
 * n_batches + 1 entries and is given both on the device and on the host. */
rg_status rg_schedule_frontier(const rg_schedule *s, uint32_t hop, const int32_t **ids_dev,
                               const int64_t **batch_off_dev, const int64_t **batch_off_host);

/* The epoch's shuffled seeds (Sec. 3 "Seeding and reproducibility": the batches' seed nodes in the order the
 * epoch's stream puts them) and the batch offsets, [n_batches + 1]: the frontier of hop 0 under its own name. */
rg_status rg_schedule_seeds(const rg_schedule *s, const int32_t **seeds_dev, const int64_t **batch_off_dev);

/* Samples of hop in [0, L): samp_off_dev has |U_hop| + 1 entries indexed by
 * position in frontier(hop); node at position j drew
 * samp_nbr_dev[samp_off[j] .. samp_off[j+1]).  *n_samples = samp_off[|U_hop|]. */
rg_status rg_schedule_samples(const rg_schedule *s, uint32_t hop, const int64_t **samp_off_dev,
                              const int32_t **samp_nbr_dev, int64_t *n_samples);

/* The metadata block on storage (Sec. 4 par. (3): the precomputed schedule --
 * ordered batches, the arrays N_i^e, offsets, per-hop samples; no features --
 * is written out once and streamed back).  rg_schedule_save writes `s` to
 * `path` (device arrays pass through a 64 MiB pinned staging buffer, `stream`
 * is waited on); rg_schedule_load reads such a file into a new handle that
 * behaves like the schedule that was saved (computation blocks are rebuilt on
 * request, not stored).  A file is checked while it is read -- magic, header
 * ranges, offsets monotone and consistent between hops, every node ID inside
 * [0, n_nodes), exact length -- and refused with RG_EIO otherwise; nothing
 * is written through `out` then. */
rg_status rg_schedule_save(const rg_schedule *s, const char *path, void *stream);
rg_status rg_schedule_load(const char *path, const rg_allocator *a, void *stream, rg_schedule **out);

/* Streaming the metadata block (Sec. 4 par. (3): blocks are streamed from storage when they exceed memory):
 * batches [first_batch, first_batch + n_batches) of the schedule in `path` as a handle of their own, batch k of
 * the handle being batch first_batch + k of the file.  Only those batches' bytes are read (a batch range is a
 * contiguous slice of every array in the file) and only they occupy device memory, so an epoch that does not fit
 * is served range after range; caches, gathers and computation blocks take the handle like any other schedule.
 * Checked like rg_schedule_load (RG_EIO); RG_ERANGE if the range leaves the file's batches. */
rg_status rg_schedule_load_range(const char *path, uint32_t first_batch, uint32_t n_batches, const rg_allocator *a,
                                 void *stream, rg_schedule **out);

/* Feature storage, as byte rows (any element type): X[v] is
 * local_rows + row_of[v] * local_stride when is_local[v], else
 * remote_rows + row_of[v] * remote_stride (is_local marks N_local, the nodes whose rows this worker holds; Eq. 2).  The remote table stands for the other
 * partitions' memory behind VectorPull / SyncPull. */
typedef struct rg_features {
    const uint8_t *is_local;    /* dev, [n_nodes], 1 = local */
    const int32_t *row_of;      /* dev, [n_nodes] */
    const void *local_rows;     /* dev */
    uint64_t local_stride;      /* bytes, >= row_bytes */
    const void *remote_rows;    /* dev-visible: pinned host memory or device memory */
    uint64_t remote_stride;     /* bytes, >= row_bytes */
    uint32_t row_bytes;         /* bytes of one feature row, > 0 */
} rg_features;

/*
 * rg_build_cache -- Alg. 1 steps 2-4 (Eq. 2; Sec. 4 par. (5)-(6)).
 *
 * Tallies freq(v) = number of batches, over the given epochs, whose N_i^e
 * contains v; takes N_remote = {v : !is_local[v], freq(v) > 0}; selects
 * N_cache = the min(K, |N_remote|) members ranked first by (freq descending,
 * id ascending); pulls their rows from the remote table into a device table
 * (VectorPull; slot j holds the j-th smallest cached id); and prepares, for
 * every batch of every given epoch, the routing of each input node (local
 * table / cache slot / remote miss), the miss list M_i^e and the batch's
 * counts.
 *
 *   epochs    host array of n_epochs >= 1 schedule handles over the same n_nodes
 *   f         feature storage (borrowed for the life of the cache)
 *   K         n_hot, the cache capacity in rows (0 = no row cached)
 * Device memory of the table: K_eff * round_up(row_bytes, 16) <= n_hot * d
 * (one buffer of the bound in Sec. 3 "Invariants and bounds").  Beside it the
 * cache keeps a map from node to slot (half a byte per node: which IDs are
 * cached and local, and ranks) and the tally: 1 byte per node where the given
 * epochs have at most 255 batches together (no frequency can then exceed 255),
 * else 4.  Environment: RAPIDGNN_NARROW_TALLY=0 forbids the byte form (same
 * results either way).  The fill of the table runs on a stream the library
 * owns, beside the routing work on `stream`; the call returns after both.
 */
rg_status rg_build_cache(const rg_schedule *const *epochs, uint32_t n_epochs, const rg_features *f,
                         uint64_t K, const rg_allocator *a, void *stream, rg_cache **out);

/* Views of the cache: K_eff, the cached ids (dev, ascending), freq (dev,
 * [n_nodes]), slot_of (dev, [n_nodes], -1 = not cached), the table and its row
 * stride.  Any output pointer may be NULL.  The cache itself keeps slot_of as
 * a rank map and, where it could, the tally in bytes: the first call that asks
 * for slot_of (for freq) makes the array (4 bytes per node from the cache's
 * allocator, one kernel, waited for); calls that pass NULL for both never pay
 * for them.  Safe to call from several threads. */
rg_status rg_cache_view(const rg_cache *c, uint64_t *K_eff, const int32_t **cache_ids_dev,
                        const uint32_t **freq_dev, const int32_t **slot_of_dev,
                        const void **rows_dev, uint64_t *stride);

typedef struct rg_gather_stats {
    uint64_t n_rows;    /* |N_i^e| */
    uint64_t n_local;   /* served from the local table */
    uint64_t n_hit;     /* served from the steady cache C_s */
    uint64_t n_miss;    /* |M_i^e|: the batch's RPC count (Alg. 1 inner loop) */
} rg_gather_stats;

/*
 * rg_gather_batch -- the feature block of batch `batch` (Alg. 1 inner loop:
 * GetFeatureFromCache, M_i^e, SyncPull; Sec. 4 par. (7)):
 *     out[r, 0:row_bytes] = X[N_i^e[r], 0:row_bytes],  r < |N_i^e|,
 * bytes between row_bytes and out_stride are left untouched.  Local rows and
 * cache hits are read from HBM on `stream`; the miss set is pulled from the
 * remote table on `side_stream` (NULL = on `stream`) and joined back, so on
 * return all writes to `out` are ordered before later work on `stream`.
 * Routing never changes a byte of the result.
 *
 *   c      cache or NULL (no cache: every remote row is a miss).  If `s` is
 *          one of the epochs the cache was built from, the prepared plan is
 *          used and the call does not synchronise; otherwise rows are
 *          classified on the fly and the call waits for its counts.
 *   out    dev, out_capacity_rows * out_stride bytes; out_stride >= row_bytes
 *   stats  host or NULL; filled on return
 * RG_ERANGE if out_capacity_rows < |N_i^e| or batch >= n_batches (nothing is written).
 */
rg_status rg_gather_batch(const rg_schedule *s, const rg_cache *c, const rg_features *f, uint32_t batch,
                          void *out, uint64_t out_stride, uint64_t out_capacity_rows,
                          void *stream, void *side_stream, rg_gather_stats *stats);

/*
 * rg_gather_batches -- the blocks of batches [first_batch, first_batch + n_batches)
 * back to back: the block of batch b starts at row off[b] - off[first_batch] of
 * `out`, off being the batch offsets of rg_schedule_frontier(s, L).  Same bytes
 * as n_batches calls of rg_gather_batch (the prefetcher's "next Q batches" in
 * one go, Sec. 3 "Rolling prefetch and execution").  With a cache built from
 * `s` the range is one launch (plus one per batch with misses when the remote
 * table is pinned host memory); otherwise it runs batch by batch.
 *   stats  host, [n_batches], or NULL
 * RG_ERANGE if the range leaves the schedule or its rows exceed
 * out_capacity_rows (nothing is written).
 */
rg_status rg_gather_batches(const rg_schedule *s, const rg_cache *c, const rg_features *f, uint32_t first_batch,
                            uint32_t n_batches, void *out, uint64_t out_stride, uint64_t out_capacity_rows,
                            void *stream, void *side_stream, rg_gather_stats *stats);

/*
 * rg_gather_batch_noalloc -- rg_gather_batch for callers that cannot allocate:
 * code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same result as rg_gather_batch when the cache holds no prepared
 * plan for `s`: the batch's rows are classified on the fly (c == NULL: every
 * remote row is a miss) and every row is copied by one launch on `stream`,
 * remote rows read in place.  The routing entries and counters that
 * rg_gather_batch takes from an allocation live in a fixed array inside the
 * library's image instead, RG_NOALLOC_SCRATCH_BYTES per GPU the library runs
 * on, held until the process ends.  The call makes no hipMalloc / hipFree and
 * uses no allocator, block cache or event timer.
 *
 *   stats  host or NULL.  NULL: the call only enqueues kernels on `stream` (it
 *          may be recorded into a graph), and `s` and `c` must stay alive
 *          until that work has finished.  Otherwise the counts are copied back
 *          and the call waits for `stream`.
 * RG_ERANGE, with nothing written, if the batch has more than
 * RG_NOALLOC_MAX_ROWS rows, more than out_capacity_rows, or batch >= n_batches.
 * Every call on a GPU uses that GPU's one scratch array: calls on the same GPU
 * must be ordered (same stream, or otherwise serialised); two that overlap race.
 */
#define RG_NOALLOC_MAX_ROWS      ((uint64_t)1 << 22)                       /* 4,194,304 rows per batch */
#define RG_NOALLOC_SCRATCH_BYTES (256u + 8u * RG_NOALLOC_MAX_ROWS)         /* 32 MiB + 256 B */
rg_status rg_gather_batch_noalloc(const rg_schedule *s, const rg_cache *c, const rg_features *f, uint32_t batch,
                                  void *out, uint64_t out_stride, uint64_t out_capacity_rows, void *stream,
                                  rg_gather_stats *stats);

/* The counts of rg_gather_batch without the copy (Alg. 1 inner loop: the miss
 * set M_i^e and rpc_e += |M_i^e|): what a cache-size sweep needs.  From the
 * prepared plan when `c` was built from `s` (no device work), otherwise one
 * classification kernel on `stream` and a wait.  stats: host, required. */
rg_status rg_classify_batch(const rg_schedule *s, const rg_cache *c, const rg_features *f, uint32_t batch,
                            void *stream, rg_gather_stats *stats);

/* Release a handle.  Neither waits for the device: a handle that gathers enqueued by rg_gather_batch /
 * rg_gather_batches still read is released once exactly those have finished -- with a caller-supplied
 * allocator the call waits for them (and for nothing else), with the default allocator it returns at
 * once and a later library call lets go of the memory.  The device blocks then go to a per-process cache
 * that later builds draw from; rg_trim_memory() waits for every handle released so far and hands the
 * cached blocks back to the driver. */
void rg_schedule_destroy(rg_schedule *s);
void rg_cache_destroy(rg_cache *c);
void rg_trim_memory(void);

/* ------------------------------------------------------------------------
 * Computation blocks (Sec. 4 par. (8): the subgraph information of a batch is
 * gathered into the block the trainer runs on).  Block of hop l, batch b:
 *   destinations = U_l of the batch, sources = U_{l+1} of the batch (U_{l+1}
 *   starts with U_l, so destination j is source j), edges = the hop's samples.
 * rg_schedule_build_blocks computes, for every hop, src_pos[k] = the position
 * of samp_nbr[k] in its batch's U_{l+1}.  With samp_off (rg_schedule_samples)
 * this is the block's CSR in block-local indices; rows of the gathered feature
 * block (rg_gather_batch) are in source order of the outermost block.
 *   workspace_limit_bytes  device scratch for position tables, 4 * n_nodes
 *                          bytes per batch processed together; 0 = 4 GiB.
 *                          At least one batch's table is always allocated.
 * Waits for `stream`.  A second call is a no-op.  rg_schedule_block returns
 * RG_EINVAL before the blocks are built, RG_ERANGE for hop >= L.
 *   src_pos_dev  dev int32 [n_samples of the hop], owned by the schedule */
rg_status rg_schedule_build_blocks(rg_schedule *s, uint64_t workspace_limit_bytes, void *stream);
rg_status rg_schedule_block(const rg_schedule *s, uint32_t hop, const int32_t **src_pos_dev);

/* ------------------------------------------------------------------------
 * Double-buffered cache (Sec. 3 "Rolling prefetch and execution"; Alg. 1, the
 * secondary-cache build that runs beside an epoch and the swap at its end;
 * Sec. 4 par. (6)): a secondary cache C_sec is built from the next epoch's
 * schedule while the current epoch runs and takes over at the boundary if it
 * is ready by then.  Device bytes of
 * the two tables never exceed 2 * n_hot * row stride (Sec. 3, memory bound).
 *
 *   rg_cache_pair_create      builds C_s from `first_epoch` (as rg_build_cache with one epoch)
 *   rg_cache_pair_begin_next  starts building C_sec from `next_epoch` on a stream and a host
 *                             thread of the pair's own and returns at once; `next_epoch` and
 *                             the feature tables must stay alive until the swap (or destroy).
 *                             RG_EINVAL while a build is still running.
 *   rg_cache_pair_swap        at the epoch boundary.  wait == 0: swaps only if C_sec is ready,
 *                             otherwise C_s keeps serving (gathers of the new epoch then
 *                             classify on the fly: same bytes, more misses).  wait != 0: waits
 *                             for the build.  *swapped (host, may be NULL) says what happened.
 *                             The old C_s is released once the gathers that still read it have
 *                             finished; the call does not wait for them (staged blocks stay valid).
 *                             Returns the build's error if it failed.
 *   rg_cache_pair_primary     the current C_s: valid until the next successful swap
 *   rg_cache_pair_table_bytes device bytes held by C_s's table plus C_sec's, finished or under construction
 * One host thread drives a pair; the calls are not re-entrant. */
typedef struct rg_cache_pair rg_cache_pair;
rg_status rg_cache_pair_create(const rg_schedule *first_epoch, const rg_features *f, uint64_t K,
                               const rg_allocator *a, void *stream, rg_cache_pair **out);
rg_status rg_cache_pair_begin_next(rg_cache_pair *p, const rg_schedule *next_epoch);
rg_status rg_cache_pair_swap(rg_cache_pair *p, int wait, int *swapped);
const rg_cache *rg_cache_pair_primary(const rg_cache_pair *p);
uint64_t rg_cache_pair_table_bytes(const rg_cache_pair *p);
void rg_cache_pair_destroy(rg_cache_pair *p);

/* ------------------------------------------------------------------------
 * Rolling prefetch queue of depth Q (Sec. 3 "Rolling prefetch and execution";
 * Alg. 1, the prefetch of the next Q batches beside the batch loop; Sec. 4
 * par. (4), (7)): feature blocks of upcoming batches are staged, in schedule order, into
 * Q caller-owned device buffers by gathers on a stream of the prefetcher's
 * own; the consumer takes them in order.  Device memory for staged blocks is
 * Q * slot_capacity_rows * out_stride (the Q * m_max * d term of the bound).
 *
 *   slot_buffers   host array of Q device pointers, each slot_capacity_rows * out_stride bytes
 *   rg_prefetcher_fill     stages batches until staged + held slots == Q or the epoch ends
 *                          (back-pressure); asynchronous when `c` was built from `s`
 *   rg_prefetcher_acquire  the next batch in order: *out is its slot.  If it was staged,
 *                          consumer_stream is made to wait for the data (*was_staged = 1);
 *                          if not, it is gathered now on consumer_stream -- the default path
 *                          of Sec. 3 -- and *was_staged = 0.  RG_EINVAL if Q slots are held,
 *                          RG_ERANGE past the last batch.
 *   rg_prefetcher_release  the consumer's work queued so far on consumer_stream is the last
 *                          use of the oldest held slot; it may be refilled after that.
 * RG_ERANGE at create if a batch has more rows than a slot.  One host thread
 * drives a prefetcher; s, c and the feature tables are borrowed. */
typedef struct rg_prefetcher rg_prefetcher;
rg_status rg_prefetcher_create(const rg_schedule *s, const rg_cache *c, const rg_features *f, uint32_t Q,
                               void *const *slot_buffers, uint64_t out_stride, uint64_t slot_capacity_rows,
                               rg_prefetcher **out);
rg_status rg_prefetcher_fill(rg_prefetcher *p, uint32_t *issued /* host or NULL */);
rg_status rg_prefetcher_acquire(rg_prefetcher *p, void *consumer_stream, uint32_t *batch, void **out,
                                rg_gather_stats *stats, int *was_staged);
rg_status rg_prefetcher_release(rg_prefetcher *p, void *consumer_stream);
rg_status rg_prefetcher_depth(const rg_prefetcher *p, uint32_t *staged_not_acquired, uint32_t *held);
void rg_prefetcher_destroy(rg_prefetcher *p);

/* Timing aid for benchmarks: sums, since the last reset, the device time spent
 * in the named kernel group when profiling is enabled (HIP events around each
 * launch on the launch stream; adds a little latency).  Groups: 0 sampler
 * (the per-node sampling kernel alone), 1 frontier (mark/scan/emit), 2 shuffle
 * sort, 3 histogram, 4 top-K, 5 plan, 6 cache fill, 7 gather (HBM sources),
 * 8 gather (miss pull), 9 sample sizes and their prefix sum, 10 computation
 * blocks. */
#define RG_N_KERNEL_GROUPS 11
void rg_profile_enable(int on);
void rg_profile_reset(void);
rg_status rg_profile_read(double *ms /* host, [RG_N_KERNEL_GROUPS] */, uint64_t *launches /* host, same */);

#ifdef __cplusplus
}
#endif
#endif /* RAPIDGNN_H */
