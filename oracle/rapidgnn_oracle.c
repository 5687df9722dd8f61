/*
 * rapidgnn_oracle.c -- CPU oracle for the RapidGNN data path.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain, slow, obviously-correct
 * definition that the HIP library is checked against.  It shares no code,
 * header, table or helper with the HIP path and must never be called from the
 * product path: only the tests, the smoke check and the benchmark's
 * cpu_baseline leg load it.
 *
 * What it computes (paper: RapidGNN, arXiv 2509.05207):
 *   - per-(worker, epoch, batch) seeds s_{e,i}^{(w)} = H(s0, w, e, i)
 *     (Sec. 3 "Seeding and reproducibility"; Sec. 4 par. (1));
 *   - the epoch's beta = ceil(T/B) batches and, per batch, the K-hop uniform
 *     fan-out sample and its input-node set N_i^e (Sec. 3 "Offline enumeration
 *     and cache construction"; Sec. 4 par. (2); Alg. 1 step 1);
 *   - freq(v) over the epoch's batches, N_remote, and
 *     N_cache = TopHot(N_remote, n_hot, freq) (Eq. 2; Alg. 1 steps 2-3;
 *     Sec. 4 par. (5));
 *   - the steady cache C_s = VectorPull(N_cache) (Alg. 1 step 4);
 *   - per batch: the feature block of N_i^e and the local / hit / miss split,
 *     |M_i^e| being the batch's RPC count (Sec. 3 "Invariants and bounds";
 *     Alg. 1 inner loop).
 *
 * Where the paper leaves a choice open the reading taken is stated at the
 * function.  Everything is written as the definition itself: full key lists,
 * qsort, stamp arrays, direct indexing.  No blocking, fusion or reordering.
 *
 * Pin status (tests/test_oracle_*.py, all CPU):
 *   - hash family H: the paper names no function and prints no value, so the
 *     VALUES are a reading.  Pinned by what the paper requires of H (Prop. 1:
 *     statistically independent uniform outputs): constants re-derived by
 *     integer square root, bijectivity by an independently written inverse,
 *     avalanche and uniformity statistics.
 *   - sampler: brute force (full sort of all keys in numpy) on small graphs,
 *     subset / size / no-duplicate invariants, Prop. 1(a) inclusion
 *     frequencies and pairwise inclusion, Prop. 1(b) decorrelation across
 *     (e, i, w, hop), row-permutation invariance.
 *   - position sampler (the O(f) alternative): the permutation property by
 *     enumeration, distinctness and range, the selection branch against a
 *     python re-statement with an explicit list of free positions, inclusion
 *     and pairwise-inclusion frequencies on both branches.
 *   - batching: the paper's worked example ceil(153431/1000) = 154.
 *   - frontier, freq, TopHot, gather, stats: python set / Counter / full
 *     lexsort / fancy indexing on the same inputs.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------ */
/* Hash family H (reading: 64-bit multiply / xor-shift mixer).         */
/* Constants: floor(2^64/phi); frac(sqrt 2)*2^64 made odd;             */
/* frac(sqrt 3)*2^64.  32-bit ones: the top words of the same numbers. */
/* ------------------------------------------------------------------ */
#define ORC_G64 0x9E3779B97F4A7C15ull
#define ORC_A64 0x6A09E667F3BCC909ull
#define ORC_B64 0xBB67AE8584CAA73Bull
#define ORC_G32 0x9E3779B9u
#define ORC_A32 0x6A09E667u
#define ORC_B32 0xBB67AE85u

uint64_t orc_mix64(uint64_t x)
{
    x ^= x >> 32;
    x *= ORC_A64;
    x ^= x >> 29;
    x *= ORC_B64;
    x ^= x >> 32;
    return x;
}

uint64_t orc_combine(uint64_t h, uint64_t x)
{
    return orc_mix64(h ^ orc_mix64(x + ORC_G64));
}

/* s_{e,i}^{(w)} = H(s0, w, e, i): fold the four words in, in that order. */
uint64_t orc_batch_seed(uint64_t s0, uint32_t w, uint32_t e, uint32_t i)
{
    uint64_t h = orc_mix64(s0 ^ ORC_G64);
    h = orc_combine(h, (uint64_t)w);
    h = orc_combine(h, (uint64_t)e);
    h = orc_combine(h, (uint64_t)i);
    return h;
}

/* One independent stream per hop of a batch, one per frontier node of a hop. */
uint64_t orc_hop_state(uint64_t batch_seed, uint32_t hop)
{
    return orc_combine(batch_seed, (uint64_t)hop + 1u);
}

uint64_t orc_node_state(uint64_t hop_state, int32_t v)
{
    return orc_combine(hop_state, (uint64_t)(uint32_t)v);
}

/* Key of neighbour u under node state s: 32-bit mixer keyed by both halves. */
uint32_t orc_key32(uint64_t s, int32_t u)
{
    uint32_t lo = (uint32_t)s, hi = (uint32_t)(s >> 32);
    uint32_t x = (uint32_t)u ^ lo;
    x *= ORC_G32;
    x ^= x >> 16;
    x += hi;
    x *= ORC_A32;
    x ^= x >> 15;
    x *= ORC_B32;
    x ^= x >> 16;
    return x;
}

/* The epoch-shuffle stream is separated from the batch streams by folding in
 * 2^32 + e where a batch seed folds in e (< 2^32). */
uint64_t orc_epoch_state(uint64_t s0, uint32_t w, uint32_t e)
{
    uint64_t h = orc_mix64(s0 ^ ORC_G64);
    h = orc_combine(h, (uint64_t)w);
    h = orc_combine(h, ((uint64_t)1 << 32) + (uint64_t)e);
    return h;
}

/* ------------------------------------------------------------------ */
/* Epoch batch list.  The paper only says an epoch has beta batches;   */
/* reading: shuffle the train nodes by sorting on a hash key of their  */
/* position (ties by position), cut into ceil(T/B) consecutive slices, */
/* last one partial.                                                   */
/* ------------------------------------------------------------------ */
typedef struct { uint64_t key; uint64_t t; } orc_kt;

static int cmp_kt(const void *a, const void *b)
{
    const orc_kt *x = (const orc_kt *)a, *y = (const orc_kt *)b;
    if (x->key != y->key) return x->key < y->key ? -1 : 1;
    if (x->t != y->t) return x->t < y->t ? -1 : 1;
    return 0;
}

int orc_epoch_seeds(const int32_t *train, uint64_t T, uint64_t s0, uint32_t w,
                    uint32_t e, int32_t *seeds_out)
{
    uint64_t P = orc_epoch_state(s0, w, e);
    orc_kt *a = (orc_kt *)malloc((T ? T : 1) * sizeof(orc_kt));
    if (!a) return -1;
    for (uint64_t t = 0; t < T; ++t) { a[t].key = orc_combine(P, t); a[t].t = t; }
    qsort(a, T, sizeof(orc_kt), cmp_kt);
    for (uint64_t t = 0; t < T; ++t) seeds_out[t] = train[a[t].t];
    free(a);
    return 0;
}

uint64_t orc_num_batches(uint64_t T, uint64_t B)
{
    return B ? (T + B - 1) / B : 0;
}

/* ------------------------------------------------------------------ */
/* SAMPLE(eta(v), f): uniform, without replacement, |.| = min(deg, f). */
/* Every neighbour u gets the composite (key32(s_v,u) << 32) | u; the  */
/* f smallest composites are the sample, emitted in row order.  A      */
/* bounded max-heap finds the f-th smallest composite (the cut); the   */
/* row is then walked once more and everything <= cut is emitted.      */
/* ------------------------------------------------------------------ */
static uint64_t composite(uint64_t s, int32_t u)
{
    return ((uint64_t)orc_key32(s, u) << 32) | (uint64_t)(uint32_t)u;
}

static void heap_sift_down(uint64_t *h, uint32_t n, uint32_t i)
{
    for (;;) {
        uint32_t l = 2 * i + 1, r = l + 1, m = i;
        if (l < n && h[l] > h[m]) m = l;
        if (r < n && h[r] > h[m]) m = r;
        if (m == i) return;
        uint64_t t = h[i]; h[i] = h[m]; h[m] = t;
        i = m;
    }
}

/* heap: caller scratch of f entries.  Returns the number written to out. */
uint32_t orc_sample_row(const int32_t *row, int64_t deg, uint32_t f, uint64_t s,
                        uint64_t *heap, int32_t *out)
{
    if (f == 0 || deg <= 0) return 0;
    if (deg <= (int64_t)f) {
        for (int64_t j = 0; j < deg; ++j) out[j] = row[j];
        return (uint32_t)deg;
    }
    uint32_t n = 0;
    for (int64_t j = 0; j < deg; ++j) {
        uint64_t c = composite(s, row[j]);
        if (n < f) {
            heap[n++] = c;
            if (n == f)
                for (int32_t k = (int32_t)(f / 2); k >= 0; --k) heap_sift_down(heap, f, (uint32_t)k);
        } else if (c < heap[0]) {
            heap[0] = c;
            heap_sift_down(heap, f, 0);
        }
    }
    uint64_t cut = heap[0];
    uint32_t m = 0;
    for (int64_t j = 0; j < deg; ++j)
        if (composite(s, row[j]) <= cut) out[m++] = row[j];
    return m;
}

/* ------------------------------------------------------------------ */
/* Alternative SAMPLE for deg >> f: draw positions, read only those.   */
/* (The paper fixes the law -- uniform, without replacement -- not the */
/* procedure; this second reading costs O(f) per node instead of       */
/* O(deg).)  With deg > f, the sample is row[p_0], ..., row[p_{f-1}]   */
/* in draw order, where p_0.. are f distinct positions in [0, deg):    */
/*                                                                     */
/*  deg <= 64: sequential selection.  Draw t takes r_t uniform in      */
/*    [0, deg - t) (top 32 bits of mix64(s + (t+1)G), scaled by        */
/*    multiply-high) and picks the r_t-th position not picked before.  */
/*    Exactly uniform given uniform r_t.                               */
/*  deg > 64: p_t = pi_s(t), pi_s a keyed permutation of [0, deg):     */
/*    an alternating Feistel network on n = bitlen(deg-1) bits (left   */
/*    part n - n/2 bits, right part n/2 bits, six rounds, round value  */
/*    = top 32 bits of mix64((s ^ other half) + (r+1)G)), walked       */
/*    along its cycle until the value falls below deg.  A permutation  */
/*    restricted this way is a permutation of [0, deg); its first f    */
/*    images are distinct, and uniform as far as pi_s is random.       */
/* With deg <= f the whole row is the sample, in row order.            */
/* ------------------------------------------------------------------ */
static uint32_t draw32(uint64_t s, uint64_t t)
{
    return (uint32_t)(orc_mix64(s + (t + 1) * ORC_G64) >> 32);
}

uint64_t orc_feistel(uint64_t x, uint32_t n_bits, uint64_t s)
{
    const uint32_t hb = n_bits / 2, ha = n_bits - hb;
    const uint64_t mask_a = (1ull << ha) - 1, mask_b = (1ull << hb) - 1;
    uint64_t a = x >> hb, b = x & mask_b;
    for (uint32_t r = 0; r < 6; ++r) {
        if (r % 2 == 0) a ^= (orc_mix64((s ^ b) + (uint64_t)(r + 1) * ORC_G64) >> 32) & mask_a;
        else            b ^= (orc_mix64((s ^ a) + (uint64_t)(r + 1) * ORC_G64) >> 32) & mask_b;
    }
    return (a << hb) | b;
}

/* pos: f entries.  Requires deg > f >= 1. */
void orc_draw_positions(int64_t deg, uint32_t f, uint64_t s, int64_t *pos)
{
    if (deg <= 64) {
        uint8_t taken[64];
        memset(taken, 0, sizeof taken);
        for (uint32_t t = 0; t < f; ++t) {
            uint64_t r = ((uint64_t)draw32(s, t) * (uint64_t)(deg - t)) >> 32;
            int64_t p = 0;
            for (;; ++p) {
                if (taken[p]) continue;
                if (r == 0) break;
                --r;
            }
            taken[p] = 1;
            pos[t] = p;
        }
        return;
    }
    uint32_t n_bits = 0;
    while (((uint64_t)1 << n_bits) < (uint64_t)deg) ++n_bits;
    for (uint32_t t = 0; t < f; ++t) {
        uint64_t x = orc_feistel(t, n_bits, s);
        while (x >= (uint64_t)deg) x = orc_feistel(x, n_bits, s);
        pos[t] = (int64_t)x;
    }
}

/* pos_scratch: f entries.  Returns the number written to out. */
uint32_t orc_sample_row_positions(const int32_t *row, int64_t deg, uint32_t f, uint64_t s,
                                  int64_t *pos_scratch, int32_t *out)
{
    if (f == 0 || deg <= 0) return 0;
    if (deg <= (int64_t)f) {
        for (int64_t j = 0; j < deg; ++j) out[j] = row[j];
        return (uint32_t)deg;
    }
    orc_draw_positions(deg, f, s, pos_scratch);
    for (uint32_t t = 0; t < f; ++t) out[t] = row[pos_scratch[t]];
    return f;
}

/* ------------------------------------------------------------------ */
/* Schedule of one epoch.                                              */
/*   U_0 = the batch's seeds in shuffle order.                         */
/*   hop l: every v in U_l is sampled with fanout[l] (fan-outs count   */
/*   from the seeds outwards).                                         */
/*   U_{l+1} = U_l followed by the not-yet-present sampled IDs in      */
/*   ascending order.  N_i^e = U_L.                                    */
/* ------------------------------------------------------------------ */
typedef struct {
    int64_t  n_nodes;
    uint32_t n_batches, L;
    uint64_t T;
    int32_t *seeds;          /* [T] */
    int64_t *seeds_off;      /* [beta+1] */
    int32_t **fr_ids;        /* [L+1][...] frontier U_l, batches concatenated */
    int64_t **fr_off;        /* [L+1][beta+1] */
    int64_t **samp_off;      /* [L][|U_l| total + 1], by position in fr_ids[l] */
    int32_t **samp_nbr;      /* [L][...] */
} orc_schedule;

typedef struct { int32_t *p; int64_t n, cap; } vec32;
typedef struct { int64_t *p; int64_t n, cap; } vec64;

static int v32_push(vec32 *v, int32_t x)
{
    if (v->n == v->cap) {
        int64_t c = v->cap ? v->cap * 2 : 1024;
        int32_t *q = (int32_t *)realloc(v->p, (size_t)c * sizeof(int32_t));
        if (!q) return -1;
        v->p = q; v->cap = c;
    }
    v->p[v->n++] = x;
    return 0;
}

static int v64_push(vec64 *v, int64_t x)
{
    if (v->n == v->cap) {
        int64_t c = v->cap ? v->cap * 2 : 1024;
        int64_t *q = (int64_t *)realloc(v->p, (size_t)c * sizeof(int64_t));
        if (!q) return -1;
        v->p = q; v->cap = c;
    }
    v->p[v->n++] = x;
    return 0;
}

static int cmp_i32(const void *a, const void *b)
{
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return x < y ? -1 : (x > y ? 1 : 0);
}

/* per-batch result, before concatenation */
typedef struct {
    vec32 *fr;       /* [L+1] */
    vec64 *soff;     /* [L]  counts per frontier node (not yet prefix sums) */
    vec32 *snbr;     /* [L] */
    int err;
} batch_out;

static void build_one_batch(int64_t n_nodes, const int64_t *indptr, const int32_t *indices,
                            const int32_t *seeds, int64_t n_seeds, const uint32_t *fanout,
                            uint32_t L, uint64_t batch_seed, uint8_t *present,
                            int sampler, batch_out *o)
{
    (void)n_nodes;
    uint32_t fmax = 1;
    for (uint32_t l = 0; l < L; ++l) if (fanout[l] > fmax) fmax = fanout[l];
    uint64_t *heap = (uint64_t *)malloc((size_t)fmax * sizeof(uint64_t));
    int32_t *tmp = (int32_t *)malloc((size_t)fmax * sizeof(int32_t));
    int64_t *pos = (int64_t *)malloc((size_t)fmax * sizeof(int64_t));
    if (!heap || !tmp || !pos) { o->err = -1; free(heap); free(tmp); free(pos); return; }

    for (int64_t j = 0; j < n_seeds; ++j) {
        if (v32_push(&o->fr[0], seeds[j])) o->err = -1;
        present[seeds[j]] = 1;
    }
    for (uint32_t l = 0; l < L && !o->err; ++l) {
        uint64_t hs = orc_hop_state(batch_seed, l);
        vec32 fresh = {0, 0, 0};
        const vec32 *U = &o->fr[l];
        for (int64_t j = 0; j < U->n; ++j) {
            int32_t v = U->p[j];
            int64_t b = indptr[v], deg = indptr[v + 1] - b;
            uint64_t sv = orc_node_state(hs, v);
            uint32_t m = sampler == 1 ? orc_sample_row_positions(indices + b, deg, fanout[l], sv, pos, tmp)
                                      : orc_sample_row(indices + b, deg, fanout[l], sv, heap, tmp);
            if (v64_push(&o->soff[l], (int64_t)m)) o->err = -1;
            for (uint32_t k = 0; k < m; ++k) {
                if (v32_push(&o->snbr[l], tmp[k])) o->err = -1;
                if (!present[tmp[k]]) {
                    present[tmp[k]] = 1;
                    if (v32_push(&fresh, tmp[k])) o->err = -1;
                }
            }
        }
        qsort(fresh.p, (size_t)fresh.n, sizeof(int32_t), cmp_i32);
        for (int64_t j = 0; j < U->n; ++j) if (v32_push(&o->fr[l + 1], U->p[j])) o->err = -1;
        for (int64_t j = 0; j < fresh.n; ++j) if (v32_push(&o->fr[l + 1], fresh.p[j])) o->err = -1;
        free(fresh.p);
    }
    /* leave the stamp array clean for the next batch on this thread */
    for (uint32_t l = 0; l <= L; ++l)
        for (int64_t j = 0; j < o->fr[l].n; ++j) present[o->fr[l].p[j]] = 0;
    free(heap);
    free(tmp);
    free(pos);
}

void orc_schedule_destroy(orc_schedule *s)
{
    if (!s) return;
    free(s->seeds); free(s->seeds_off);
    if (s->fr_ids)  for (uint32_t l = 0; l <= s->L; ++l) free(s->fr_ids[l]);
    if (s->fr_off)  for (uint32_t l = 0; l <= s->L; ++l) free(s->fr_off[l]);
    if (s->samp_off) for (uint32_t l = 0; l < s->L; ++l) free(s->samp_off[l]);
    if (s->samp_nbr) for (uint32_t l = 0; l < s->L; ++l) free(s->samp_nbr[l]);
    free(s->fr_ids); free(s->fr_off); free(s->samp_off); free(s->samp_nbr);
    free(s);
}

/* batch_lo/batch_hi: build only batches [lo, hi) of the epoch (hi = 0 means
 * all); used to check sampled batches of big workloads and that a batch built
 * alone equals the same batch built inside the epoch.  n_threads: batches are
 * independent, so they may be built by several threads; results do not depend
 * on it.  sampler: 0 = the f smallest keys of the row (the main reading),
 * 1 = drawn positions (the O(f) alternative above). */
orc_schedule *orc_build_schedule_with(int64_t n_nodes, const int64_t *indptr, const int32_t *indices,
                                      const int32_t *train, uint64_t T, uint32_t batch_size,
                                      const uint32_t *fanout, uint32_t L, uint64_t s0, uint32_t worker,
                                      uint32_t epoch, uint32_t batch_lo, uint32_t batch_hi, int n_threads,
                                      int sampler)
{
    if (batch_size == 0 && T > 0) return NULL;
    orc_schedule *s = (orc_schedule *)calloc(1, sizeof(orc_schedule));
    if (!s) return NULL;
    uint32_t beta_all = (uint32_t)orc_num_batches(T, batch_size);
    if (batch_hi == 0 || batch_hi > beta_all) batch_hi = beta_all;
    if (batch_lo > batch_hi) batch_lo = batch_hi;
    uint32_t beta = batch_hi - batch_lo;
    s->n_nodes = n_nodes; s->L = L; s->n_batches = beta; s->T = T;

    int32_t *all_seeds = (int32_t *)malloc((T ? T : 1) * sizeof(int32_t));
    orc_epoch_seeds(train, T, s0, worker, epoch, all_seeds);

    batch_out *bo = (batch_out *)calloc(beta ? beta : 1, sizeof(batch_out));
    for (uint32_t b = 0; b < beta; ++b) {
        bo[b].fr = (vec32 *)calloc(L + 1, sizeof(vec32));
        bo[b].soff = (vec64 *)calloc(L ? L : 1, sizeof(vec64));
        bo[b].snbr = (vec32 *)calloc(L ? L : 1, sizeof(vec32));
    }
#ifdef _OPENMP
    if (n_threads < 1) n_threads = 1;
#pragma omp parallel num_threads(n_threads)
#endif
    {
        uint8_t *present = (uint8_t *)calloc((size_t)(n_nodes ? n_nodes : 1), 1);
#ifdef _OPENMP
#pragma omp for schedule(dynamic, 1)
#endif
        for (int64_t b = 0; b < (int64_t)beta; ++b) {
            uint64_t gi = (uint64_t)batch_lo + (uint64_t)b;       /* index within the epoch */
            uint64_t lo = gi * batch_size, hi = lo + batch_size;
            if (hi > T) hi = T;
            build_one_batch(n_nodes, indptr, indices, all_seeds + lo, (int64_t)(hi - lo), fanout, L,
                            orc_batch_seed(s0, worker, epoch, (uint32_t)gi), present, sampler, &bo[b]);
        }
        free(present);
    }
    (void)n_threads;

    /* concatenate */
    s->seeds_off = (int64_t *)calloc(beta + 1, sizeof(int64_t));
    s->fr_ids = (int32_t **)calloc(L + 1, sizeof(int32_t *));
    s->fr_off = (int64_t **)calloc(L + 1, sizeof(int64_t *));
    s->samp_off = (int64_t **)calloc(L ? L : 1, sizeof(int64_t *));
    s->samp_nbr = (int32_t **)calloc(L ? L : 1, sizeof(int32_t *));
    for (uint32_t l = 0; l <= L; ++l) {
        s->fr_off[l] = (int64_t *)calloc(beta + 1, sizeof(int64_t));
        for (uint32_t b = 0; b < beta; ++b) s->fr_off[l][b + 1] = s->fr_off[l][b] + bo[b].fr[l].n;
        int64_t tot = s->fr_off[l][beta];
        s->fr_ids[l] = (int32_t *)malloc((size_t)(tot ? tot : 1) * sizeof(int32_t));
        for (uint32_t b = 0; b < beta; ++b)
            memcpy(s->fr_ids[l] + s->fr_off[l][b], bo[b].fr[l].p, (size_t)bo[b].fr[l].n * sizeof(int32_t));
    }
    for (uint32_t b = 0; b <= beta; ++b) s->seeds_off[b] = s->fr_off[0][b];
    s->seeds = (int32_t *)malloc((size_t)(s->fr_off[0][beta] ? s->fr_off[0][beta] : 1) * sizeof(int32_t));
    memcpy(s->seeds, s->fr_ids[0], (size_t)s->fr_off[0][beta] * sizeof(int32_t));
    for (uint32_t l = 0; l < L; ++l) {
        int64_t tot_nodes = s->fr_off[l][beta];
        s->samp_off[l] = (int64_t *)calloc((size_t)tot_nodes + 1, sizeof(int64_t));
        int64_t k = 0, acc = 0;
        for (uint32_t b = 0; b < beta; ++b)
            for (int64_t j = 0; j < bo[b].soff[l].n; ++j) {
                s->samp_off[l][k++] = acc;
                acc += bo[b].soff[l].p[j];
            }
        s->samp_off[l][k] = acc;
        s->samp_nbr[l] = (int32_t *)malloc((size_t)(acc ? acc : 1) * sizeof(int32_t));
        int64_t w = 0;
        for (uint32_t b = 0; b < beta; ++b) {
            memcpy(s->samp_nbr[l] + w, bo[b].snbr[l].p, (size_t)bo[b].snbr[l].n * sizeof(int32_t));
            w += bo[b].snbr[l].n;
        }
    }
    int err = 0;
    for (uint32_t b = 0; b < beta; ++b) {
        err |= bo[b].err;
        for (uint32_t l = 0; l <= L; ++l) free(bo[b].fr[l].p);
        for (uint32_t l = 0; l < L; ++l) { free(bo[b].soff[l].p); free(bo[b].snbr[l].p); }
        free(bo[b].fr); free(bo[b].soff); free(bo[b].snbr);
    }
    free(bo);
    free(all_seeds);
    if (err) { orc_schedule_destroy(s); return NULL; }
    return s;
}

orc_schedule *orc_build_schedule(int64_t n_nodes, const int64_t *indptr, const int32_t *indices,
                                 const int32_t *train, uint64_t T, uint32_t batch_size,
                                 const uint32_t *fanout, uint32_t L, uint64_t s0, uint32_t worker,
                                 uint32_t epoch, uint32_t batch_lo, uint32_t batch_hi, int n_threads)
{
    return orc_build_schedule_with(n_nodes, indptr, indices, train, T, batch_size, fanout, L, s0, worker, epoch,
                                   batch_lo, batch_hi, n_threads, 0);
}

uint32_t orc_schedule_n_batches(const orc_schedule *s) { return s->n_batches; }
uint32_t orc_schedule_hops(const orc_schedule *s) { return s->L; }
int64_t orc_schedule_frontier_size(const orc_schedule *s, uint32_t hop) { return s->fr_off[hop][s->n_batches]; }
int64_t orc_schedule_samples_size(const orc_schedule *s, uint32_t hop)
{
    return s->samp_off[hop][s->fr_off[hop][s->n_batches]];
}
void orc_schedule_get_frontier(const orc_schedule *s, uint32_t hop, int32_t *ids, int64_t *batch_off)
{
    memcpy(ids, s->fr_ids[hop], (size_t)s->fr_off[hop][s->n_batches] * sizeof(int32_t));
    memcpy(batch_off, s->fr_off[hop], ((size_t)s->n_batches + 1) * sizeof(int64_t));
}
void orc_schedule_get_samples(const orc_schedule *s, uint32_t hop, int64_t *samp_off, int32_t *samp_nbr)
{
    int64_t n = s->fr_off[hop][s->n_batches];
    memcpy(samp_off, s->samp_off[hop], ((size_t)n + 1) * sizeof(int64_t));
    memcpy(samp_nbr, s->samp_nbr[hop], (size_t)s->samp_off[hop][n] * sizeof(int32_t));
}

/* ------------------------------------------------------------------ */
/* Computation block of hop l, batch b (Sec. 4 par. (8): the sampled   */
/* subgraph handed to the trainer).  Destination nodes are U_l of the  */
/* batch, source nodes are U_{l+1} of the batch; since U_{l+1} starts  */
/* with U_l, destination j is also source j.  The block's edges are    */
/* the hop's samples with every neighbour ID replaced by its position  */
/* in the batch's U_{l+1}: src_pos[k] = p  <=>  U_{l+1,b}[p] = nbr[k]. */
/* Returns 0, or -1 if a sampled ID is missing from U_{l+1} (never,    */
/* for a schedule built above) or memory ran out.                      */
/* ------------------------------------------------------------------ */
int orc_schedule_get_block(const orc_schedule *s, uint32_t hop, int32_t *src_pos)
{
    if (hop >= s->L) return -1;
    int32_t *where = (int32_t *)malloc(((size_t)s->n_nodes + 1) * sizeof(int32_t));
    if (!where) return -1;
    for (int64_t v = 0; v < s->n_nodes; ++v) where[v] = -1;
    int err = 0;
    for (uint32_t b = 0; b < s->n_batches && !err; ++b) {
        const int64_t u0 = s->fr_off[hop + 1][b], u1 = s->fr_off[hop + 1][b + 1];
        for (int64_t j = u0; j < u1; ++j) where[s->fr_ids[hop + 1][j]] = (int32_t)(j - u0);
        const int64_t k0 = s->samp_off[hop][s->fr_off[hop][b]], k1 = s->samp_off[hop][s->fr_off[hop][b + 1]];
        for (int64_t k = k0; k < k1; ++k) {
            const int32_t p = where[s->samp_nbr[hop][k]];
            if (p < 0) err = 1;
            src_pos[k] = p;
        }
        for (int64_t j = u0; j < u1; ++j) where[s->fr_ids[hop + 1][j]] = -1;
    }
    free(where);
    return err ? -1 : 0;
}

/* ------------------------------------------------------------------ */
/* freq(v) = number of batches whose input set N_i^e contains v        */
/* (a feature is fetched once per batch that needs it), over all the   */
/* epochs given.  Tallied for every ID; the remote filter is applied   */
/* at selection.                                                       */
/* ------------------------------------------------------------------ */
void orc_frequency(const orc_schedule *const *eps, uint32_t n_eps, int64_t n_nodes, uint32_t *freq)
{
    memset(freq, 0, (size_t)n_nodes * sizeof(uint32_t));
    for (uint32_t e = 0; e < n_eps; ++e) {
        const orc_schedule *s = eps[e];
        int64_t tot = s->fr_off[s->L][s->n_batches];
        for (int64_t j = 0; j < tot; ++j) freq[s->fr_ids[s->L][j]] += 1;
    }
}

/* TopHot: candidates are the remote IDs that occur at all (N_remote is a
 * subset of N); rank by (freq descending, id ascending); keep the first
 * min(K, #candidates); report them ascending by id, slot = position. */
typedef struct { uint32_t f; int32_t v; } orc_fv;

static int cmp_fv(const void *a, const void *b)
{
    const orc_fv *x = (const orc_fv *)a, *y = (const orc_fv *)b;
    if (x->f != y->f) return x->f > y->f ? -1 : 1;
    if (x->v != y->v) return x->v < y->v ? -1 : 1;
    return 0;
}

int64_t orc_top_hot(const uint32_t *freq, const uint8_t *is_local, int64_t n_nodes, uint64_t K,
                    int32_t *cache_ids /* cap >= min(K, n_nodes) */, int32_t *slot_of /* [n_nodes] */)
{
    orc_fv *c = (orc_fv *)malloc((size_t)(n_nodes ? n_nodes : 1) * sizeof(orc_fv));
    if (!c) return -1;
    int64_t nc = 0;
    for (int64_t v = 0; v < n_nodes; ++v)
        if (!is_local[v] && freq[v] > 0) { c[nc].f = freq[v]; c[nc].v = (int32_t)v; ++nc; }
    qsort(c, (size_t)nc, sizeof(orc_fv), cmp_fv);
    int64_t k_eff = (uint64_t)nc < K ? nc : (int64_t)K;
    for (int64_t j = 0; j < k_eff; ++j) cache_ids[j] = c[j].v;
    qsort(cache_ids, (size_t)k_eff, sizeof(int32_t), cmp_i32);
    for (int64_t v = 0; v < n_nodes; ++v) slot_of[v] = -1;
    for (int64_t j = 0; j < k_eff; ++j) slot_of[cache_ids[j]] = (int32_t)j;
    free(c);
    return k_eff;
}

/* X[v]: the feature row of node v, wherever it lives. */
static const uint8_t *feature_row(int32_t v, const uint8_t *is_local, const int32_t *row_of,
                                  const uint8_t *local_rows, uint64_t local_stride,
                                  const uint8_t *remote_rows, uint64_t remote_stride)
{
    return is_local[v] ? local_rows + (uint64_t)row_of[v] * local_stride
                       : remote_rows + (uint64_t)row_of[v] * remote_stride;
}

/* C_s[slot, :] = X[cache_ids[slot], :] */
void orc_cache_fill(const int32_t *cache_ids, int64_t k_eff, const uint8_t *is_local, const int32_t *row_of,
                    const uint8_t *local_rows, uint64_t local_stride, const uint8_t *remote_rows,
                    uint64_t remote_stride, uint32_t row_bytes, uint8_t *table, uint64_t table_stride)
{
    for (int64_t j = 0; j < k_eff; ++j)
        memcpy(table + (uint64_t)j * table_stride,
               feature_row(cache_ids[j], is_local, row_of, local_rows, local_stride, remote_rows, remote_stride),
               row_bytes);
}

/* out[r, 0:row_bytes] = X[N_i^e[r], 0:row_bytes]; bytes between row_bytes and
 * out_stride are not touched.  Where a row is served from (local table, cache,
 * remote) cannot change a byte, so the definition has no routing in it. */
int64_t orc_gather_batch(const orc_schedule *s, uint32_t batch, const uint8_t *is_local, const int32_t *row_of,
                         const uint8_t *local_rows, uint64_t local_stride, const uint8_t *remote_rows,
                         uint64_t remote_stride, uint32_t row_bytes, uint8_t *out, uint64_t out_stride)
{
    const int64_t *off = s->fr_off[s->L];
    const int32_t *ids = s->fr_ids[s->L] + off[batch];
    int64_t m = off[batch + 1] - off[batch];
    for (int64_t r = 0; r < m; ++r)
        memcpy(out + (uint64_t)r * out_stride,
               feature_row(ids[r], is_local, row_of, local_rows, local_stride, remote_rows, remote_stride),
               row_bytes);
    return m;
}

/* stats[0..3] = |N_i|, |N_i & local|, |N_i & N_cache|, |M_i| (the batch's RPC
 * count).  slot_of == NULL means no cache: every remote row is a miss. */
void orc_batch_stats(const orc_schedule *s, uint32_t batch, const uint8_t *is_local, const int32_t *slot_of,
                     uint64_t *stats)
{
    const int64_t *off = s->fr_off[s->L];
    const int32_t *ids = s->fr_ids[s->L] + off[batch];
    int64_t m = off[batch + 1] - off[batch];
    uint64_t n_local = 0, n_hit = 0, n_miss = 0;
    for (int64_t r = 0; r < m; ++r) {
        int32_t v = ids[r];
        if (is_local[v]) ++n_local;
        else if (slot_of && slot_of[v] >= 0) ++n_hit;
        else ++n_miss;
    }
    stats[0] = (uint64_t)m; stats[1] = n_local; stats[2] = n_hit; stats[3] = n_miss;
}

int orc_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
