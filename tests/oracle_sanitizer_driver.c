/*
 * Runs every entry point of the CPU oracle (oracle/rapidgnn_oracle.c) over one small workload and writes every
 * result to a file, so that the oracle can be exercised under AddressSanitizer / UndefinedBehaviorSanitizer as an
 * ordinary executable (tests/test_oracle_sanitizers.py builds this file together with the oracle's source with
 * -fsanitize=address,undefined and compares the output with what the ordinary build of the oracle returns).
 * Test infrastructure only; CPU only.
 *
 *   driver <dir> <n_threads>
 * reads <dir>/meta.txt and the raw arrays beside it, writes <dir>/out.bin.
 */
#include <inttypes.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

typedef struct orc_schedule orc_schedule;
orc_schedule *orc_build_schedule_with(int64_t n_nodes, const int64_t *indptr, const int32_t *indices, const int32_t *train, uint64_t T,
                                      uint32_t batch_size, const uint32_t *fanout, uint32_t L, uint64_t s0, uint32_t worker, uint32_t epoch,
                                      uint32_t batch_lo, uint32_t batch_hi, int n_threads, int sampler);
void orc_schedule_destroy(orc_schedule *s);
uint32_t orc_schedule_n_batches(const orc_schedule *s);
int64_t orc_schedule_frontier_size(const orc_schedule *s, uint32_t hop);
int64_t orc_schedule_samples_size(const orc_schedule *s, uint32_t hop);
void orc_schedule_get_frontier(const orc_schedule *s, uint32_t hop, int32_t *ids, int64_t *batch_off);
void orc_schedule_get_samples(const orc_schedule *s, uint32_t hop, int64_t *samp_off, int32_t *samp_nbr);
int orc_schedule_get_block(const orc_schedule *s, uint32_t hop, int32_t *src_pos);
void orc_frequency(const orc_schedule *const *eps, uint32_t n_eps, int64_t n_nodes, uint32_t *freq);
int64_t orc_top_hot(const uint32_t *freq, const uint8_t *is_local, int64_t n_nodes, uint64_t K, int32_t *cache_ids, int32_t *slot_of);
void orc_cache_fill(const int32_t *cache_ids, int64_t k_eff, const uint8_t *is_local, const int32_t *row_of, const uint8_t *local_rows,
                    uint64_t local_stride, const uint8_t *remote_rows, uint64_t remote_stride, uint32_t row_bytes, uint8_t *table,
                    uint64_t table_stride);
int64_t orc_gather_batch(const orc_schedule *s, uint32_t batch, const uint8_t *is_local, const int32_t *row_of, const uint8_t *local_rows,
                         uint64_t local_stride, const uint8_t *remote_rows, uint64_t remote_stride, uint32_t row_bytes, uint8_t *out,
                         uint64_t out_stride);
void orc_batch_stats(const orc_schedule *s, uint32_t batch, const uint8_t *is_local, const int32_t *slot_of, uint64_t *stats);

static void die(const char *what)
{
    fprintf(stderr, "oracle_sanitizer_driver: %s\n", what);
    exit(2);
}

static void *slurp(const char *dir, const char *name, size_t bytes)
{
    char path[4096];
    snprintf(path, sizeof(path), "%s/%s", dir, name);
    FILE *f = fopen(path, "rb");
    if (!f) die(path);
    void *p = malloc(bytes ? bytes : 1);
    if (!p || fread(p, 1, bytes, f) != bytes) die(path);
    fclose(f);
    return p;
}

static void put(FILE *f, const void *p, size_t bytes)
{
    if (bytes && fwrite(p, 1, bytes, f) != bytes) die("short write");
}

static void dump_schedule(FILE *out, const orc_schedule *s, uint32_t L, int blocks)
{
    const uint32_t nb = orc_schedule_n_batches(s);
    for (uint32_t hop = 0; hop <= L; ++hop) {
        const int64_t n = orc_schedule_frontier_size(s, hop);
        int32_t *ids = (int32_t *)malloc((size_t)(n ? n : 1) * sizeof(int32_t));
        int64_t *off = (int64_t *)malloc(((size_t)nb + 1) * sizeof(int64_t));
        orc_schedule_get_frontier(s, hop, ids, off);
        put(out, off, ((size_t)nb + 1) * sizeof(int64_t));
        put(out, ids, (size_t)n * sizeof(int32_t));
        free(ids); free(off);
    }
    for (uint32_t hop = 0; hop < L; ++hop) {
        const int64_t n = orc_schedule_frontier_size(s, hop), m = orc_schedule_samples_size(s, hop);
        int64_t *so = (int64_t *)malloc(((size_t)n + 1) * sizeof(int64_t));
        int32_t *nb32 = (int32_t *)malloc((size_t)(m ? m : 1) * sizeof(int32_t));
        orc_schedule_get_samples(s, hop, so, nb32);
        put(out, so, ((size_t)n + 1) * sizeof(int64_t));
        put(out, nb32, (size_t)m * sizeof(int32_t));
        if (blocks) {
            int32_t *pos = (int32_t *)malloc((size_t)(m ? m : 1) * sizeof(int32_t));
            if (orc_schedule_get_block(s, hop, pos) != 0) die("get_block failed");
            put(out, pos, (size_t)m * sizeof(int32_t));
            free(pos);
        }
        free(so); free(nb32);
    }
}

int main(int argc, char **argv)
{
    if (argc != 3) die("usage: driver <dir> <n_threads>");
    const char *dir = argv[1];
    const int n_threads = atoi(argv[2]);
    char path[4096];
    snprintf(path, sizeof(path), "%s/meta.txt", dir);
    FILE *mf = fopen(path, "r");
    if (!mf) die(path);
    int64_t n_nodes, n_edges, T, n_local, n_remote;
    uint32_t batch_size, L, worker, epoch, row_bytes;
    uint64_t s0, K, stride;
    uint32_t fanout[8];
    if (fscanf(mf, "%" SCNd64 " %" SCNd64 " %" SCNd64 " %" SCNu32 " %" SCNu32, &n_nodes, &n_edges, &T, &batch_size, &L) != 5 || L > 8) die("meta");
    for (uint32_t l = 0; l < L; ++l)
        if (fscanf(mf, "%" SCNu32, &fanout[l]) != 1) die("meta fanout");
    if (fscanf(mf, "%" SCNu64 " %" SCNu32 " %" SCNu32 " %" SCNu64 " %" SCNu32 " %" SCNu64 " %" SCNd64 " %" SCNd64, &s0, &worker, &epoch, &K,
               &row_bytes, &stride, &n_local, &n_remote) != 8) die("meta tail");
    fclose(mf);

    int64_t *indptr = (int64_t *)slurp(dir, "indptr.i64", ((size_t)n_nodes + 1) * 8);
    int32_t *indices = (int32_t *)slurp(dir, "indices.i32", (size_t)n_edges * 4);
    int32_t *train = (int32_t *)slurp(dir, "train.i32", (size_t)T * 4);
    uint8_t *is_local = (uint8_t *)slurp(dir, "is_local.u8", (size_t)n_nodes);
    int32_t *row_of = (int32_t *)slurp(dir, "row_of.i32", (size_t)n_nodes * 4);
    uint8_t *local = (uint8_t *)slurp(dir, "local.u8", (size_t)n_local * stride);
    uint8_t *remote = (uint8_t *)slurp(dir, "remote.u8", (size_t)n_remote * stride);

    snprintf(path, sizeof(path), "%s/out.bin", dir);
    FILE *out = fopen(path, "wb");
    if (!out) die(path);

    /* the main reading: whole pipeline */
    orc_schedule *s = orc_build_schedule_with(n_nodes, indptr, indices, train, (uint64_t)T, batch_size, fanout, L, s0, worker, epoch, 0, 0,
                                              n_threads, 0);
    if (!s) die("build_schedule failed");
    dump_schedule(out, s, L, 1);
    const uint32_t nb = orc_schedule_n_batches(s);
    uint32_t *freq = (uint32_t *)malloc((size_t)(n_nodes ? n_nodes : 1) * sizeof(uint32_t));
    const orc_schedule *eps[1] = {s};
    orc_frequency(eps, 1, n_nodes, freq);
    put(out, freq, (size_t)n_nodes * sizeof(uint32_t));
    const uint64_t cap = K < (uint64_t)n_nodes ? K : (uint64_t)n_nodes;
    int32_t *cache_ids = (int32_t *)malloc((size_t)(cap ? cap : 1) * sizeof(int32_t));
    int32_t *slot_of = (int32_t *)malloc((size_t)(n_nodes ? n_nodes : 1) * sizeof(int32_t));
    const int64_t k_eff = orc_top_hot(freq, is_local, n_nodes, K, cache_ids, slot_of);
    if (k_eff < 0) die("top_hot failed");
    put(out, &k_eff, sizeof(k_eff));
    put(out, cache_ids, (size_t)k_eff * sizeof(int32_t));
    put(out, slot_of, (size_t)n_nodes * sizeof(int32_t));
    uint8_t *table = (uint8_t *)calloc((size_t)(k_eff ? k_eff : 1) * stride, 1);
    orc_cache_fill(cache_ids, k_eff, is_local, row_of, local, stride, remote, stride, row_bytes, table, stride);
    put(out, table, (size_t)k_eff * stride);
    {
        const int64_t n_in = orc_schedule_frontier_size(s, L);
        int32_t *ids = (int32_t *)malloc((size_t)(n_in ? n_in : 1) * sizeof(int32_t));
        int64_t *off = (int64_t *)malloc(((size_t)nb + 1) * sizeof(int64_t));
        orc_schedule_get_frontier(s, L, ids, off);
        for (uint32_t b = 0; b < nb; ++b) {
            const int64_t m = off[b + 1] - off[b];
            uint8_t *rows = (uint8_t *)malloc((size_t)(m ? m : 1) * row_bytes);      /* exactly m * row_bytes: a byte too many is an overflow */
            if (orc_gather_batch(s, b, is_local, row_of, local, stride, remote, stride, row_bytes, rows, row_bytes) != m) die("gather size");
            put(out, rows, (size_t)m * row_bytes);
            free(rows);
            uint64_t st[4];
            orc_batch_stats(s, b, is_local, slot_of, st);
            put(out, st, sizeof(st));
            orc_batch_stats(s, b, is_local, NULL, st);
            put(out, st, sizeof(st));
        }
        free(ids); free(off);
    }
    orc_schedule_destroy(s);

    /* a batch built alone, and the second procedure of SAMPLE */
    if (nb > 1) {
        orc_schedule *one = orc_build_schedule_with(n_nodes, indptr, indices, train, (uint64_t)T, batch_size, fanout, L, s0, worker, epoch,
                                                    nb - 1, nb, 1, 0);
        if (!one) die("single batch failed");
        dump_schedule(out, one, L, 0);
        orc_schedule_destroy(one);
    }
    orc_schedule *sp = orc_build_schedule_with(n_nodes, indptr, indices, train, (uint64_t)T, batch_size, fanout, L, s0, worker, epoch, 0, 0,
                                               n_threads, 1);
    if (!sp) die("positions schedule failed");
    dump_schedule(out, sp, L, 0);
    orc_schedule_destroy(sp);

    fclose(out);
    free(freq); free(cache_ids); free(slot_of); free(table);
    free(indptr); free(indices); free(train); free(is_local); free(row_of); free(local); free(remote);
    return 0;
}
