// The metadata block of one epoch on storage (Sec. 4 par. (3): the precomputed schedule -- ordered batches, the
// arrays N_i^e, offsets -- is written out and streamed back by the prefetcher; no features in it).
//
// rg_schedule_save writes a schedule to a file, rg_schedule_load reads one back into HBM.  Layout, little endian:
//   "RGSCHED1", n_nodes i64, T u64, n_batches u32, L u32,
//   for hop 0..L:   batch_off i64[n_batches + 1], ids i32[batch_off[n_batches]]
//   for hop 0..L-1: samp_off i64[|U_hop| + 1],    samp_nbr i32[samp_off[|U_hop|]]   (after that hop's ids)
// Device arrays go through a pinned staging buffer in pieces, so neither side needs the whole schedule in host
// memory.  A loaded file is checked before anything on the device depends on it: offsets monotone and consistent,
// every ID inside [0, n_nodes).
#include "rg_internal.h"

#include <algorithm>
#include <atomic>
#include <cstdio>
#include <cstring>

namespace rg {

extern std::atomic<uint64_t> g_next_schedule_uid;      // rg_schedule.hip

static const char MAGIC[8] = {'R', 'G', 'S', 'C', 'H', 'E', 'D', '1'};
constexpr uint64_t STAGE_BYTES = (uint64_t)64 << 20;

struct File {
    FILE *f = nullptr;
    ~File() { if (f) fclose(f); }
};

static rg_status write_all(FILE *f, const void *p, uint64_t n)
{
    if (n && fwrite(p, 1, n, f) != n) { set_error("rg_schedule_save: write failed"); return RG_EIO; }
    return RG_OK;
}

static rg_status read_all(FILE *f, void *p, uint64_t n)
{
    if (n && fread(p, 1, n, f) != n) { set_error("rg_schedule_load: file is truncated"); return RG_EIO; }
    return RG_OK;
}

static rg_status device_to_file(FILE *f, const void *dev, uint64_t bytes, void *stage, hipStream_t st)
{
    for (uint64_t at = 0; at < bytes; at += STAGE_BYTES) {
        const uint64_t n = std::min<uint64_t>(STAGE_BYTES, bytes - at);
        RG_HIP(hipMemcpyAsync(stage, (const uint8_t *)dev + at, n, hipMemcpyDeviceToHost, st));
        RG_HIP(hipStreamSynchronize(st));
        RG_TRY(write_all(f, stage, n));
    }
    return RG_OK;
}

// check(piece, count, first_index) is called on every piece before it goes to the device; it may edit the piece
template <typename T, typename Check>
static rg_status file_to_device(FILE *f, void *dev, uint64_t count, void *stage, hipStream_t st, Check check)
{
    const uint64_t per = STAGE_BYTES / sizeof(T);
    for (uint64_t at = 0; at < count; at += per) {
        const uint64_t n = std::min<uint64_t>(per, count - at);
        RG_TRY(read_all(f, stage, n * sizeof(T)));
        RG_TRY(check((T *)stage, n, at));             // (may also rewrite the piece in place)
        RG_HIP(hipMemcpyAsync((T *)dev + at, stage, n * sizeof(T), hipMemcpyHostToDevice, st));
        RG_HIP(hipStreamSynchronize(st));            // the staging buffer is reused by the next piece
    }
    return RG_OK;
}

}  // namespace rg

using namespace rg;

extern "C" {

rg_status rg_schedule_save(const rg_schedule *s, const char *path, void *stream)
{
    if (!s || !path) { set_error("rg_schedule_save: null argument"); return RG_EINVAL; }
    hipStream_t st = as_stream(stream);
    File file;
    file.f = fopen(path, "wb");
    if (!file.f) { set_error("rg_schedule_save: cannot open %s for writing", path); return RG_EIO; }
    Arena tmp(s->arena.allocator(), st);      // the staging block goes back only behind a drained stream
    void *stage = nullptr;
    RG_TRY(tmp.pinned(STAGE_BYTES, &stage));
    RG_TRY(write_all(file.f, MAGIC, 8));
    const int64_t n_nodes = s->n_nodes;
    const uint64_t T = s->T;
    const uint32_t nb = s->n_batches, L = s->L;
    RG_TRY(write_all(file.f, &n_nodes, 8));
    RG_TRY(write_all(file.f, &T, 8));
    RG_TRY(write_all(file.f, &nb, 4));
    RG_TRY(write_all(file.f, &L, 4));
    for (uint32_t l = 0; l <= L; ++l) {
        const HopData &h = s->hop[l];
        RG_TRY(write_all(file.f, h.off_host.data(), ((uint64_t)nb + 1) * sizeof(int64_t)));
        const uint64_t n = (uint64_t)h.off_host[nb];
        RG_TRY(device_to_file(file.f, h.ids, n * sizeof(int32_t), stage, st));
        if (l < L) {
            RG_TRY(device_to_file(file.f, h.samp_off, (n + 1) * sizeof(int64_t), stage, st));
            RG_TRY(device_to_file(file.f, h.samp_nbr, (uint64_t)h.n_samples * sizeof(int32_t), stage, st));
        }
    }
    if (fflush(file.f) != 0) { set_error("rg_schedule_save: flush failed"); return RG_EIO; }
    return RG_OK;
}

// Batches [first_batch, first_batch + n_batches) of the file's schedule into a new handle (n_batches == UINT32_MAX:
// up to the file's last batch).  Only the bytes of those batches are read: a hop's arrays are one after the other in the
// file, a batch range is a contiguous slice of each, and where a slice starts follows from the batch offsets and from
// the last entry of the hop's sample offsets.
static rg_status load_range(const char *path, uint32_t first_batch, uint32_t n_batches, const rg_allocator *a, hipStream_t st, rg_schedule **out)
{
    File file;
    file.f = fopen(path, "rb");
    if (!file.f) { set_error("rg_schedule_load: cannot open %s", path); return RG_EIO; }
    // Sizes read from the file are trusted only as far as the file is long: nothing is allocated for data that is not there.
    if (fseek(file.f, 0, SEEK_END) != 0) { set_error("rg_schedule_load: cannot seek in %s", path); return RG_EIO; }
    const long end_pos = ftell(file.f);
    if (end_pos < 0 || fseek(file.f, 0, SEEK_SET) != 0) { set_error("rg_schedule_load: cannot seek in %s", path); return RG_EIO; }
    const uint64_t file_bytes = (uint64_t)end_pos;
    uint64_t cur = 0;                                   // where the next section of the file starts
    auto section_fits = [&](uint64_t count, uint64_t elem) -> bool { return cur <= file_bytes && count <= (file_bytes - cur) / elem; };
    auto seek_to = [&](uint64_t pos) -> rg_status {
        if (pos > file_bytes || fseek(file.f, (long)pos, SEEK_SET) != 0) { set_error("rg_schedule_load: file is truncated"); return RG_EIO; }
        return RG_OK;
    };
    char magic[8];
    int64_t n_nodes = 0;
    uint64_t T = 0;
    uint32_t nb = 0, L = 0;
    RG_TRY(read_all(file.f, magic, 8));
    if (memcmp(magic, MAGIC, 8) != 0) { set_error("rg_schedule_load: %s is not a schedule file", path); return RG_EIO; }
    RG_TRY(read_all(file.f, &n_nodes, 8));
    RG_TRY(read_all(file.f, &T, 8));
    RG_TRY(read_all(file.f, &nb, 4));
    RG_TRY(read_all(file.f, &L, 4));
    cur = 32;
    if (n_nodes < 0 || n_nodes >= ((int64_t)1 << 31) || L > RG_MAX_HOPS || nb > RG_MAX_BATCHES) {
        set_error("rg_schedule_load: header out of range (n_nodes %lld, L %u, n_batches %u)", (long long)n_nodes, L, nb);
        return RG_EIO;
    }
    if (first_batch > nb || (n_batches != UINT32_MAX && n_batches > nb - first_batch)) {
        set_error("rg_schedule_load_range: batches [%u, %u + %u) beyond the file's %u", first_batch, first_batch, n_batches, nb);
        return RG_ERANGE;
    }
    const uint32_t lo = first_batch, hi = n_batches == UINT32_MAX ? nb : first_batch + n_batches, mb = hi - lo;
    if (!section_fits(((uint64_t)nb + 1) * ((uint64_t)L + 1), sizeof(int64_t))) { set_error("rg_schedule_load: file is truncated"); return RG_EIO; }
    rg_schedule *s = new (std::nothrow) rg_schedule(a);
    if (!s) { set_error("rg_schedule_load: out of host memory"); return RG_ENOMEM; }
    struct Guard { rg_schedule *s; hipStream_t st; ~Guard() { if (s) { (void)hipStreamSynchronize(st); delete s; } } } guard{s, st};
    s->n_nodes = n_nodes; s->T = T; s->n_batches = mb; s->L = L;
    s->uid = g_next_schedule_uid.fetch_add(1);
    s->hop.resize((size_t)L + 1);
    Arena tmp(a, st);      // the staging block goes back only behind a drained stream
    void *stage = nullptr;
    RG_TRY(tmp.pinned(STAGE_BYTES, &stage));

    auto ids_in_range = [n_nodes](int32_t *p, uint64_t n, uint64_t) -> rg_status {
        for (uint64_t i = 0; i < n; ++i)
            if (p[i] < 0 || (int64_t)p[i] >= n_nodes) { set_error("rg_schedule_load: node ID %d outside [0, %lld)", p[i], (long long)n_nodes); return RG_EIO; }
        return RG_OK;
    };
    std::vector<int64_t> off((size_t)nb + 1), prev_off;
    for (uint32_t l = 0; l <= L; ++l) {
        HopData &h = s->hop[l];
        // the hop's batch offsets (all of them: they say where everything else is)
        if (!section_fits((uint64_t)nb + 1, sizeof(int64_t))) { set_error("rg_schedule_load: file is truncated (batch offsets of hop %u)", l); return RG_EIO; }
        RG_TRY(seek_to(cur));
        RG_TRY(read_all(file.f, off.data(), ((uint64_t)nb + 1) * sizeof(int64_t)));
        cur += ((uint64_t)nb + 1) * sizeof(int64_t);
        if (off[0] != 0) { set_error("rg_schedule_load: batch offsets of hop %u do not start at 0", l); return RG_EIO; }
        for (uint32_t b = 0; b < nb; ++b)
            if (off[b + 1] < off[b]) { set_error("rg_schedule_load: batch offsets of hop %u decrease", l); return RG_EIO; }
        if (l > 0)
            for (uint32_t b = 0; b < nb; ++b)
                if (off[b + 1] - off[b] < prev_off[b + 1] - prev_off[b]) {
                    set_error("rg_schedule_load: frontier of hop %u, batch %u is smaller than the one before", l, b);
                    return RG_EIO;
                }
        const uint64_t n = (uint64_t)off[nb];
        if (!section_fits(n, sizeof(int32_t))) { set_error("rg_schedule_load: file is truncated (frontier of hop %u)", l); return RG_EIO; }
        h.off_host.resize((size_t)mb + 1);
        for (uint32_t b = 0; b <= mb; ++b) h.off_host[b] = off[lo + b] - off[lo];
        const uint64_t first = (uint64_t)off[lo], m = (uint64_t)(off[hi] - off[lo]);        // the range's slice of the hop's frontier
        RG_TRY(s->arena.dev_n<int64_t>((uint64_t)mb + 1, &h.off_dev));
        RG_HIP(hipMemcpyAsync(h.off_dev, h.off_host.data(), ((uint64_t)mb + 1) * sizeof(int64_t), hipMemcpyHostToDevice, st));
        RG_HIP(hipStreamSynchronize(st));
        RG_TRY(s->arena.dev_n<int32_t>(m, &h.ids));
        RG_TRY(seek_to(cur + first * sizeof(int32_t)));
        RG_TRY((file_to_device<int32_t>(file.f, h.ids, m, stage, st, ids_in_range)));
        cur += n * sizeof(int32_t);
        if (l < L) {
            if (!section_fits(n + 1, sizeof(int64_t))) { set_error("rg_schedule_load: file is truncated (sample offsets of hop %u)", l); return RG_EIO; }
            int64_t so_first = 0, so_total = 0;          // the hop's first and last sample offset
            RG_TRY(seek_to(cur));
            RG_TRY(read_all(file.f, &so_first, sizeof(int64_t)));
            RG_TRY(seek_to(cur + n * sizeof(int64_t)));
            RG_TRY(read_all(file.f, &so_total, sizeof(int64_t)));
            if (so_first != 0 || so_total < 0) { set_error("rg_schedule_load: sample offsets are not a prefix sum"); return RG_EIO; }
            RG_TRY(s->arena.dev_n<int64_t>(m + 1, &h.samp_off));
            int64_t base = -1, last = 0;                 // the slice is rebased to start at 0; running check: never decreases, stays within the total
            auto offsets_ok = [&](int64_t *p, uint64_t cnt, uint64_t) -> rg_status {
                for (uint64_t i = 0; i < cnt; ++i) {
                    if (base < 0) { base = p[i]; last = p[i]; if (base < 0) { set_error("rg_schedule_load: sample offsets are not a prefix sum"); return RG_EIO; } }
                    if (p[i] < last || p[i] > so_total) { set_error("rg_schedule_load: sample offsets are not a prefix sum"); return RG_EIO; }
                    last = p[i];
                    p[i] -= base;
                }
                return RG_OK;
            };
            RG_TRY(seek_to(cur + first * sizeof(int64_t)));
            RG_TRY((file_to_device<int64_t>(file.f, h.samp_off, m + 1, stage, st, offsets_ok)));
            if (first == 0 && base != 0) { set_error("rg_schedule_load: sample offsets are not a prefix sum"); return RG_EIO; }
            h.n_samples = last - base;
            cur += (n + 1) * sizeof(int64_t);
            if (!section_fits((uint64_t)so_total, sizeof(int32_t))) { set_error("rg_schedule_load: file is truncated (samples of hop %u)", l); return RG_EIO; }
            RG_TRY(s->arena.dev_n<int32_t>((uint64_t)h.n_samples, &h.samp_nbr));
            RG_TRY(seek_to(cur + (uint64_t)base * sizeof(int32_t)));
            RG_TRY((file_to_device<int32_t>(file.f, h.samp_nbr, (uint64_t)h.n_samples, stage, st, ids_in_range)));
            cur += (uint64_t)so_total * sizeof(int32_t);
        }
        prev_off = off;
    }
    if (cur != file_bytes) { set_error(cur < file_bytes ? "rg_schedule_load: trailing bytes after the schedule" : "rg_schedule_load: file is truncated"); return RG_EIO; }
    RG_HIP(hipStreamSynchronize(st));
    guard.s = nullptr;
    *out = s;
    return RG_OK;
}

rg_status rg_schedule_load(const char *path, const rg_allocator *a, void *stream, rg_schedule **out)
{
    if (!path || !out) { set_error("rg_schedule_load: null argument"); return RG_EINVAL; }
    return load_range(path, 0, UINT32_MAX, a, as_stream(stream), out);
}

rg_status rg_schedule_load_range(const char *path, uint32_t first_batch, uint32_t n_batches, const rg_allocator *a, void *stream, rg_schedule **out)
{
    if (!path || !out) { set_error("rg_schedule_load_range: null argument"); return RG_EINVAL; }
    if (n_batches == UINT32_MAX) { set_error("rg_schedule_load_range: n_batches out of range"); return RG_ERANGE; }
    return load_range(path, first_batch, n_batches, a, as_stream(stream), out);
}

}  // extern "C"
