/*
 * autohete_api.hip -- host side of libautohete.so: the C ABI declared in include/autohete.h.
 * Argument validation, the chunk layout, the workspace (device scratch + device copies of the
 * chunk tables, kept by content so that a list seen before is not uploaded again), and
 * the fp64 preparation of the per-launch constants.  All per-element work is in the kernels.
 */
#include <math.h>
#include <string.h>

#include <algorithm>
#include <new>
#include <vector>

#include "../../include/autohete.h"
#include "autohete_internal.h"

using ah::DevChunk;
using ah::GradResult;

struct autohete_ws {
    int device = 0;
    int n_cu = 0;
    uint64_t max_chunks = 0;
    /* Device copies of chunk tables, kept by content: a caller that cycles through a few chunk
     * lists (one per transformer block, or one per resident gradient buffer) uploads each list
     * once.  Least recently used entry is replaced. */
    struct Group { uint32_t first, rows; uint64_t max_tiles; }; /* rows [first, first+rows) share grid_x */
    struct Table {
        DevChunk *d = nullptr;
        std::vector<DevChunk> h;                /* what d holds */
        int kind = -1;                          /* which builder made it (layouts differ) */
        uint32_t tile_elems = 0;                /* ... and for which tile size */
        uint64_t hash = 0, last_use = 0;
        std::vector<Group> groups;              /* launch groups (step / cast tables) */
        uint64_t tiles = 0;                     /* all tiles of the table */
        hipEvent_t uploaded = nullptr;          /* the upload into d has completed */
        hipStream_t upload_stream = nullptr;
        bool upload_pending = false;
    };
    std::vector<Table> tables;
    DevChunk *d_tables = nullptr;               /* one allocation; tables[i].d points into it */
    uint64_t use_clock = 0;
    /* Pinned staging for the asynchronous uploads: a small ring, so that a caller that brings a
     * new chunk list with every call does not have to wait for the previous upload -- queued
     * behind earlier kernels -- before it can stage the next one. */
    static constexpr int kRing = 8;
    int ring_depth = 1;
    int ring_next = 0;
    DevChunk *h_stage[kRing] = {};
    hipEvent_t staged[kRing] = {};              /* upload from h_stage[i] has completed */
    bool staged_pending[kRing] = {};
    double *d_partials = nullptr;
    uint32_t *d_ticket = nullptr;
    GradResult *d_res = nullptr;
    GradResult *h_res = nullptr;                /* pinned read-back */
    int64_t tune_step_blocks_per_cu = 0, tune_prep_blocks = 0, tune_step_variant = 0, tune_cast_blocks_per_cu = 0;
    size_t lds_per_cu = 0;
    /* Norm carried INTO this workspace by autohete_adamw_step_carry calls: one fp64 slot per
     * wavefront of those calls, appended call after call and summed into d_res by one fold kernel
     * when the result is next needed.  Grown on demand, never shrunk. */
    double *d_wave_partials = nullptr;
    uint64_t wave_partials_cap = 0;
    uint64_t carried_slots = 0;                 /* written (or enqueued) but not folded yet */
    double carried_inv_scale = 1.0;             /* 1 / loss_scale of those slots */
};

namespace {

/* Encoding of AH_TUNE_STEP_VARIANT: vec | mode << 4 | (block / 64) << 8.
 * Default: 4 elements per lane, one wavefront per block, Newton fp64, at most 10 blocks per CU. */
constexpr int64_t kDefaultVariant = 4 | (0 << 4) | (1 << 8);
/* Default cap on resident update blocks per CU, by the elements one call covers.  The steady state
 * of a long launch is fastest at 10 (6.7 G elements: 9 -> 82.2, 10 -> 82.1, 11 -> 81.7, 12 -> 80.9 % of
 * peak); in shorter launches the ramp and the tail weigh more and one or two more resident waves pay
 * (1.3 G elements: 10 -> 82.3, 11 -> 83.2, 12 -> 82.8, 13 -> 81.9; 2.7 G: 10 -> 82.2, 11 -> 83.1,
 * 12 -> 82.7; 0.13 G: 8 -> 80.2, 10 -> 82.5, 12 -> 83.7, 14 -> 81.4, 16 -> 80.2). */
int default_blocks_per_cu(uint64_t call_elems)
{
    return call_elems < (1ull << 29) ? 12 : call_elems < (1ull << 32) ? 11 : 10;
}
/* The update without the 16-bit store (6.7 G elements: 10 -> 80.4, 11 -> 82.2, 12 -> 83.0, 14 -> 81.5). */
constexpr int kDefaultMasterBlocksPerCu = 12;
/* The norm-carrying update: its waves live a little longer, one more than the plain update, at most 12
 * (6.7 G elements in one call: 10 -> 28.9, 11 -> 28.5, 14 -> 29.0 ms; one transformer block (0.2 G) per
 * call: 10 -> 76.7, 11 -> 80.0, 12 -> 80.6, 13 -> 80.3, 14 -> 79.3 % of peak). */
int default_carry_blocks_per_cu(uint64_t call_elems) { return std::min(default_blocks_per_cu(call_elems) + 1, 12); }
constexpr int kDefaultCastBlocksPerCu = 24; /* measured: 64 -> 6.38, 24 -> 6.88, 16 -> 6.10 TB/s */

bool decode_variant(int64_t v, ah::StepVariant *out)
{
    if (v == 0) v = kDefaultVariant;
    ah::StepVariant s{(int)(v & 0xF), (int)((v >> 8) & 0xFF) * 64, (int)((v >> 4) & 0xF)};
    if ((v >> 16) || !ah::step_variant_valid(s)) return false;
    *out = s;
    return true;
}

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

/* Which streams of a chunk a call touches. */
enum : unsigned { kGrad = 1, kLowp = 2, kMaster = 4, kMom1 = 8, kMom2 = 16 };

int validate_chunk(const autohete_chunk &c, unsigned need)
{
    if (c.numel == 0) return AH_EINVAL;
    const void *ptr[5] = {c.grad, c.param_lp, c.master, c.exp_avg, c.exp_avg_sq};
    for (int i = 0; i < 5; ++i)
        if ((need >> i & 1u) && !ptr[i]) return AH_EINVAL;
    for (int i = 0; i < 5; ++i)
        if ((need >> i & 1u) && !aligned16(ptr[i])) return AH_EALIGN;
    return AH_OK;
}

void fill_row(DevChunk &d, const autohete_chunk &c, uint64_t tile_begin)
{
    d.grad = static_cast<const uint16_t *>(c.grad);
    d.param_lp = static_cast<uint16_t *>(c.param_lp);
    d.master = c.master;
    d.exp_avg = c.exp_avg;
    d.exp_avg_sq = c.exp_avg_sq;
    d.numel = c.numel;
    d.tile_begin = tile_begin;
    d.reserved = 0;
}

enum : int { kPrepTable = 0, kStepTable = 1 };

uint64_t table_hash(const std::vector<DevChunk> &tab, int kind, uint32_t tile_elems)
{
    uint64_t h = 0x9E3779B97F4A7C15ull ^ ((uint64_t)kind << 32 | tile_elems);
    const uint64_t *w = reinterpret_cast<const uint64_t *>(tab.data());
    const size_t n = tab.size() * (sizeof(DevChunk) / sizeof(uint64_t));
    for (size_t i = 0; i < n; ++i) {
        h = (h ^ w[i]) * 0xFF51AFD7ED558CCDull;
        h ^= h >> 29;
    }
    return h;
}

/* The device copy of `tab`: an entry that already holds exactly this content, else the least
 * recently used entry, overwritten by an upload enqueued on `stream`.  *fresh tells the caller
 * that it still has to fill in the entry's launch groups. */
int find_or_upload(autohete_ws *ws, int kind, uint32_t tile_elems, std::vector<DevChunk> &tab, hipStream_t stream,
                   autohete_ws::Table **out, bool *fresh)
{
    const uint64_t h = table_hash(tab, kind, tile_elems);
    autohete_ws::Table *lru = &ws->tables[0];
    for (autohete_ws::Table &t : ws->tables) {
        if (t.kind == kind && t.tile_elems == tile_elems && t.hash == h && t.h.size() == tab.size() &&
            memcmp(t.h.data(), tab.data(), tab.size() * sizeof(DevChunk)) == 0) {
            /* uploaded on another stream and perhaps still on its way: order this stream after it */
            if (t.upload_pending && t.upload_stream != stream) {
                if (hipEventQuery(t.uploaded) == hipSuccess) t.upload_pending = false;
                else if (hipStreamWaitEvent(stream, t.uploaded, 0) != hipSuccess) return AH_EHIP;
                (void)hipGetLastError(); /* hipErrorNotReady from the query is not an error */
            }
            t.last_use = ++ws->use_clock;
            *out = &t;
            *fresh = false;
            return AH_OK;
        }
        if (t.last_use < lru->last_use) lru = &t;
    }
    const int r = ws->ring_next;
    ws->ring_next = (r + 1) % ws->ring_depth;
    if (ws->staged_pending[r]) { /* an upload issued ring_depth misses ago may still read this buffer */
        if (hipEventSynchronize(ws->staged[r]) != hipSuccess) return AH_EHIP;
        ws->staged_pending[r] = false;
    }
    memcpy(ws->h_stage[r], tab.data(), tab.size() * sizeof(DevChunk));
    lru->kind = -1; /* not a valid entry until everything below has succeeded */
    if (hipMemcpyAsync(lru->d, ws->h_stage[r], tab.size() * sizeof(DevChunk), hipMemcpyHostToDevice, stream) !=
            hipSuccess ||
        hipEventRecord(ws->staged[r], stream) != hipSuccess || hipEventRecord(lru->uploaded, stream) != hipSuccess)
        return AH_EHIP;
    ws->staged_pending[r] = true;
    lru->h.swap(tab);
    lru->hash = h;
    lru->kind = kind;
    lru->tile_elems = tile_elems;
    lru->upload_stream = stream;
    lru->upload_pending = true;
    lru->groups.clear();
    lru->tiles = 0;
    lru->last_use = ++ws->use_clock;
    *out = lru;
    *fresh = true;
    return AH_OK;
}

/* Table of the prep kernel: rows in the caller's order, each with the index of its first tile;
 * row n is a sentinel holding the total tile count. */
int build_prep_table(autohete_ws *ws, const autohete_chunk *chunks, uint64_t n, uint32_t tile_elems,
                     hipStream_t stream, autohete_ws::Table **out)
{
    if (n > ws->max_chunks) return AH_ENOMEM;
    if (n && !chunks) return AH_EINVAL;
    std::vector<DevChunk> tab(n + 1);
    uint64_t tiles = 0;
    for (uint64_t i = 0; i < n; ++i) {
        int rc = validate_chunk(chunks[i], kGrad);
        if (rc != AH_OK) return rc;
        fill_row(tab[i], chunks[i], tiles);
        tiles += (chunks[i].numel + tile_elems - 1) / tile_elems;
    }
    memset(&tab[n], 0, sizeof(DevChunk));
    tab[n].tile_begin = tiles;
    bool fresh;
    int rc = find_or_upload(ws, kPrepTable, tile_elems, tab, stream, out, &fresh);
    if (rc == AH_OK && fresh) (*out)->tiles = tiles;
    return rc;
}

/* Table of the step kernel: one row per chunk, rows grouped by ceil(log2(tile count)) so that
 * each group can be launched as a 2-D grid (x = tile, y = row) in which at most half of the
 * blocks fall beyond the end of their chunk.  Equal-sized chunks form a single group. */
int build_step_table(autohete_ws *ws, const autohete_chunk *chunks, uint64_t n, uint32_t tile_elems,
                     uint32_t block_threads, unsigned need, hipStream_t stream, autohete_ws::Table **out)
{
    /* A launch may have at most 2^31 - 1 blocks along x and fewer than 2^32 threads along x; a chunk
     * with more tiles than that is refused here, before anything is launched for the call. */
    const uint64_t max_tiles = std::min<uint64_t>(0x7FFFFFFFull, 0xFFFFFFFFull / block_threads);
    if (n > ws->max_chunks) return AH_ENOMEM;
    if (n && !chunks) return AH_EINVAL;
    std::vector<uint64_t> tiles(n);
    std::vector<uint32_t> bucket(n);
    uint32_t count[65] = {0};
    for (uint64_t i = 0; i < n; ++i) {
        int rc = validate_chunk(chunks[i], need);
        if (rc != AH_OK) return rc;
        tiles[i] = (chunks[i].numel + tile_elems - 1) / tile_elems;
        if (tiles[i] > max_tiles) return AH_EINVAL; /* chunk too large for one launch of this kernel shape */
        bucket[i] = tiles[i] <= 1 ? 0 : 64 - (uint32_t)__builtin_clzll(tiles[i] - 1);
        ++count[bucket[i]];
    }
    uint32_t start[65];
    uint32_t run = 0;
    for (int b = 0; b < 65; ++b) {
        start[b] = run;
        run += count[b];
    }
    std::vector<DevChunk> tab(n + 1);
    std::vector<uint64_t> row_tiles(n);
    uint32_t fillpos[65];
    memcpy(fillpos, start, sizeof(start));
    for (uint64_t i = 0; i < n; ++i) {
        const uint32_t r = fillpos[bucket[i]]++;
        fill_row(tab[r], chunks[i], 0);
        row_tiles[r] = tiles[i];
    }
    uint64_t tile_run = 0; /* rows number their tiles consecutively in table order */
    for (uint64_t r = 0; r < n; ++r) {
        tab[r].tile_begin = tile_run;
        tile_run += row_tiles[r];
    }
    memset(&tab[n], 0, sizeof(DevChunk));
    tab[n].tile_begin = tile_run;
    std::vector<autohete_ws::Group> groups; /* built before the entry is touched: this may throw */
    for (int b = 0; b < 65; ++b) {
        for (uint32_t first = start[b]; first < start[b] + count[b]; first += 65535u) {
            const uint32_t rows = std::min<uint32_t>(65535u, start[b] + count[b] - first);
            uint64_t mx = 0;
            for (uint32_t r = first; r < first + rows; ++r) mx = std::max(mx, row_tiles[r]);
            groups.push_back({first, rows, mx});
        }
    }
    bool fresh;
    int rc = find_or_upload(ws, kStepTable, tile_elems, tab, stream, out, &fresh);
    if (rc != AH_OK || !fresh) return rc;
    (*out)->groups.swap(groups);
    (*out)->tiles = tile_run;
    return AH_OK;
}

/* Cap on resident blocks per CU, enforced through the dynamic LDS request: the launcher asks for
 * 1/cap of a CU's LDS per block (the kernels themselves use none).  cap >= 64: no request.  A block
 * may ask for at most 64 KB, so with 160 KB per CU the smallest cap this can express is 3
 * (53 KB per block); autohete_ws_tune refuses 1 and 2. */
constexpr int64_t kMinBlocksPerCu = 3;
constexpr size_t kLdsPerCuGfx950 = 160 * 1024;
unsigned lds_for_cap(const autohete_ws *ws, int64_t cap)
{
    if (cap >= 64 || !ws->lds_per_cu) return 0;
    size_t want = ws->lds_per_cu / (size_t)cap;
    want = want > 1024 ? want - 512 : want; /* stay clear of allocation-granule rounding */
    return (unsigned)std::min<size_t>(want, 64 * 1024);
}

struct DeviceGuard { /* run on the workspace's device, restore the caller's afterwards */
    int prev = -1;
    bool ok = false;
    explicit DeviceGuard(int dev)
    {
        if (hipGetDevice(&prev) != hipSuccess) return;
        ok = (prev == dev) || hipSetDevice(dev) == hipSuccess;
        if (prev == dev) prev = -1;
    }
    ~DeviceGuard()
    {
        if (ok && prev >= 0) (void)hipSetDevice(prev);
    }
};

/* Fold the carried slots into the workspace's result, on `stream` (which the caller has ordered
 * after the kernels that wrote them, as for any use of the result). */
int flush_carried(autohete_ws *ws, hipStream_t stream)
{
    if (!ws->carried_slots) return AH_OK;
    const uint64_t per_block = (uint64_t)ah::kThreads * 16;
    const uint64_t blocks = std::min<uint64_t>((uint64_t)ws->n_cu, (ws->carried_slots + per_block - 1) / per_block);
    const uint64_t n = ws->carried_slots;
    ws->carried_slots = 0;
    return ah::launch_fold((unsigned)blocks, stream, ws->d_wave_partials, n, ws->carried_inv_scale, ws->d_partials,
                           ws->d_ticket, ws->d_res) == hipSuccess
               ? AH_OK : AH_EHIP;
}

/* Room for `slots` more carried slots with the given scale; returns the index of the first.
 * When the buffer is full the pending slots are folded first; it then at least doubles, so that
 * after a few calls a whole iteration of per-block calls is folded by a single launch.  Growing
 * frees the old buffer, which waits for the device. */
int reserve_carried(autohete_ws *ws, uint64_t slots, double inv_scale, hipStream_t stream, uint64_t *base)
{
    if (ws->carried_slots && ws->carried_inv_scale != inv_scale) {
        int rc = flush_carried(ws, stream);
        if (rc != AH_OK) return rc;
    }
    if (ws->carried_slots + slots > ws->wave_partials_cap) {
        const uint64_t want = std::max(ws->carried_slots + slots, 2 * ws->wave_partials_cap);
        int rc = flush_carried(ws, stream);
        if (rc != AH_OK) return rc;
        if (ws->d_wave_partials) (void)hipFree(ws->d_wave_partials);
        ws->d_wave_partials = nullptr;
        ws->wave_partials_cap = 0;
        if (hipMalloc(&ws->d_wave_partials, want * sizeof(double)) != hipSuccess) {
            (void)hipGetLastError();
            return AH_ENOMEM;
        }
        ws->wave_partials_cap = want;
    }
    *base = ws->carried_slots;
    ws->carried_slots += slots;
    ws->carried_inv_scale = inv_scale;
    return AH_OK;
}

}  // namespace

extern "C" {

const char *autohete_strerror(int status)
{
    switch (status) {
        case AH_OK: return "ok";
        case AH_EINVAL: return "invalid argument";
        case AH_EALIGN: return "device pointer not 16-byte aligned";
        case AH_ENOMEM: return "out of memory or more chunks than the workspace holds";
        case AH_EHIP: return "HIP runtime error";
        case AH_EINFEASIBLE: return "no strategy satisfies the memory constraints";
        case AH_ELIMIT: return "more chunks than the allocation-free entry point takes";
        default: return "unknown status";
    }
}

int autohete_chunk_layout(const uint64_t *tensor_numel, uint64_t n_tensors, uint64_t chunk_elems,
                          uint64_t *tensor_offset, uint64_t *n_chunks, uint64_t *total_elems,
                          uint64_t *padded_elems)
{
    if (chunk_elems == 0 || !n_chunks || !total_elems || !padded_elems) return AH_EINVAL;
    if (n_tensors && !tensor_numel) return AH_EINVAL;
    uint64_t run = 0;
    for (uint64_t t = 0; t < n_tensors; ++t) {
        if (tensor_offset) tensor_offset[t] = run;
        if (__builtin_add_overflow(run, tensor_numel[t], &run)) return AH_EINVAL;
    }
    const uint64_t full = run / chunk_elems, rem = run % chunk_elems;
    *n_chunks = full + (rem ? 1 : 0);
    *total_elems = run;
    *padded_elems = rem ? chunk_elems - rem : 0;
    return AH_OK;
}

int autohete_ws_create(autohete_ws **out, uint64_t max_chunks)
{
    if (!out || max_chunks == 0 || max_chunks > (1u << 24)) return AH_EINVAL;
    *out = nullptr;
    autohete_ws *ws = new (std::nothrow) autohete_ws;
    if (!ws) return AH_ENOMEM;
    ws->max_chunks = max_chunks;
    hipDeviceProp_t prop;
    if (hipGetDevice(&ws->device) != hipSuccess || hipGetDeviceProperties(&prop, ws->device) != hipSuccess) {
        (void)hipGetLastError();
        delete ws;
        return AH_EHIP;
    }
    ws->n_cu = prop.multiProcessorCount;
    /* The residency caps divide the LDS of one CU.  This library is built for gfx950 only, whose CUs
     * have 160 KB; a runtime that reports less (the 64 KB a single block may use) would silently turn
     * a cap of 10 into 25. */
    ws->lds_per_cu = std::max<size_t>(prop.maxSharedMemoryPerMultiProcessor, kLdsPerCuGfx950);
    bool ok = true;
    const size_t tab_bytes = (max_chunks + 1) * sizeof(DevChunk);
    /* As many cached tables and staging buffers as fit a few MB, at least the two a prep + step pair
     * needs.  128 covers one table per transformer block and kernel for models of up to ~60 blocks; a
     * caller cycling through more lists than there are entries misses every time (least recently used). */
    const size_t n_tables = std::min<size_t>(128, std::max<size_t>(2, (8u << 20) / tab_bytes));
    ws->ring_depth = (int)std::min<size_t>(autohete_ws::kRing, std::max<size_t>(1, (4u << 20) / tab_bytes));
    try {
        ws->tables.resize(n_tables);
    } catch (...) {
        delete ws;
        return AH_ENOMEM;
    }
    ok = hipMalloc(&ws->d_tables, n_tables * tab_bytes) == hipSuccess; /* rows are 64 bytes: every table stays aligned */
    for (size_t i = 0; ok && i < n_tables; ++i) {
        ws->tables[i].d = ws->d_tables + i * (max_chunks + 1);
        ok = hipEventCreateWithFlags(&ws->tables[i].uploaded, hipEventDisableTiming) == hipSuccess;
    }
    for (int r = 0; ok && r < ws->ring_depth; ++r)
        ok = hipHostMalloc(&ws->h_stage[r], tab_bytes, hipHostMallocDefault) == hipSuccess &&
             hipEventCreateWithFlags(&ws->staged[r], hipEventDisableTiming) == hipSuccess;
    ok = ok && hipMalloc(&ws->d_partials, ah::kMaxPartials * sizeof(double)) == hipSuccess &&
         hipMalloc(&ws->d_ticket, 256) == hipSuccess && hipMalloc(&ws->d_res, 256) == hipSuccess &&
         hipHostMalloc(&ws->h_res, sizeof(GradResult), hipHostMallocDefault) == hipSuccess;
    if (!ok) {
        (void)hipGetLastError();
        autohete_ws_destroy(ws);
        return AH_ENOMEM;
    }
    /* The ticket must start at zero (each prep launch re-arms it); the result starts as
     * "no gradient seen": S = 0, no skip. */
    if (hipMemset(ws->d_ticket, 0, 256) != hipSuccess || hipMemset(ws->d_res, 0, 256) != hipSuccess ||
        hipDeviceSynchronize() != hipSuccess) {
        (void)hipGetLastError();
        autohete_ws_destroy(ws);
        return AH_EHIP;
    }
    *out = ws;
    return AH_OK;
}

int autohete_ws_destroy(autohete_ws *ws)
{
    if (!ws) return AH_EINVAL;
    DeviceGuard g(ws->device);
    (void)hipDeviceSynchronize();
    for (autohete_ws::Table &t : ws->tables)
        if (t.uploaded) (void)hipEventDestroy(t.uploaded);
    if (ws->d_tables) (void)hipFree(ws->d_tables);
    for (int r = 0; r < autohete_ws::kRing; ++r) {
        if (ws->h_stage[r]) (void)hipHostFree(ws->h_stage[r]);
        if (ws->staged[r]) (void)hipEventDestroy(ws->staged[r]);
    }
    if (ws->d_partials) (void)hipFree(ws->d_partials);
    if (ws->d_wave_partials) (void)hipFree(ws->d_wave_partials);
    if (ws->d_ticket) (void)hipFree(ws->d_ticket);
    if (ws->d_res) (void)hipFree(ws->d_res);
    if (ws->h_res) (void)hipHostFree(ws->h_res);
    delete ws;
    return AH_OK;
}

int autohete_ws_tune(autohete_ws *ws, int knob, int64_t value)
{
    if (!ws || value < 0) return AH_EINVAL;
    switch (knob) {
        case AH_TUNE_STEP_BLOCKS_PER_CU:
            if (value > 64 || (value && value < kMinBlocksPerCu)) return AH_EINVAL;
            ws->tune_step_blocks_per_cu = value;
            return AH_OK;
        case AH_TUNE_CAST_BLOCKS_PER_CU:
            if (value > 64 || (value && value < kMinBlocksPerCu)) return AH_EINVAL;
            ws->tune_cast_blocks_per_cu = value;
            return AH_OK;
        case AH_TUNE_CARRY_ELEMS: {
            /* Room for the per-wavefront partials that autohete_adamw_step_carry calls carry INTO this
             * workspace during one iteration over `value` elements: one slot per 64 * vec elements
             * (current step variant) plus, per chunk descriptor, the waves (at most 8) of one ragged last
             * tile -- with room for eight times max_chunks descriptors per iteration, since a chunk may
             * be cut into several descriptors by the per-block calls. */
            ah::StepVariant v;
            if (!decode_variant(ws->tune_step_variant, &v)) return AH_EINVAL;
            DeviceGuard g(ws->device);
            if (!g.ok) return AH_EHIP;
            const uint64_t slots = (uint64_t)value / (uint64_t)(64 * v.vec) + (ws->max_chunks + 1) * 64;
            if (slots <= ws->wave_partials_cap) return AH_OK;
            if (ws->carried_slots) return AH_EINVAL; /* a carried sum is pending: fold it first (read the result) */
            if (hipDeviceSynchronize() != hipSuccess) return AH_EHIP;
            if (ws->d_wave_partials) (void)hipFree(ws->d_wave_partials);
            ws->d_wave_partials = nullptr;
            ws->wave_partials_cap = 0;
            if (hipMalloc(&ws->d_wave_partials, slots * sizeof(double)) != hipSuccess) {
                (void)hipGetLastError();
                return AH_ENOMEM;
            }
            ws->wave_partials_cap = slots;
            return AH_OK;
        }
        case AH_TUNE_PREP_BLOCKS:
            if (value > ah::kMaxPartials) return AH_EINVAL;
            ws->tune_prep_blocks = value;
            return AH_OK;
        case AH_TUNE_STEP_VARIANT: {
            ah::StepVariant v;
            if (!decode_variant(value, &v)) return AH_EINVAL;
            ws->tune_step_variant = value;
            return AH_OK;
        }
        default: return AH_EINVAL;
    }
}

static int read_result(autohete_ws *ws, hipStream_t stream, double *sumsq, float *norm, uint32_t *found_inf)
{
    if (hipMemcpyAsync(ws->h_res, ws->d_res, sizeof(GradResult), hipMemcpyDeviceToHost, stream) != hipSuccess ||
        hipStreamSynchronize(stream) != hipSuccess)
        return AH_EHIP;
    if (sumsq) *sumsq = ws->h_res->sumsq;
    if (norm) *norm = ws->h_res->norm;
    if (found_inf) *found_inf = ws->h_res->found_inf;
    return AH_OK;
}

static int prep_common(autohete_ws *ws, const autohete_chunk *chunks, uint64_t n_chunks, int lowp_dtype,
                       float loss_scale, double extra_sumsq, bool accumulate, void *stream_, float *norm_out,
                       uint32_t *found_inf_out)
{
    if (!ws || (lowp_dtype != AH_BF16 && lowp_dtype != AH_FP16)) return AH_EINVAL;
    if (!(loss_scale > 0.0f) || !isfinite(loss_scale)) return AH_EINVAL;
    DeviceGuard g(ws->device);
    if (!g.ok) return AH_EHIP;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    autohete_ws::Table *tab = nullptr;
    int rc;
    if (accumulate) {
        if ((rc = flush_carried(ws, stream)) != AH_OK) return rc;
    } else {
        ws->carried_slots = 0; /* the result is replaced: a carried sum not folded yet goes with it */
    }
    try {
        rc = build_prep_table(ws, chunks, n_chunks, ah::prep_tile_elems(), stream, &tab);
    } catch (...) { /* std::bad_alloc from the host-side table: nothing may be thrown across the C ABI */
        return AH_ENOMEM;
    }
    if (rc != AH_OK) return rc;

    /* One 256-thread block per CU, each with 32 KB of loads in flight: the measured optimum for
     * a read-only stream on this chip (more resident blocks widen the window and lose bandwidth). */
    const uint64_t tiles = tab->tiles;
    uint64_t blocks = ws->tune_prep_blocks ? (uint64_t)ws->tune_prep_blocks : (uint64_t)ws->n_cu;
    if (blocks > (uint64_t)ah::kMaxPartials) blocks = ah::kMaxPartials;
    if (blocks > tiles) blocks = tiles;
    if (ah::launch_prep(lowp_dtype, (unsigned)blocks, stream, tab->d, (uint32_t)n_chunks, tiles,
                        1.0 / (double)loss_scale, extra_sumsq, accumulate, ws->d_partials, ws->d_ticket,
                        ws->d_res) != hipSuccess)
        return AH_EHIP;
    if (norm_out || found_inf_out) return read_result(ws, stream, nullptr, norm_out, found_inf_out);
    return AH_OK;
}

int autohete_grad_prep(autohete_ws *ws, const autohete_chunk *chunks, uint64_t n_chunks, int lowp_dtype,
                       float loss_scale, double extra_sumsq, void *stream, float *norm_out,
                       uint32_t *found_inf_out)
{
    return prep_common(ws, chunks, n_chunks, lowp_dtype, loss_scale, extra_sumsq, false, stream, norm_out,
                       found_inf_out);
}

int autohete_grad_prep_accumulate(autohete_ws *ws, const autohete_chunk *chunks, uint64_t n_chunks,
                                  int lowp_dtype, float loss_scale, void *stream)
{
    return prep_common(ws, chunks, n_chunks, lowp_dtype, loss_scale, 0.0, true, stream, nullptr, nullptr);
}

int autohete_grad_prep_static(const autohete_chunk *chunks, uint64_t n_chunks, int lowp_dtype, float loss_scale,
                              double extra_sumsq, void *stream, autohete_grad_result *result)
{
    static_assert(sizeof(autohete_grad_result) == sizeof(GradResult), "the public result is the kernels' result");
    static_assert(AUTOHETE_STATIC_MAX_CHUNKS == ah::kStaticMaxChunks, "header and kernels agree on the limit");
    if (lowp_dtype != AH_BF16 && lowp_dtype != AH_FP16) return AH_EINVAL;
    if (!(loss_scale > 0.0f) || !isfinite(loss_scale)) return AH_EINVAL;
    if (!result || (n_chunks && !chunks)) return AH_EINVAL;
    if (reinterpret_cast<uintptr_t>(result) & 7u) return AH_EALIGN;
    if (n_chunks > (uint64_t)ah::kStaticMaxChunks) return AH_ELIMIT;
    ah::PrepRows rows; /* on the stack: copied into the launch's argument buffer by the runtime */
    const uint32_t tile_elems = ah::prep_tile_elems();
    uint64_t tiles = 0;
    for (uint64_t i = 0; i < n_chunks; ++i) {
        int rc = validate_chunk(chunks[i], kGrad);
        if (rc != AH_OK) return rc;
        rows.grad[i] = static_cast<const uint16_t *>(chunks[i].grad);
        rows.numel[i] = chunks[i].numel;
        rows.tile_begin[i] = tiles;
        tiles += (chunks[i].numel + tile_elems - 1) / tile_elems;
    }
    for (uint64_t i = n_chunks; i <= (uint64_t)ah::kStaticMaxChunks; ++i) { /* sentinel, and defined values beyond */
        rows.grad[i] = nullptr;
        rows.numel[i] = 0;
        rows.tile_begin[i] = tiles;
    }
    return ah::launch_prep_static(lowp_dtype, static_cast<hipStream_t>(stream), rows, tiles,
                                  1.0 / (double)loss_scale, extra_sumsq,
                                  reinterpret_cast<GradResult *>(result)) == hipSuccess
               ? AH_OK : AH_EHIP;
}

/* carry_to != NULL: the norm-carrying update; the squares of these chunks' gradients are folded
 * into carry_to's result. */
static int step_common(autohete_ws *ws, const autohete_chunk *chunks, uint64_t n_chunks, int lowp_dtype,
                       uint64_t step, const autohete_hparams *hp, void *stream_, bool write_back,
                       autohete_ws *carry_to = nullptr)
{
    if (!ws || !hp || step == 0 || (lowp_dtype != AH_BF16 && lowp_dtype != AH_FP16)) return AH_EINVAL;
    if (carry_to && (carry_to == ws || carry_to->device != ws->device)) return AH_EINVAL;
    auto nonneg = [](float x) { return isfinite(x) && x >= 0.0f; };
    if (!nonneg(hp->lr) || !nonneg(hp->eps) || !nonneg(hp->weight_decay) || !isfinite(hp->max_grad_norm) ||
        !(hp->beta1 >= 0.0f && hp->beta1 < 1.0f) || !(hp->beta2 >= 0.0f && hp->beta2 < 1.0f) ||
        !(hp->loss_scale > 0.0f) || !isfinite(hp->loss_scale))
        return AH_EINVAL;
    DeviceGuard g(ws->device);
    if (!g.ok) return AH_EHIP;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    ah::StepVariant var;
    if (!decode_variant(ws->tune_step_variant, &var)) return AH_EINVAL;
    var.write_back = write_back;
    autohete_ws::Table *tab = nullptr;
    int rc;
    try {
        rc = build_step_table(ws, chunks, n_chunks, (uint32_t)(var.vec * var.block), (uint32_t)var.block,
                              kGrad | kMaster | kMom1 | kMom2 | (write_back ? kLowp : 0u), stream, &tab);
    } catch (...) {
        return AH_ENOMEM;
    }
    if (rc != AH_OK) return rc;
    if (n_chunks == 0) return AH_OK;
    if ((rc = flush_carried(ws, stream)) != AH_OK) return rc; /* the result this update clips with */

    /* Per-launch constants, fp64 from the fp32 hyper-parameters. */
    ah::StepConsts k;
    k.inv_scale = 1.0 / (double)hp->loss_scale;
    k.max_norm = (double)hp->max_grad_norm;
    k.b1 = (double)hp->beta1;
    k.b2 = (double)hp->beta2;
    k.omb1 = 1.0 - k.b1;
    k.omb2 = 1.0 - k.b2;
    k.bc1 = 1.0 - pow(k.b1, (double)step);
    k.bc2 = 1.0 - pow(k.b2, (double)step);
    k.rbc1 = 1.0 / k.bc1;
    k.rbc2 = 1.0 / k.bc2;
    k.lr = (double)hp->lr;
    k.eps = (double)hp->eps;
    k.wd = (double)hp->weight_decay;

    const uint64_t call_elems = tab->tiles * (uint64_t)(var.vec * var.block);
    const unsigned lds = lds_for_cap(ws, ws->tune_step_blocks_per_cu ? ws->tune_step_blocks_per_cu
                                         : carry_to ? default_carry_blocks_per_cu(call_elems)
                                         : write_back ? default_blocks_per_cu(call_elems) : kDefaultMasterBlocksPerCu);
    if (!carry_to) {
        for (const autohete_ws::Group &grp : tab->groups) {
            if (ah::launch_step(lowp_dtype, var, (unsigned)grp.max_tiles, grp.rows, lds, stream,
                                tab->d + grp.first, ws->d_res, k) != hipSuccess)
                return AH_EHIP;
        }
        return AH_OK;
    }
    /* One slot per wavefront, appended to what earlier calls carried into the same workspace. */
    uint64_t base = 0;
    rc = reserve_carried(carry_to, tab->tiles * (uint64_t)(var.block / 64), k.inv_scale, stream, &base);
    if (rc != AH_OK) return rc;
    for (const autohete_ws::Group &grp : tab->groups) {
        if (ah::launch_step_carry(lowp_dtype, var, (unsigned)grp.max_tiles, grp.rows, lds, stream,
                                  tab->d + grp.first, ws->d_res, k, carry_to->d_wave_partials, base) !=
            hipSuccess)
            return AH_EHIP;
    }
    return AH_OK;
}

int autohete_adamw_step(autohete_ws *ws, const autohete_chunk *chunks, uint64_t n_chunks, int lowp_dtype,
                        uint64_t step, const autohete_hparams *hp, void *stream)
{
    return step_common(ws, chunks, n_chunks, lowp_dtype, step, hp, stream, true);
}

int autohete_adamw_step_carry(autohete_ws *ws, autohete_ws *ws_next, const autohete_chunk *chunks,
                              uint64_t n_chunks, int lowp_dtype, uint64_t step, const autohete_hparams *hp,
                              void *stream)
{
    if (!ws_next) return AH_EINVAL;
    return step_common(ws, chunks, n_chunks, lowp_dtype, step, hp, stream, true, ws_next);
}

int autohete_adamw_step_master(autohete_ws *ws, const autohete_chunk *chunks, uint64_t n_chunks, int lowp_dtype,
                               uint64_t step, const autohete_hparams *hp, void *stream)
{
    return step_common(ws, chunks, n_chunks, lowp_dtype, step, hp, stream, false);
}

int autohete_cast_params(autohete_ws *ws, const autohete_chunk *chunks, uint64_t n_chunks, int lowp_dtype,
                         void *stream_)
{
    if (!ws || (lowp_dtype != AH_BF16 && lowp_dtype != AH_FP16)) return AH_EINVAL;
    DeviceGuard g(ws->device);
    if (!g.ok) return AH_EHIP;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    autohete_ws::Table *tab = nullptr;
    int rc;
    try {
        rc = build_step_table(ws, chunks, n_chunks, ah::kCastTileElems, 64u, kLowp | kMaster, stream, &tab);
    } catch (...) {
        return AH_ENOMEM;
    }
    if (rc != AH_OK) return rc;
    const unsigned lds = lds_for_cap(ws, ws->tune_cast_blocks_per_cu ? ws->tune_cast_blocks_per_cu
                                                                      : kDefaultCastBlocksPerCu);
    for (const autohete_ws::Group &grp : tab->groups) {
        if (ah::launch_cast(lowp_dtype, (unsigned)grp.max_tiles, grp.rows, lds, stream, tab->d + grp.first) !=
            hipSuccess)
            return AH_EHIP;
    }
    return AH_OK;
}

int autohete_grad_result_get(autohete_ws *ws, void *stream, double *sumsq, float *norm, uint32_t *found_inf)
{
    if (!ws) return AH_EINVAL;
    DeviceGuard g(ws->device);
    if (!g.ok) return AH_EHIP;
    int rc = flush_carried(ws, static_cast<hipStream_t>(stream));
    if (rc != AH_OK) return rc;
    return read_result(ws, static_cast<hipStream_t>(stream), sumsq, norm, found_inf);
}

int autohete_grad_result_set(autohete_ws *ws, double sumsq, uint32_t found_inf, void *stream)
{
    if (!ws) return AH_EINVAL;
    DeviceGuard g(ws->device);
    if (!g.ok) return AH_EHIP;
    ws->carried_slots = 0; /* overwritten with the rest of the result */
    return ah::launch_set_result(static_cast<hipStream_t>(stream), ws->d_res, sumsq, found_inf) == hipSuccess
               ? AH_OK : AH_EHIP;
}

}  // extern "C"
