// Host side of liblora_gfx950: the ragged adapter pool, the per-batch planner (grouping of tokens
// by adapter, byte-balanced work units) and the C boundary declared in include/lora.h.
#include "../../include/lora.h"
#include "lora_internal.h"

#include <algorithm>
#include <atomic>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <map>
#include <memory>
#include <mutex>
#include <new>
#include <shared_mutex>
#include <unordered_map>
#include <vector>

using lora::LinBlock;
using lora::SegRec;
using lora::Unit;

// ------------------------------------------------------------------------------------------------
// errors
// ------------------------------------------------------------------------------------------------
static thread_local char g_err[512] = "";

static lora_status_t fail(lora_status_t st, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return st;
}

static lora_status_t hip_fail(hipError_t e, const char *what)
{
    return fail(LORA_ERR_DEVICE, "%s: %s", what, hipGetErrorString(e));
}

#define HIP_TRY(call)                                         \
    do {                                                      \
        hipError_t e_ = (call);                               \
        if (e_ != hipSuccess) return hip_fail(e_, #call);     \
    } while (0)

// No exception crosses the C boundary: every entry point is a function-try-block that ends in this
// (the containers of the host objects can throw std::bad_alloc).
#define API_CATCH                                                                               \
    catch (const std::bad_alloc &) { return fail(LORA_ERR_OOM, "host allocation failed"); }     \
    catch (...) { return fail(LORA_ERR_INVALID_ARG, "unexpected C++ exception in the library"); }

static inline int round_up(int v, int m) { return (v + m - 1) / m * m; }
static inline size_t round_up_sz(size_t v, size_t m) { return (v + m - 1) / m * m; }

// ------------------------------------------------------------------------------------------------
// objects
// ------------------------------------------------------------------------------------------------
struct lora_pool {
    uint32_t magic;
    int in_features, out_features, n_adapters;
    std::vector<int32_t> rank, r8;
    std::vector<float> scale;
    std::vector<uint64_t> a_off, b_off;  // element offsets
    std::vector<uint8_t> resident;
    // every load, eviction, declaration of residency or move of an adapter gives it a new stamp; a
    // segment object remembers the stamps of the adapters it uses
    std::vector<uint64_t> epoch;
    uint64_t next_epoch;
    uint16_t *arena;
    size_t arena_bytes;
    uint64_t id;
    // live pool: space is handed out at load time from a free list (element offset -> length, both
    // multiples of 128 elements = 256 bytes); an adapter without space has a_off == kNoOffset
    bool live;
    std::map<uint64_t, uint64_t> free_blocks;
};
static const uint64_t kNoOffset = ~0ull;

struct lora_segments {
    uint32_t magic;
    const lora_pool *pool;
    uint64_t pool_id;
    std::vector<uint64_t> seg_epoch;  // stamp of each used adapter when the plan was made
    int32_t T, n_active;
    int n_k_slices, k_slice_len;
    int64_t v_floats, weight_bytes;
    std::vector<int32_t> perm, seg_start, seg_adapter;
    std::vector<int64_t> v_offset;
    // feature sizes of the pool the plan was made for (for launches on sibling pools)
    int layout_in, layout_out;
    std::vector<SegRec> segs;
    std::vector<Unit> shrink_units, prefill_units, expand_units, expand_big_units;
    // the one-launch decode form's own lists, by place in the launch (empty places have ntok == 0)
    std::vector<Unit> fused_shrink, fused_expand;
    // the adapted layer's row order (lora_linear): batch row of every place (-1: none) and the adapter of
    // every 16 places; all T tokens are in it, the ones without adapter last
    std::vector<int32_t> lin_rows;
    std::vector<LinBlock> lin_blocks;
    size_t off_lin_rows, off_lin_blocks;
    // device table: [perm | shrink units | prefill shrink units | expand units | arrival counters,
    // ready counters, time-out flag]
    char *dev;
    size_t dev_capacity;
    char *staging;  // pinned host copy of the table
    size_t staging_capacity;
    size_t off_perm, off_shrink, off_prefill, off_expand, off_expand_big, off_fused_shrink, off_fused_expand, off_sync,
        table_bytes;
    bool has_big_units;     // some unit holds more than 16 tokens (token-heavy groups)
    bool heavy_small_expand;  // a token-heavy group above kBigExpandMaxRank (none, as the pool's ranks stand): shrunk by token-heavy units, expanded by 16-token units
    bool wide;              // decode shrink units span all of k (work groups of 16 wavefronts, no partial sums)
    int wide_slices, wide_slice_len;  // the k-slices such a work group's wavefronts divide k into
    int n_prefill_hi;       // how many of prefill_units are above rank 64
    bool decode_fused;      // whole-k decode batch that can run as one launch (see finish_decode_fused)
    int fused_grid;         // work groups of that launch
    int n_sync;             // counters: one per (group, token tile), then the time-out flag
    unsigned launches;      // fused launches since the table was uploaded (the counters' epoch)
    bool caller_memory;     // dev / staging belong to the caller (lora_segments_upload_to): never freed, never grown here
    lora_plan_options_t opts;  // as given at planning (-1 / 0 fields: the process-wide default at the time of use)
    hipEvent_t copied;  // recorded after the upload; guards re-use of `staging`
    // mixed batches: the decode-sized groups' launches go to a stream of the object's own, between a
    // fork and a join event, and run beside the token-heavy groups' launches on the caller's stream
    hipStream_t side;
    hipEvent_t fork, join;
    bool uploaded;
    // Several projections in one object (they read the same x and write column blocks of one y): the
    // unit lists of all of them, one after the other.  Unit offsets are relative to `mbase`, the lowest
    // of the pools' arenas; projection q's v rows, counters and output columns follow those of q - 1.
    std::vector<const lora_pool *> mpools;
    std::vector<uint64_t> mpool_ids;
    std::vector<std::vector<SegRec>> msegs;
    std::vector<std::vector<uint64_t>> mepochs;
    std::vector<int> mouts;          // out_features of each projection
    std::vector<uint64_t> mdelta;    // element distance of each pool's arena from the lowest one
    int out_total;
};

static const uint32_t kPoolMagic = 0x4C505231u, kSegMagic = 0x4C534731u;
static std::atomic<uint64_t> g_next_pool_id{1};

// Live pools by address: a pointer is looked up here before it is dereferenced, so a handle that was
// destroyed (by the caller, or the pool a segment object was planned for) is refused instead of read.
static std::shared_mutex g_pools_mu;
static std::unordered_map<const lora_pool *, uint64_t> g_live_pools;  // address -> id

static bool pool_ok(const lora_pool *p)
{
    if (!p) return false;
    std::shared_lock<std::shared_mutex> lk(g_pools_mu);
    return g_live_pools.find(p) != g_live_pools.end();
}
// the pool a segment object remembers: alive, and still the one with that id (not a new pool at the address)
static bool pool_is(const lora_pool *p, uint64_t id)
{
    if (!p) return false;
    std::shared_lock<std::shared_mutex> lk(g_pools_mu);
    auto it = g_live_pools.find(p);
    return it != g_live_pools.end() && it->second == id;
}
static bool seg_ok(const lora_segments *s) { return s && s->magic == kSegMagic; }

// ------------------------------------------------------------------------------------------------
// pool
// ------------------------------------------------------------------------------------------------
static lora_status_t check_desc(const lora_pool_desc_t *d)
{
    if (!d) return fail(LORA_ERR_INVALID_ARG, "desc is NULL");
    if (d->n_adapters < 0) return fail(LORA_ERR_INVALID_ARG, "n_adapters = %d", d->n_adapters);
    if (d->n_adapters > 0 && (!d->ranks || !d->scales)) return fail(LORA_ERR_INVALID_ARG, "ranks/scales is NULL");
    if (d->dtype != LORA_BF16) return fail(LORA_ERR_INVALID_ARG, "dtype %d is not LORA_BF16", d->dtype);
    if (d->in_features <= 0 || d->out_features <= 0 || d->in_features % 64 || d->out_features % 128)
        return fail(LORA_ERR_SHAPE, "in_features (%d) must be a positive multiple of 64 and out_features (%d) of 128",
                    d->in_features, d->out_features);
    for (int a = 0; a < d->n_adapters; ++a)
        if (d->ranks[a] < 1 || d->ranks[a] > LORA_MAX_RANK)
            return fail(LORA_ERR_SHAPE, "adapter %d: rank %d outside 1..%d", a, d->ranks[a], LORA_MAX_RANK);
    return LORA_OK;
}

static size_t adapter_elems(const lora_pool_desc_t *d, int a)
{
    const size_t r8 = (size_t)round_up(d->ranks[a], 8);
    return r8 * ((size_t)d->in_features + (size_t)d->out_features);
}

extern "C" lora_status_t lora_pool_bytes(const lora_pool_desc_t *desc, size_t *arena_bytes)
try {
    lora_status_t st = check_desc(desc);
    if (st != LORA_OK) return st;
    if (!arena_bytes) return fail(LORA_ERR_INVALID_ARG, "arena_bytes is NULL");
    size_t elems = 0;
    for (int a = 0; a < desc->n_adapters; ++a) elems += adapter_elems(desc, a);
    *arena_bytes = round_up_sz(elems * 2, 256);
    return LORA_OK;
}
API_CATCH

static uint64_t block_elems(const lora_pool *p, int a)
{
    const uint64_t e = (uint64_t)p->r8[a] * ((uint64_t)p->in_features + (uint64_t)p->out_features);
    return (e + 127) / 128 * 128;  // 256-byte granules
}

static lora_status_t create_pool(const lora_pool_desc_t *desc, void *dev_arena, size_t arena_bytes, bool live,
                                 lora_pool_t **out)
{
    if (!out) return fail(LORA_ERR_INVALID_ARG, "out is NULL");
    *out = nullptr;
    size_t need = 0;
    lora_status_t st = lora_pool_bytes(desc, &need);
    if (st != LORA_OK) return st;
    if ((need > 0 || live) && !dev_arena) return fail(LORA_ERR_INVALID_ARG, "dev_arena is NULL");
    if (((uintptr_t)dev_arena) % 256) return fail(LORA_ERR_INVALID_ARG, "dev_arena is not 256-byte aligned");
    if (!live && arena_bytes < need)
        return fail(LORA_ERR_OOM, "arena of %zu bytes is smaller than the %zu bytes the pool needs", arena_bytes, need);
    lora_pool *p = new (std::nothrow) lora_pool();
    if (!p) return fail(LORA_ERR_OOM, "host allocation failed");
    p->magic = kPoolMagic;
    p->in_features = desc->in_features;
    p->out_features = desc->out_features;
    p->n_adapters = desc->n_adapters;
    p->arena = (uint16_t *)dev_arena;
    p->arena_bytes = arena_bytes;
    p->next_epoch = 1;
    p->id = g_next_pool_id++;
    p->live = live;
    uint64_t off = 0;
    for (int a = 0; a < desc->n_adapters; ++a) {
        const int r8 = round_up(desc->ranks[a], 8);
        p->rank.push_back(desc->ranks[a]);
        p->r8.push_back(r8);
        p->scale.push_back(desc->scales[a]);
        p->a_off.push_back(live ? kNoOffset : off);
        p->b_off.push_back(live ? kNoOffset : off + (uint64_t)r8 * desc->in_features);
        p->resident.push_back(0);
        p->epoch.push_back(0);
        off += (uint64_t)adapter_elems(desc, a);
    }
    if (live) {
        const uint64_t elems = (uint64_t)(arena_bytes / 256) * 128;
        if (elems) p->free_blocks[0] = elems;
    }
    {
        std::unique_lock<std::shared_mutex> lk(g_pools_mu);
        g_live_pools[p] = p->id;
    }
    *out = p;
    return LORA_OK;
}

extern "C" lora_status_t lora_pool_create(const lora_pool_desc_t *desc, void *dev_arena, size_t arena_bytes,
                                          lora_pool_t **out)
try {
    return create_pool(desc, dev_arena, arena_bytes, false, out);
}
API_CATCH

extern "C" lora_status_t lora_pool_create_live(const lora_pool_desc_t *desc, void *dev_arena, size_t arena_bytes,
                                               lora_pool_t **out)
try {
    return create_pool(desc, dev_arena, arena_bytes, true, out);
}
API_CATCH

// ---- live pool: first-fit free list with coalescing -------------------------------------------------
static void space_of(const lora_pool *p, uint64_t *free_elems, uint64_t *largest)
{
    *free_elems = *largest = 0;
    for (const auto &b : p->free_blocks) {
        *free_elems += b.second;
        *largest = std::max(*largest, b.second);
    }
}

static lora_status_t live_place(lora_pool *p, int a)
{
    if (p->a_off[a] != kNoOffset) return LORA_OK;
    const uint64_t need = block_elems(p, a);
    for (auto it = p->free_blocks.begin(); it != p->free_blocks.end(); ++it) {
        if (it->second < need) continue;
        const uint64_t off = it->first, rest = it->second - need;
        p->free_blocks.erase(it);
        if (rest) p->free_blocks[off + need] = rest;
        p->a_off[a] = off;
        p->b_off[a] = off + (uint64_t)p->r8[a] * p->in_features;
        return LORA_OK;
    }
    uint64_t fr, lg;
    space_of(p, &fr, &lg);
    return fail(LORA_ERR_OOM,
                "adapter %d needs %llu bytes in one piece; the arena has %llu bytes free, the largest piece %llu%s", a,
                (unsigned long long)(need * 2), (unsigned long long)(fr * 2), (unsigned long long)(lg * 2),
                fr >= need ? " (lora_pool_compact would make room)" : "");
}

static void live_release(lora_pool *p, int a)
{
    if (p->a_off[a] == kNoOffset) return;
    uint64_t off = p->a_off[a], len = block_elems(p, a);
    auto next = p->free_blocks.lower_bound(off);
    if (next != p->free_blocks.end() && off + len == next->first) {
        len += next->second;
        next = p->free_blocks.erase(next);
    }
    if (next != p->free_blocks.begin()) {
        auto prev = std::prev(next);
        if (prev->first + prev->second == off) {
            prev->second += len;
            len = 0;
        }
    }
    if (len) p->free_blocks[off] = len;
    p->a_off[a] = p->b_off[a] = kNoOffset;
}

static lora_status_t check_adapter(const lora_pool *pool, int32_t adapter)
{
    if (!pool_ok(pool)) return fail(LORA_ERR_INVALID_ARG, "pool is NULL or not a pool");
    if (adapter < 0 || adapter >= pool->n_adapters)
        return fail(LORA_ERR_INVALID_ARG, "adapter %d outside 0..%d", adapter, pool->n_adapters - 1);
    return LORA_OK;
}

extern "C" lora_status_t lora_pool_reserve(lora_pool_t *pool, int32_t adapter)
try {
    lora_status_t st = check_adapter(pool, adapter);
    if (st != LORA_OK) return st;
    return pool->live ? live_place(pool, adapter) : LORA_OK;
}
API_CATCH

extern "C" lora_status_t lora_pool_space(const lora_pool_t *pool, size_t *free_bytes, size_t *largest_free_bytes)
try {
    if (!pool_ok(pool)) return fail(LORA_ERR_INVALID_ARG, "pool is NULL or not a pool");
    uint64_t fr, lg;
    space_of(pool, &fr, &lg);
    if (free_bytes) *free_bytes = (size_t)(fr * 2);
    if (largest_free_bytes) *largest_free_bytes = (size_t)(lg * 2);
    return LORA_OK;
}
API_CATCH

// Slides the placed adapters of a live pool towards the start of the arena, in address order, with
// device-to-device copies on `stream`.  A move whose source and destination overlap goes through
// `dev_scratch` when that is large enough, else in pieces no longer than the gap (each piece then
// lies wholly before its own source, and the stream runs the pieces in order).
extern "C" lora_status_t lora_pool_compact(lora_pool_t *pool, void *dev_scratch, size_t scratch_bytes, void *stream,
                                           int32_t *n_moved)
try {
    if (!pool_ok(pool)) return fail(LORA_ERR_INVALID_ARG, "pool is NULL or not a pool");
    if (n_moved) *n_moved = 0;
    if (!pool->live) return LORA_OK;
    hipStream_t s = (hipStream_t)stream;
    std::vector<int> order;
    for (int a = 0; a < pool->n_adapters; ++a)
        if (pool->a_off[a] != kNoOffset) order.push_back(a);
    std::sort(order.begin(), order.end(), [&](int x, int y) { return pool->a_off[x] < pool->a_off[y]; });
    // Whatever way this function is left (a copy may fail half-way), the free list is rebuilt from the
    // places the adapters then have: the gaps between them, in address order.
    struct FreeListGuard {
        lora_pool *p;
        ~FreeListGuard()
        {
            std::vector<std::pair<uint64_t, uint64_t>> placed;  // offset, length
            for (int a = 0; a < p->n_adapters; ++a)
                if (p->a_off[a] != kNoOffset) placed.push_back({p->a_off[a], block_elems(p, a)});
            std::sort(placed.begin(), placed.end());
            p->free_blocks.clear();
            const uint64_t total = (uint64_t)(p->arena_bytes / 256) * 128;
            uint64_t at = 0;
            for (const auto &b : placed) {
                if (b.first > at) p->free_blocks[at] = b.first - at;
                at = std::max(at, b.first + b.second);
            }
            if (total > at) p->free_blocks[at] = total - at;
        }
    } free_list_guard{pool};
    uint64_t cursor = 0;
    int moved = 0;
    for (int a : order) {
        const uint64_t len = block_elems(pool, a), src = pool->a_off[a];
        if (src != cursor) {
            const uint64_t gap = src - cursor;
            char *d = (char *)(pool->arena + cursor), *f = (char *)(pool->arena + src);
            const size_t bytes = (size_t)len * 2, gap_bytes = (size_t)gap * 2;
            if (gap_bytes >= bytes) {
                HIP_TRY(hipMemcpyAsync(d, f, bytes, hipMemcpyDeviceToDevice, s));
            } else if (dev_scratch && scratch_bytes >= bytes) {
                HIP_TRY(hipMemcpyAsync(dev_scratch, f, bytes, hipMemcpyDeviceToDevice, s));
                HIP_TRY(hipMemcpyAsync(d, dev_scratch, bytes, hipMemcpyDeviceToDevice, s));
            } else {
                for (size_t o = 0; o < bytes; o += gap_bytes)
                    HIP_TRY(hipMemcpyAsync(d + o, f + o, std::min(gap_bytes, bytes - o), hipMemcpyDeviceToDevice, s));
            }
            pool->a_off[a] = cursor;
            pool->b_off[a] = cursor + (uint64_t)pool->r8[a] * pool->in_features;
            pool->epoch[a] = pool->next_epoch++;
            ++moved;
        }
        cursor += len;
    }
    if (n_moved) *n_moved = moved;
    return LORA_OK;
}
API_CATCH

extern "C" lora_status_t lora_pool_adapter_info(const lora_pool_t *pool, int32_t adapter, lora_adapter_info_t *info)
try {
    if (!pool_ok(pool)) return fail(LORA_ERR_INVALID_ARG, "pool is NULL or not a pool");
    if (!info) return fail(LORA_ERR_INVALID_ARG, "info is NULL");
    if (adapter < 0 || adapter >= pool->n_adapters)
        return fail(LORA_ERR_INVALID_ARG, "adapter %d outside 0..%d", adapter, pool->n_adapters - 1);
    info->a_offset = pool->a_off[adapter];
    info->b_offset = pool->b_off[adapter];
    info->rank = pool->rank[adapter];
    info->rank_padded = pool->r8[adapter];
    info->scale = pool->scale[adapter];
    info->resident = pool->resident[adapter];
    return LORA_OK;
}
API_CATCH

extern "C" lora_status_t lora_pool_load_staging_bytes(const lora_pool_t *pool, int32_t adapter, size_t *bytes)
try {
    lora_status_t st = check_adapter(pool, adapter);
    if (st != LORA_OK) return st;
    if (!bytes) return fail(LORA_ERR_INVALID_ARG, "bytes is NULL");
    *bytes = round_up_sz(2 * (size_t)pool->rank[adapter] * ((size_t)pool->in_features + (size_t)pool->out_features), 256);
    return LORA_OK;
}
API_CATCH

extern "C" lora_status_t lora_pool_load_staged(lora_pool_t *pool, int32_t adapter, const void *A, const void *B,
                                               void *dev_staging, size_t staging_bytes, void *stream)
try {
    lora_status_t st = check_adapter(pool, adapter);
    if (st != LORA_OK) return st;
    if (!A || !B) return fail(LORA_ERR_INVALID_ARG, "A or B is NULL");
    const int r = pool->rank[adapter], r8 = pool->r8[adapter];
    const int in = pool->in_features, out = pool->out_features;
    const size_t nA = (size_t)in * r, nB = (size_t)r * out;
    if (!dev_staging || ((uintptr_t)dev_staging) % 16) return fail(LORA_ERR_INVALID_ARG, "dev_staging is NULL or not 16-byte aligned");
    if (staging_bytes < (nA + nB) * 2)
        return fail(LORA_ERR_OOM, "dev_staging of %zu bytes is smaller than the %zu the adapter's A and B take", staging_bytes,
                    (nA + nB) * 2);
    hipStream_t s = (hipStream_t)stream;
    if (pool->live && (st = live_place(pool, adapter)) != LORA_OK) return st;
    uint16_t *tmp = (uint16_t *)dev_staging;
    HIP_TRY(hipMemcpyAsync(tmp, A, nA * 2, hipMemcpyHostToDevice, s));
    HIP_TRY(hipMemcpyAsync(tmp + nA, B, nB * 2, hipMemcpyHostToDevice, s));
    HIP_TRY(lora::launch_pack_adapter(tmp, tmp + nA, in, out, r, r8, pool->arena + pool->a_off[adapter],
                                      pool->arena + pool->b_off[adapter], s));
    pool->resident[adapter] = 1;
    pool->epoch[adapter] = pool->next_epoch++;
    return LORA_OK;
}
API_CATCH

extern "C" lora_status_t lora_pool_load(lora_pool_t *pool, int32_t adapter, const void *A, const void *B,
                                        int src_is_device, void *stream)
try {
    if (!pool_ok(pool)) return fail(LORA_ERR_INVALID_ARG, "pool is NULL or not a pool");
    if (adapter < 0 || adapter >= pool->n_adapters)
        return fail(LORA_ERR_INVALID_ARG, "adapter %d outside 0..%d", adapter, pool->n_adapters - 1);
    if (!A || !B) return fail(LORA_ERR_INVALID_ARG, "A or B is NULL");
    if (src_is_device != 0 && src_is_device != 1) return fail(LORA_ERR_INVALID_ARG, "src_is_device = %d", src_is_device);
    hipStream_t s = (hipStream_t)stream;
    const int r = pool->rank[adapter], r8 = pool->r8[adapter];
    const int in = pool->in_features, out = pool->out_features;
    if (pool->live) {
        lora_status_t st = live_place(pool, adapter);
        if (st != LORA_OK) return st;
    }
    uint16_t *dstA = pool->arena + pool->a_off[adapter];
    uint16_t *dstB = pool->arena + pool->b_off[adapter];
    const size_t nA = (size_t)in * r, nB = (size_t)r * out;
    if (src_is_device) {
        HIP_TRY(lora::launch_pack_adapter((const uint16_t *)A, (const uint16_t *)B, in, out, r, r8, dstA, dstB, s));
    } else {
        uint16_t *tmp = nullptr;
        hipError_t e = hipMalloc((void **)&tmp, (nA + nB) * 2);
        if (e != hipSuccess) return hip_fail(e, "hipMalloc(staging for lora_pool_load)");
        lora_status_t st = LORA_OK;
        do {
            if ((e = hipMemcpyAsync(tmp, A, nA * 2, hipMemcpyHostToDevice, s)) != hipSuccess) break;
            if ((e = hipMemcpyAsync(tmp + nA, B, nB * 2, hipMemcpyHostToDevice, s)) != hipSuccess) break;
            if ((e = lora::launch_pack_adapter(tmp, tmp + nA, in, out, r, r8, dstA, dstB, s)) != hipSuccess) break;
            e = hipStreamSynchronize(s);
        } while (0);
        if (e != hipSuccess) st = hip_fail(e, "lora_pool_load copy/pack");
        hipError_t e2 = hipFree(tmp);
        if (st == LORA_OK && e2 != hipSuccess) st = hip_fail(e2, "hipFree(staging)");
        if (st != LORA_OK) return st;
    }
    pool->resident[adapter] = 1;
    pool->epoch[adapter] = pool->next_epoch++;
    return LORA_OK;
}
API_CATCH

extern "C" lora_status_t lora_pool_evict(lora_pool_t *pool, int32_t adapter)
try {
    if (!pool_ok(pool)) return fail(LORA_ERR_INVALID_ARG, "pool is NULL or not a pool");
    if (adapter < 0 || adapter >= pool->n_adapters)
        return fail(LORA_ERR_INVALID_ARG, "adapter %d outside 0..%d", adapter, pool->n_adapters - 1);
    pool->resident[adapter] = 0;
    pool->epoch[adapter] = pool->next_epoch++;
    if (pool->live) live_release(pool, adapter);
    return LORA_OK;
}
API_CATCH

extern "C" lora_status_t lora_pool_mark_resident(lora_pool_t *pool, int32_t adapter)
try {
    if (!pool_ok(pool)) return fail(LORA_ERR_INVALID_ARG, "pool is NULL or not a pool");
    if (adapter < 0 || adapter >= pool->n_adapters)
        return fail(LORA_ERR_INVALID_ARG, "adapter %d outside 0..%d", adapter, pool->n_adapters - 1);
    if (pool->live && pool->a_off[adapter] == kNoOffset)
        return fail(LORA_ERR_INVALID_ARG, "adapter %d has no space in the live pool: lora_pool_reserve first", adapter);
    pool->resident[adapter] = 1;
    pool->epoch[adapter] = pool->next_epoch++;
    return LORA_OK;
}
API_CATCH

extern "C" lora_status_t lora_pool_destroy(lora_pool_t *pool)
try {
    if (!pool) return LORA_OK;
    {
        std::unique_lock<std::shared_mutex> lk(g_pools_mu);
        if (g_live_pools.erase(pool) == 0) return fail(LORA_ERR_INVALID_ARG, "not a pool (or destroyed already)");
    }
    pool->magic = 0;
    delete pool;
    return LORA_OK;
}
API_CATCH

// ------------------------------------------------------------------------------------------------
// planner
// ------------------------------------------------------------------------------------------------
// Split-K of the shrink: up to 4 k-slices, each at least 1024 long, each a multiple of 128 so that a
// wavefront's quarter of a slice is a whole number of 32-wide MFMA k steps.
static void choose_k_slices(int in, int *n_slices, int *slice_len)
{
    int n = in / 1024;
    n = std::max(1, std::min(4, n));
    int len = round_up((in + n - 1) / n, 128);
    n = (in + len - 1) / len;
    *n_slices = n;
    *slice_len = len;
}

// Output columns per expand unit.  A work group's four wavefronts take 128-column strips of B^T,
// splitting a strip by rank when the rank is large: one pass covers 512 columns for ranks up to
// 32, 256 for ranks up to 64 and 128 beyond.  A unit is one pass for ranks above 32 (<= 32 KiB of
// B^T, 64 KiB for ranks above 128) and 512 columns (one pass, <= 32 KiB) below.
static int expand_cols_per_unit(int r8, int out)
{
    const int cols = r8 <= 32 ? 512 : (r8 <= 64 ? 256 : 128);
    return std::min(cols, out);
}

// Groups with at least this many tokens are token-heavy: their shrink runs on token tiles that read x
// once (instead of once per 16 rank rows), their expand units hold up to 64 tokens and several column passes.
// Only in batches of at least kPrefillMinBatch tokens: a 128-token tile streams about 1 MB of x, far
// longer than a whole decode-sized launch lasts.
static const int kPrefillMinTokens = 32;
static const int kPrefillMinBatch = 1024;
// Between kWholeKMin and this many whole-k shrink units (four rounds of one work group per compute
// unit of the chip) the decode shrink runs without k-slices; measured on the rank-skew batches, 442
// and 544 such units beat their 4 x as many k-slice units by 8 %, 32 units lose 9 % to their 128.
static std::atomic<int> g_whole_k_limit{1024};
// Mixed batches (token-heavy groups beside decode-sized ones) in two launches that hold both kinds of
// unit: the decode-sized groups are then planned in k-slices, whose work groups have the size of the
// token-heavy ones'.
static std::atomic<int> g_merged_mixed{1};
static const int kSplitRowsFloor = 1;   // fewest tokens of a whole-k unit that may be cut into 8-row halves
static const int kWholeKMin = 64;  // below this, k-slices are what spreads the batch over the chip
// A wavefront of a whole-k unit walks in_features / 16 of k in passes of 256, one trip to memory each:
// beyond this many input features the k-slice units win.  cfg1's routing, ms per step of 32 projections,
// whole-k (one launch per apply) against k-slices (two launches): 0.663 / 0.744 at 8192 input features,
// 0.668 / 0.769 at 8256, 0.942 / 0.963 at 14336, 1.002 / 1.041 at 16384, 1.038 / 1.079 at 16448, 1.290 /
// 1.228 at 20480, 1.442 / 1.380 at 24576, 1.592 / 1.533 at 28672; the rank-skew batch at 28672: 1.024 /
// 0.951.  (Before the one-launch form the shrink launches alone crossed at 8192.)
static const int kWholeKMaxIn = 18432;
// Tokens of a token-heavy shrink unit: up to rank 64 the wavefronts split k and hold 32 tokens; above,
// they split the rank rows and share 64 tokens of x through LDS (A^T is then loaded once per 64
// tokens); above rank 192, 32 tokens (the accumulators of 64 tokens x 256 rank rows do not fit the registers).
static int heavy_tile(int r8) { return r8 <= 64 || r8 > 192 ? 32 : 64; }
// token-heavy groups take 64-token expand units up to this padded rank (a strip's tile of B^T, 128 columns x
// rank, must fit the kernel's 64 KiB of LDS): every rank the pool holds
static const int kBigExpandMaxRank = 256;
static_assert(kBigExpandMaxRank >= LORA_MAX_RANK_PADDED, "the 16-token expand units of token-heavy groups are gone");
// A token-heavy shrink unit is one walk through k (a wavefront takes a quarter of k in passes of 128, one
// trip to memory each), and a launch of few such units lasts as long as one unit's walk (cfg3's routing
// scaled to 1.5 k .. 9.5 k tokens: 32-37 us at 4096 input features, 99-116 us at 14336, whatever the
// number of tokens).  In a batch planned in k-slices such units are cut into 4 or 2 slices along k while
// the cut units stay within these counts.  Measured, shrink launch in us uncut / 2 / 4 slices; 4096: 41
// units 32 / 28 / 23, 79 units 33 / 28 / 25, 148 units 33 / 30 / 33, 161 units 19.5 / 21.4, 291 units
// 37 / 40 / 45, 321 units 28.2 / 28.2; 8192: 250 units 38.7 / 38.9; 14336: 41 units 99 / 67 / 52, 79
// units 102 / 67 / 59, 148 units 102 / 75 / 77, 291 units 116 / 102 / 109, 301 units 85.6 / 75.7, 450
// units 94 / 101.5, 600 units 126.6 / 126.3, cfg2's 718 units 155 / 155 / 162.  So two slices pay up
// to about 320 cut units at 4096 .. 8192 input features and up to 600 .. 900 at 14336, where a unit's
// walk is 3.5 times as long.
static const int kHeavyKCutMaxUnits = 320;
static const int kHeavyKCutLongK = 8192;          // beyond this many input features:
static const int kHeavyKCutMaxUnitsLongK = 750;
// 64-token expand units take a group's columns in 8 runs instead of 4 while the launch stays within one
// round of work groups (two per compute unit): expand launch, 4 / 8 runs, 50 tiles of 64 tokens 15.3 /
// 14.0 us, 51 tiles 15.7 / 14.2, 64 tiles 17.2 / 15.9, 72 tiles 21.7 / 21.9; cfg3's routing at 1.5 k /
// 2.7 k tokens 25.7 -> 19.5 / 26.6 -> 23.1 us at 4096 columns, 78.6 -> 60.8 / 80.5 -> 72.8 us at 14336;
// at 4.9 k tokens and beyond 8 runs are level or lose.
static const int kBigRunsWorkGroupsPerComputeUnit = 2;

extern "C" lora_status_t lora_set_whole_k_limit(int32_t max_units)
try {
    if (max_units < 0) return fail(LORA_ERR_INVALID_ARG, "max_units = %d", max_units);
    g_whole_k_limit = max_units;
    return LORA_OK;
}
API_CATCH

// Order of the decode shrink units in their launch.  The work groups of a launch go to the chip's
// eight XCDs in turn (work group b to XCD b mod 8) and each XCD has an L2 of its own, so the units of
// one group of tokens (one per 16 rank rows, k-slice and token tile, all reading the group's rows of
// x) are given places of one residue mod 8: the rows of x then come from memory once per group instead
// of once per XCD that holds one of its units.  Groups are dealt to the eight lists heaviest first,
// each to the list with the fewest bytes that still has room (every list takes its share of the
// units, so a launch of up to one work group per compute unit stays a single round; a group that does
// not fit is cut); inside a list the heaviest units come first, and the lists are interleaved.
static void order_units_by_xcd(std::vector<Unit> &units)
{
    const int X = 8;
    const size_t n = units.size();
    if (n < 2 * (size_t)X) return;
    const size_t cap = (n + X - 1) / X;
    auto weight = [](const Unit &u) { return (int64_t)(u.pn + u.ntok); };
    // units of a group are adjacent in the list as planned
    std::vector<std::pair<size_t, size_t>> groups;  // [first, last)
    for (size_t i = 0; i < n;) {
        size_t j = i + 1;
        while (j < n && units[j].seg == units[i].seg) ++j;
        groups.push_back({i, j});
        i = j;
    }
    std::vector<int64_t> gw(groups.size(), 0);
    for (size_t g = 0; g < groups.size(); ++g)
        for (size_t i = groups[g].first; i < groups[g].second; ++i) gw[g] += weight(units[i]);
    std::vector<size_t> gorder(groups.size());
    for (size_t g = 0; g < gorder.size(); ++g) gorder[g] = g;
    std::stable_sort(gorder.begin(), gorder.end(), [&](size_t a, size_t b) { return gw[a] > gw[b]; });
    std::vector<std::vector<size_t>> list(X);
    std::vector<int64_t> load(X, 0);
    for (size_t g : gorder) {
        size_t i = groups[g].first;
        while (i < groups[g].second) {
            int best = -1;
            for (int q = 0; q < X; ++q)
                if (list[q].size() < cap && (best < 0 || load[q] < load[best])) best = q;
            while (i < groups[g].second && list[best].size() < cap) {
                list[best].push_back(i);
                load[best] += weight(units[i]);
                ++i;
            }
        }
    }
    for (int q = 0; q < X; ++q)
        std::stable_sort(list[q].begin(), list[q].end(),
                         [&](size_t a, size_t b) { return weight(units[a]) > weight(units[b]); });
    std::vector<Unit> out;
    out.reserve(n);
    for (size_t j = 0; j < cap; ++j)
        for (int q = 0; q < X; ++q)
            if (j < list[q].size()) out.push_back(units[list[q][j]]);
    units.swap(out);
}

// Token-heavy shrink units: the tiles of one adapter on one XCD, so that its A^T comes from memory once
// instead of once per XCD (cfg2 4096 -> 4096: the eight fetches of every A^T were a quarter of the
// launch's traffic).  Such a launch runs several rounds, every XCD takes every eighth work group whatever
// its units cost, and a compute unit passes about 50 GB/s to its work groups whatever they are, so equal
// numbers of units per XCD would leave the XCD that holds the high ranks running alone at the end.  The
// eight lists are therefore filled to equal bytes (tokens + rank rows of the unit, each in_features
// long), heaviest group first, a group cut where a list reaches its share; the shorter lists are padded
// at their end with units of no tokens, which return at once.
static void order_heavy_units_by_xcd(std::vector<Unit> &units)
{
    const int X = 8;
    const size_t n = units.size();
    if (n < 2 * (size_t)X) return;
    auto cost = [](const Unit &u) { return (int64_t)(u.ntok + u.pn); };  // rows of x and of A^T, each in_features long
    std::vector<std::pair<size_t, size_t>> groups;  // [first, last): units of a group are adjacent as planned
    for (size_t i = 0; i < n;) {
        size_t j = i + 1;
        while (j < n && units[j].seg == units[i].seg) ++j;
        groups.push_back({i, j});
        i = j;
    }
    std::vector<int64_t> gw(groups.size(), 0);
    int64_t total = 0;
    for (size_t g = 0; g < groups.size(); ++g) {
        for (size_t i = groups[g].first; i < groups[g].second; ++i) gw[g] += cost(units[i]);
        total += gw[g];
    }
    const int64_t share = total / X + total / (100 * X) + 1;
    std::vector<size_t> gorder(groups.size());
    for (size_t g = 0; g < gorder.size(); ++g) gorder[g] = g;
    std::stable_sort(gorder.begin(), gorder.end(), [&](size_t a, size_t b) { return gw[a] > gw[b]; });
    std::vector<std::vector<size_t>> list(X);
    std::vector<int64_t> load(X, 0);
    for (size_t g : gorder) {
        size_t i = groups[g].first;
        while (i < groups[g].second) {
            int best = 0;
            for (int q = 1; q < X; ++q)
                if (load[q] < load[best]) best = q;
            bool first = true;  // the lightest list takes at least one unit, so the loop ends
            while (i < groups[g].second && (first || load[best] + cost(units[i]) <= share)) {
                list[best].push_back(i);
                load[best] += cost(units[i]);
                first = false;
                ++i;
            }
        }
    }
    size_t longest = 0;
    for (int q = 0; q < X; ++q) {
        std::stable_sort(list[q].begin(), list[q].end(),
                         [&](size_t a, size_t b) { return cost(units[a]) > cost(units[b]); });
        longest = std::max(longest, list[q].size());
    }
    Unit none;
    memset(&none, 0, sizeof none);  // ntok = 0: the kernels leave such a unit at once
    none.seg = -1;
    std::vector<Unit> out;
    out.reserve(longest * X);
    for (size_t j = 0; j < longest; ++j)
        for (int q = 0; q < X; ++q) out.push_back(j < list[q].size() ? units[list[q][j]] : none);
    units.swap(out);
}

static int g_compute_units = 256;  // of the chip: a whole-k launch within this many units is one round
static int opt_big_runs_max_units(const lora_segments *sg)
{
    return sg->opts.big_runs_max_units >= 0 ? sg->opts.big_runs_max_units : kBigRunsWorkGroupsPerComputeUnit * g_compute_units;
}
static const int kXcds = 8;         // XCDs of the chip, each with an L2 of its own; work group b of a launch runs on XCD b mod 8
static std::atomic<int> g_decode_single_launch{1};
static std::atomic<int> g_side_stream{1};
static std::atomic<int> g_fused_apply{0};
static const unsigned kSpinLimit = 1u << 18;  // polls of a waiting expand unit before it gives up
static std::atomic<unsigned> g_spin_limit{kSpinLimit};

// A segment object's plan settings: what was given at planning, else the process-wide default now.
static const lora_plan_options_t kDefaultOptions = LORA_PLAN_OPTIONS_DEFAULT;
static int opt_whole_k_limit(const lora_segments *sg) { return sg->opts.whole_k_limit >= 0 ? sg->opts.whole_k_limit : g_whole_k_limit.load(); }
static bool opt_merged(const lora_segments *sg) { return (sg->opts.merged_launches >= 0 ? sg->opts.merged_launches : g_merged_mixed.load()) != 0; }
static bool opt_side_stream(const lora_segments *sg) { return (sg->opts.side_stream >= 0 ? sg->opts.side_stream : g_side_stream.load()) != 0; }
static bool opt_fused_apply(const lora_segments *sg) { return (sg->opts.fused_apply >= 0 ? sg->opts.fused_apply : g_fused_apply.load()) != 0; }
static bool opt_decode_single(const lora_segments *sg) { return (sg->opts.decode_single_launch >= 0 ? sg->opts.decode_single_launch : g_decode_single_launch.load()) != 0; }
static int opt_whole_k_max_in(const lora_segments *sg) { return sg->opts.whole_k_max_in >= 0 ? sg->opts.whole_k_max_in : kWholeKMaxIn; }
static int opt_heavy_min_tokens(const lora_segments *sg) { return sg->opts.heavy_min_tokens >= 0 ? sg->opts.heavy_min_tokens : kPrefillMinTokens; }
static int opt_heavy_min_batch(const lora_segments *sg) { return sg->opts.heavy_min_batch >= 0 ? sg->opts.heavy_min_batch : kPrefillMinBatch; }
static int opt_big_runs_max_units(const lora_segments *sg);
static int opt_heavy_k_cut_max_units(const lora_segments *sg, int in_features)
{
    if (sg->opts.heavy_k_cut_max_units >= 0) return sg->opts.heavy_k_cut_max_units;
    return in_features > kHeavyKCutLongK ? kHeavyKCutMaxUnitsLongK : kHeavyKCutMaxUnits;
}
static unsigned opt_spin_limit(const lora_segments *sg) { return sg->opts.fused_wait_limit ? sg->opts.fused_wait_limit : g_spin_limit.load(); }

// Offsets of the lists inside the device table.
static void layout_table(lora_segments *sg)
{
    sg->off_perm = 0;
    sg->off_shrink = round_up_sz(sg->perm.size() * sizeof(int32_t), 256);
    sg->off_prefill = round_up_sz(sg->off_shrink + sg->shrink_units.size() * sizeof(Unit), 256);
    sg->off_expand = round_up_sz(sg->off_prefill + sg->prefill_units.size() * sizeof(Unit), 256);
    sg->off_expand_big = round_up_sz(sg->off_expand + sg->expand_units.size() * sizeof(Unit), 256);
    sg->off_fused_shrink = round_up_sz(sg->off_expand_big + sg->expand_big_units.size() * sizeof(Unit), 256);
    sg->off_fused_expand = round_up_sz(sg->off_fused_shrink + sg->fused_shrink.size() * sizeof(Unit), 256);
    sg->off_lin_rows = round_up_sz(sg->off_fused_expand + sg->fused_expand.size() * sizeof(Unit), 256);
    sg->off_lin_blocks = round_up_sz(sg->off_lin_rows + sg->lin_rows.size() * sizeof(int32_t), 256);
    sg->off_sync = round_up_sz(sg->off_lin_blocks + sg->lin_blocks.size() * sizeof(LinBlock), 256);
    sg->table_bytes = round_up_sz(sg->off_sync + (size_t)(2 * sg->n_sync + 4 + 2 * 256) * sizeof(unsigned), 256);
}

// The one-launch form of a whole-k decode batch (k_decode_fused): at most one work group per compute
// unit, work group b running one shrink unit and then four expand units, v handed over through the L2
// of the XCD the work group runs on (b mod 8).  So every unit of one (group, token tile), the shrink
// units that write its part of v and the expand units that read it, must sit at places of one residue
// mod 8, and the launch must be a single round: at most compute units / 8 shrink units and four
// times as many expand units per XCD.  The tiles are dealt to the eight XCDs heaviest group first,
// each to the XCD with the fewest bytes that still has room (a group's tiles together where they fit:
// they read the same A^T and B^T, which that L2 then serves); if some tile finds no room the batch
// keeps its two launches.  Then, per XCD, while places are left, the 16 rank rows of the shrink units
// with the most tokens are cut into two units of 8 (they pass the most bytes, x beside A^T, through
// their compute unit and would end the launch).  Inside an XCD the heaviest shrink units share a work
// group with the lightest expand units.
static void finish_decode_fused(lora_segments *sg, int in_features)
{
    sg->fused_shrink.clear();
    sg->fused_expand.clear();
    sg->fused_grid = 0;
    const int cap_s = g_compute_units / kXcds, cap_e = 4 * cap_s;
    sg->decode_fused = opt_decode_single(sg) && sg->wide && sg->prefill_units.empty() && sg->expand_big_units.empty() &&
                       !sg->shrink_units.empty() && !sg->expand_units.empty() && sg->n_sync > 0 &&
                       sg->shrink_units.size() <= (size_t)g_compute_units &&
                       sg->expand_units.size() <= (size_t)(4 * g_compute_units) && g_compute_units % kXcds == 0;
    if (!sg->decode_fused) return;
    struct Tile {
        std::vector<int> s, e;
        int seg = -1;
        int64_t bytes = 0;
    };
    std::vector<Tile> tiles(sg->n_sync);
    auto s_bytes = [&](const Unit &u) { return 2 * (int64_t)in_features * (u.pn + u.ntok); };
    auto e_bytes = [&](const Unit &u) { return 2 * (int64_t)u.pn * (u.r8 + 2 * u.ntok); };
    for (size_t k = 0; k < sg->shrink_units.size(); ++k) {
        const Unit &u = sg->shrink_units[k];
        tiles[u.sync_idx].s.push_back((int)k);
        tiles[u.sync_idx].seg = u.seg;
        tiles[u.sync_idx].bytes += s_bytes(u);
    }
    for (size_t k = 0; k < sg->expand_units.size(); ++k) {
        const Unit &u = sg->expand_units[k];
        const int pass = u.r8 <= 32 ? 512 : (u.r8 <= 64 ? 256 : 128);
        if (u.pn > pass || u.ntok > lora::kTokTile) sg->decode_fused = false;  // not a single column pass
        tiles[u.sync_idx].e.push_back((int)k);
        tiles[u.sync_idx].bytes += e_bytes(u);
    }
    for (const Tile &t : tiles)
        if (t.s.empty() || t.e.empty() || (int)t.s.size() > cap_s || (int)t.e.size() > cap_e) sg->decode_fused = false;
    if (!sg->decode_fused) return;
    // groups (a group's tiles have consecutive counters), heaviest first
    std::vector<std::vector<int>> groups;
    for (int t = 0; t < sg->n_sync; ++t) {
        if (groups.empty() || tiles[groups.back().back()].seg != tiles[t].seg) groups.emplace_back();
        groups.back().push_back(t);
    }
    std::vector<int64_t> gbytes(groups.size(), 0);
    for (size_t g = 0; g < groups.size(); ++g)
        for (int t : groups[g]) gbytes[g] += tiles[t].bytes;
    std::vector<size_t> gorder(groups.size());
    for (size_t g = 0; g < gorder.size(); ++g) gorder[g] = g;
    std::stable_sort(gorder.begin(), gorder.end(), [&](size_t a, size_t b) { return gbytes[a] > gbytes[b]; });
    std::vector<std::vector<int>> on_xcd(kXcds);  // tiles of each XCD
    std::vector<int64_t> load(kXcds, 0);
    std::vector<int> ns(kXcds, 0), ne(kXcds, 0);
    auto place = [&](const std::vector<int> &ts) {
        int need_s = 0, need_e = 0;
        int64_t bytes = 0;
        for (int t : ts) {
            need_s += (int)tiles[t].s.size();
            need_e += (int)tiles[t].e.size();
            bytes += tiles[t].bytes;
        }
        int best = -1;
        for (int q = 0; q < kXcds; ++q)
            if (ns[q] + need_s <= cap_s && ne[q] + need_e <= cap_e && (best < 0 || load[q] < load[best])) best = q;
        if (best < 0) return false;
        for (int t : ts) on_xcd[best].push_back(t);
        ns[best] += need_s;
        ne[best] += need_e;
        load[best] += bytes;
        return true;
    };
    for (size_t g : gorder) {
        if (place(groups[g])) continue;
        for (int t : groups[g])
            if (!place(std::vector<int>{t})) {
                sg->decode_fused = false;
                return;
            }
    }
    // per XCD: the lists, the cut of the heaviest shrink units into row halves, the order
    std::vector<std::vector<Unit>> xs(kXcds), xe(kXcds);
    int rounds = 0;
    for (int q = 0; q < kXcds; ++q) {
        for (int t : on_xcd[q]) {
            for (int k : tiles[t].s) xs[q].push_back(sg->shrink_units[k]);
            for (int k : tiles[t].e) xe[q].push_back(sg->expand_units[k]);
        }
        std::stable_sort(xs[q].begin(), xs[q].end(), [&](const Unit &a, const Unit &b) { return s_bytes(a) > s_bytes(b); });
        const size_t n0 = xs[q].size();
        for (size_t k = 0; k < n0 && (int)xs[q].size() < cap_s; ++k) {
            if (xs[q][k].pn != lora::kRowTile) continue;
            Unit lo = xs[q][k], hi = xs[q][k];
            lo.pn = hi.pn = lora::kRowTile / 2;
            hi.p0 += lora::kRowTile / 2;
            hi.v_off += lora::kRowTile / 2;
            xs[q][k] = lo;
            xs[q].push_back(hi);
        }
        std::stable_sort(xs[q].begin(), xs[q].end(), [&](const Unit &a, const Unit &b) { return s_bytes(a) > s_bytes(b); });
        std::stable_sort(xe[q].begin(), xe[q].end(), [&](const Unit &a, const Unit &b) { return e_bytes(a) < e_bytes(b); });
        rounds = std::max(rounds, std::max((int)xs[q].size(), ((int)xe[q].size() + 3) / 4));
    }
    std::vector<int32_t> feeders(sg->n_sync, 0);
    for (int q = 0; q < kXcds; ++q)
        for (const Unit &u : xs[q]) ++feeders[u.sync_idx];
    sg->fused_grid = rounds * kXcds;
    Unit empty;
    memset(&empty, 0, sizeof empty);
    sg->fused_shrink.assign((size_t)sg->fused_grid, empty);
    sg->fused_expand.assign((size_t)sg->fused_grid * 4, empty);
    for (int q = 0; q < kXcds; ++q) {
        for (size_t j = 0; j < xs[q].size(); ++j) sg->fused_shrink[j * kXcds + q] = xs[q][j];
        for (size_t j = 0; j < xe[q].size(); ++j) {
            Unit u = xe[q][j];
            u.sync_n = feeders[u.sync_idx];
            sg->fused_expand[((j / 4) * kXcds + q) * 4 + j % 4] = u;
        }
    }
}

static lora_status_t plan_into(lora_segments *sg, const lora_pool *pool, const int32_t *ta, int32_t T,
                               int n_projections = 1)  // projections whose units share the launches
{
    const int N = pool->n_adapters;
    std::vector<int32_t> count(N, 0);
    int32_t n_active = 0;
    for (int32_t t = 0; t < T; ++t) {
        const int32_t a = ta[t];
        if (a == -1) continue;
        if (a < 0 || a >= N) return fail(LORA_ERR_INVALID_ARG, "token %d: adapter id %d outside -1..%d", t, a, N - 1);
        if (!pool->resident[a]) return fail(LORA_ERR_NOT_RESIDENT, "token %d: adapter %d is not loaded", t, a);
        ++count[a];
        ++n_active;
    }
    const int heavy_min_tokens = opt_heavy_min_tokens(sg), heavy_min_batch = opt_heavy_min_batch(sg);
    sg->pool = pool;
    sg->pool_id = pool->id;
    sg->layout_in = pool->in_features;
    sg->layout_out = pool->out_features;
    sg->T = T;
    sg->n_active = n_active;
    sg->uploaded = false;
    // Up to a few rounds of work groups, a unit takes the whole of k, so v needs no partial sums in
    // memory.  Very few units, or very many: k-slices, which spread a small batch over more compute
    // units and fill the last round of a large one better.
    int64_t whole_k_units = 0;
    for (int a = 0; a < N; ++a) {
        if (!count[a] || (count[a] >= heavy_min_tokens && n_active >= heavy_min_batch)) continue;
        whole_k_units += (int64_t)((pool->r8[a] + lora::kRowTile - 1) / lora::kRowTile) *
                         ((count[a] + lora::kTokTile - 1) / lora::kTokTile);
    }
    bool heavy_groups = false;
    for (int a = 0; a < N; ++a) heavy_groups |= count[a] >= heavy_min_tokens && n_active >= heavy_min_batch;
    sg->wide = whole_k_units >= kWholeKMin && whole_k_units <= opt_whole_k_limit(sg) &&
               pool->in_features <= opt_whole_k_max_in(sg) && !(opt_merged(sg) && heavy_groups);
    choose_k_slices(pool->in_features, &sg->wide_slices, &sg->wide_slice_len);
    // Whole-k units of many tokens pass up to twice the bytes of the others through their compute unit
    // (x beside A^T) and end the launch.  While the launch stays at one work group per compute unit,
    // the 16 rank rows of the units with the most tokens are cut into two units of 8, which share x
    // through the XCD's L2 as they already share A^T (cfg1: 217 -> 249 units, shrink launch 9.3 -> 8.9
    // us): split_min_tokens is the smallest token count whose units can all be cut within that budget.
    int split_min_tokens = 0;
    // (a batch that may run as one launch gets its row halves per XCD, in finish_decode_fused)
    const bool want_fused = opt_decode_single(sg) && sg->wide && !heavy_groups && n_projections == 1 &&
                            whole_k_units <= g_compute_units;
    if (sg->wide && !want_fused) {
        int64_t per_tokens[lora::kTokTile + 1] = {0};  // full 16-row units by their token count
        for (int a = 0; a < N; ++a) {
            if (!count[a] || (count[a] >= heavy_min_tokens && n_active >= heavy_min_batch)) continue;
            for (int tok0 = 0; tok0 < count[a]; tok0 += lora::kTokTile)
                per_tokens[std::min(lora::kTokTile, count[a] - tok0)] += pool->r8[a] / lora::kRowTile;
        }
        int64_t extra = 0;
        for (int m = lora::kTokTile; m >= kSplitRowsFloor && whole_k_units + extra + per_tokens[m] <= g_compute_units; --m) {
            extra += per_tokens[m];
            if (per_tokens[m]) split_min_tokens = m;
        }
    }
    if (sg->wide) {
        sg->n_k_slices = 1;
        sg->k_slice_len = pool->in_features;
    } else {
        sg->n_k_slices = sg->wide_slices;
        sg->k_slice_len = sg->wide_slice_len;
    }

    sg->seg_start.clear();
    sg->seg_adapter.clear();
    sg->seg_epoch.clear();
    sg->segs.clear();
    std::vector<int32_t> seg_of(N, -1), cursor(N, 0);
    int32_t pos = 0;
    int64_t voff = 0, wbytes = 0;
    for (int a = 0; a < N; ++a) {
        if (!count[a]) continue;
        SegRec r;
        memset(&r, 0, sizeof r);
        r.a_off = pool->a_off[a];
        r.b_off = pool->b_off[a];
        r.v_off = voff;
        r.rank = pool->rank[a];
        r.r8 = pool->r8[a];
        r.scale = pool->scale[a];
        r.tok_start = pos;
        r.ntok = count[a];
        seg_of[a] = (int32_t)sg->segs.size();
        cursor[a] = pos;
        sg->segs.push_back(r);
        sg->seg_start.push_back(pos);
        sg->seg_adapter.push_back(a);
        sg->seg_epoch.push_back(pool->epoch[a]);
        pos += count[a];
        voff += (int64_t)count[a] * r.r8;
        wbytes += 2LL * r.r8 * ((int64_t)pool->in_features + pool->out_features);
    }
    sg->seg_start.push_back(pos);
    sg->v_floats = voff;
    sg->weight_bytes = wbytes;

    sg->perm.assign(n_active, 0);
    sg->v_offset.assign(T, -1);
    for (int32_t t = 0; t < T; ++t) {
        const int32_t a = ta[t];
        if (a < 0) continue;
        const SegRec &r = sg->segs[seg_of[a]];
        const int32_t p = cursor[a]++;
        sg->perm[p] = t;
        sg->v_offset[t] = r.v_off + (int64_t)(p - r.tok_start) * r.r8;
    }

    // work units, heaviest adapters first so the launch's tail is made of small units
    std::vector<int32_t> order(sg->segs.size());
    for (size_t i = 0; i < order.size(); ++i) order[i] = (int32_t)i;
    std::stable_sort(order.begin(), order.end(),
                     [&](int32_t x, int32_t y) { return sg->segs[x].r8 > sg->segs[y].r8; });
    sg->shrink_units.clear();
    sg->prefill_units.clear();
    sg->expand_units.clear();
    sg->expand_big_units.clear();
    const int out = pool->out_features;
    auto fill_tokens = [&](Unit &u, const SegRec &r) {
        u.perm_off = r.tok_start + u.tok0;
        for (int q = 0; q < 16; ++q) u.tok[q] = sg->perm[r.tok_start + u.tok0 + (q < u.ntok ? q : 0)];
    };
    // counters of the hand-over of v: one per (group, token tile)
    std::vector<int32_t> sync_base(sg->segs.size(), 0);
    int n_sync = 0;
    for (size_t si = 0; si < sg->segs.size(); ++si) {
        sync_base[si] = n_sync;
        n_sync += (sg->segs[si].ntok + lora::kTokTile - 1) / lora::kTokTile;
    }
    sg->n_sync = n_sync;
    sg->has_big_units = false;
    sg->heavy_small_expand = false;
    sg->n_prefill_hi = 0;
    // A launch of few token-heavy shrink units lasts as long as one unit's walk through k (a wavefront
    // takes a quarter of k in passes of 128, one trip to memory each); such units are cut into k-slices.
    int64_t heavy_units = 0;
    for (const SegRec &r : sg->segs)
        if (r.ntok >= heavy_min_tokens && n_active >= heavy_min_batch)
            heavy_units += (r.ntok + heavy_tile(r.r8) - 1) / heavy_tile(r.r8);
    int heavy_k_slices = 1;
    if (sg->n_k_slices >= 2 && heavy_units > 0) {
        const int64_t limit = opt_heavy_k_cut_max_units(sg, pool->in_features);
        for (int c = std::min(4, sg->n_k_slices); c >= 2 && heavy_k_slices == 1; c /= 2)
            if (heavy_units * c <= limit) heavy_k_slices = c;  // per projection: lora_apply_multi gives the bits of separate applies
    }
    // The 64-token expand units: a group's columns in 4 runs, or in 8 shorter ones while that keeps the
    // launch at few such units (it then lasts as long as one of them; cfg3's routing at 1.5 k / 2.7 k
    // tokens: expand launch 25.7 -> 19.5 / 26.6 -> 23.1 us at 4096 columns, 78.6 -> 60.8 / 80.5 -> 72.8
    // us at 14336; at 4.9 k tokens and beyond 8 runs are level or lose).
    int64_t big_tiles = 0;
    for (const SegRec &r : sg->segs)
        if (r.ntok >= heavy_min_tokens && n_active >= heavy_min_batch && r.r8 <= kBigExpandMaxRank) big_tiles += (r.ntok + 63) / 64;
    const int big_runs = big_tiles * 8 * n_projections <= opt_big_runs_max_units(sg) ? 8 : 4;
    for (int32_t si : order) {
        const SegRec &r = sg->segs[si];
        const bool token_heavy = r.ntok >= heavy_min_tokens && n_active >= heavy_min_batch;
        const int sync_n = ((r.r8 + lora::kRowTile - 1) / lora::kRowTile) * sg->n_k_slices;
        if (token_heavy) {
            // shrink: tiles of 32 tokens (64 for ranks 65..192), all rank rows, all of k or
            // (heavy_k_slices > 1) a slice of it, the slices' sums meeting at the counter of the tile's
            // first 16 tokens
            sg->has_big_units = true;
            if (r.r8 > kBigExpandMaxRank) sg->heavy_small_expand = true;
            const int tile = heavy_tile(r.r8);
            for (int tok0 = 0; tok0 < r.ntok; tok0 += tile)
                for (int ks = 0; ks < heavy_k_slices; ++ks) {
                    Unit u;
                    memset(&u, 0, sizeof u);
                    u.seg = si;
                    u.tok0 = tok0;
                    u.ntok = std::min(tile, r.ntok - tok0);
                    u.p0 = 0;
                    u.pn = r.r8;
                    u.ks = ks;
                    u.r8 = r.r8;
                    u.scale = r.scale;
                    u.w_off = r.a_off;
                    u.v_off = r.v_off + (int64_t)tok0 * r.r8;
                    u.sync_idx = sync_base[si] + tok0 / lora::kTokTile;
                    u.sync_n = heavy_k_slices;
                    fill_tokens(u, r);
                    sg->prefill_units.push_back(u);
                    if (r.r8 > 64) ++sg->n_prefill_hi;
                }
        } else {
            for (int row0 = 0; row0 < r.r8; row0 += lora::kRowTile)
                for (int ks = 0; ks < sg->n_k_slices; ++ks)
                    for (int tok0 = 0; tok0 < r.ntok; tok0 += lora::kTokTile) {
                        const int ntok = std::min(lora::kTokTile, r.ntok - tok0);
                        const int rows = std::min(lora::kRowTile, r.r8 - row0);
                        // w_off stays the start of the 16-row block of A^T the unit's rows lie in
                        const int halves = split_min_tokens && rows == lora::kRowTile && ntok >= split_min_tokens ? 2 : 1;
                        for (int hf = 0; hf < halves; ++hf) {
                            Unit u;
                            memset(&u, 0, sizeof u);
                            u.seg = si;
                            u.tok0 = tok0;
                            u.ntok = ntok;
                            u.p0 = row0 + hf * (rows / halves);
                            u.pn = rows / halves;
                            u.ks = ks;
                            u.r8 = r.r8;
                            u.scale = r.scale;
                            u.w_off = r.a_off + (uint64_t)row0 * pool->in_features;
                            u.v_off = r.v_off + (int64_t)tok0 * r.r8 + u.p0;
                            u.sync_idx = sync_base[si] + tok0 / lora::kTokTile;
                            u.sync_n = sync_n;
                            fill_tokens(u, r);
                            sg->shrink_units.push_back(u);
                        }
                    }
        }
        // expand: small groups one column pass and <= 16 tokens per unit; token-heavy groups 64 tokens
        // (16 per wavefront, v kept in registers) and a quarter (or an eighth) of the columns, at least 512
        int cols = expand_cols_per_unit(r.r8, out);
        int etile = lora::kTokTile;
        if (token_heavy && r.r8 <= kBigExpandMaxRank) {
            etile = 64;
            cols = std::min(out, std::max(512, (out / big_runs + 127) / 128 * 128));
        }
        auto emit = [&](int c0, int tok0) {
            Unit u;
            memset(&u, 0, sizeof u);
            u.seg = si;
            u.tok0 = tok0;
            u.ntok = std::min(etile, r.ntok - tok0);
            u.p0 = c0;
            u.pn = std::min(cols, out - c0);
            u.r8 = r.r8;
            u.scale = r.scale;
            u.w_off = r.b_off + (uint64_t)c0 * r.r8;
            u.v_off = r.v_off + (int64_t)tok0 * r.r8;
            u.sync_idx = sync_base[si] + tok0 / lora::kTokTile;
            u.sync_n = sync_n;
            fill_tokens(u, r);
            (etile > lora::kTokTile ? sg->expand_big_units : sg->expand_units).push_back(u);
        };
        const int ncb = (out + cols - 1) / cols;
        if (etile > lora::kTokTile && (ncb == 2 || ncb == 4 || ncb == 8)) {
            // Work group b of a launch runs on XCD b mod 8, each XCD with an L2 of its own.  With the
            // units of a group in rows of 8 (each column run with 8 / ncb consecutive token tiles) a
            // column run's rows of B^T are fetched by 8 / ncb XCDs instead of all eight (cfg2 4096->4096:
            // 276 -> 231 MB fetched per launch for 185 MB of y, 78.5 -> 75.3 us).
            const int tiles_per_row = 8 / ncb;
            const int ntiles = (r.ntok + etile - 1) / etile;
            for (int t0 = 0; t0 < ntiles; t0 += tiles_per_row)
                for (int cb = 0; cb < ncb; ++cb)
                    for (int t = t0; t < std::min(ntiles, t0 + tiles_per_row); ++t) emit(cb * cols, t * etile);
        } else {
            for (int c0 = 0; c0 < out; c0 += cols)
                for (int tok0 = 0; tok0 < r.ntok; tok0 += etile) emit(c0, tok0);
        }
    }

    order_units_by_xcd(sg->shrink_units);
    order_heavy_units_by_xcd(sg->prefill_units);

    if (n_projections == 1)
        finish_decode_fused(sg, pool->in_features);
    else
        sg->decode_fused = false;
    // row order of the adapted layer: groups in table order, each padded to a multiple of 16 places, then
    // the tokens without adapter, the whole padded to a multiple of the kernel's row tile
    sg->lin_rows.clear();
    sg->lin_blocks.clear();
    if (n_projections == 1 && T > 0) {
        auto add_group = [&](const int32_t *toks, int n, const SegRec *r) {
            for (int t0 = 0; t0 < n; t0 += 16) {
                LinBlock b;
                memset(&b, 0, sizeof b);
                b.ntok = std::min(16, n - t0);
                if (r) {
                    b.b_off = r->b_off;
                    b.v_off = r->v_off + (int64_t)t0 * r->r8;
                    b.r8 = r->r8;
                    b.scale = r->scale;
                }
                sg->lin_blocks.push_back(b);
                for (int q = 0; q < 16; ++q) sg->lin_rows.push_back(q < b.ntok ? toks[t0 + q] : -1);
            }
        };
        for (const SegRec &r : sg->segs) add_group(sg->perm.data() + r.tok_start, r.ntok, &r);
        std::vector<int32_t> none;
        for (int32_t t = 0; t < T; ++t)
            if (ta[t] < 0) none.push_back(t);
        add_group(none.data(), (int)none.size(), nullptr);
        while (sg->lin_rows.size() % lora::kLinTileM) {
            LinBlock b;
            memset(&b, 0, sizeof b);
            sg->lin_blocks.push_back(b);
            sg->lin_rows.insert(sg->lin_rows.end(), 16, -1);
        }
    }
    layout_table(sg);
    return LORA_OK;
}

static lora_segments *new_segments()
{
    lora_segments *sg = new (std::nothrow) lora_segments();
    if (!sg) return nullptr;
    sg->magic = kSegMagic;
    sg->dev = nullptr;
    sg->dev_capacity = 0;
    sg->staging = nullptr;
    sg->staging_capacity = 0;
    sg->copied = nullptr;
    sg->side = nullptr;
    sg->fork = sg->join = nullptr;
    sg->uploaded = false;
    sg->n_sync = 0;
    sg->launches = 0;
    sg->caller_memory = false;
    sg->opts = kDefaultOptions;
    return sg;
}

extern "C" lora_status_t lora_segments_destroy(lora_segments_t *seg)
try {
    if (!seg) return LORA_OK;
    if (!seg_ok(seg)) return fail(LORA_ERR_INVALID_ARG, "not a segment object");
    lora_status_t st = LORA_OK;
    if (seg->copied) {
        (void)hipEventSynchronize(seg->copied);
        (void)hipEventDestroy(seg->copied);
    }
    if (seg->side) {
        (void)hipStreamSynchronize(seg->side);
        (void)hipStreamDestroy(seg->side);
    }
    if (seg->fork) (void)hipEventDestroy(seg->fork);
    if (seg->join) (void)hipEventDestroy(seg->join);
    if (seg->dev && !seg->caller_memory) {
        hipError_t e = hipFree(seg->dev);
        if (e != hipSuccess) st = hip_fail(e, "hipFree(segment table)");
    }
    if (seg->staging && !seg->caller_memory) {
        hipError_t e = hipHostFree(seg->staging);
        if (e != hipSuccess) st = hip_fail(e, "hipHostFree(segment staging)");
    }
    seg->magic = 0;
    delete seg;
    return st;
}
API_CATCH

// Owns a segment object until it is handed to the caller, so that an early return or an exception
// on the way does not leak it (or its device table).
struct SegmentsGuard {
    lora_segments *sg;
    explicit SegmentsGuard(lora_segments *s) : sg(s) {}
    ~SegmentsGuard()
    {
        if (sg) (void)lora_segments_destroy(sg);
    }
    lora_segments *release()
    {
        lora_segments *s = sg;
        sg = nullptr;
        return s;
    }
    SegmentsGuard(const SegmentsGuard &) = delete;
    SegmentsGuard &operator=(const SegmentsGuard &) = delete;
};

static lora_status_t check_options(const lora_plan_options_t *o)
{
    if (!o) return LORA_OK;
    if (o->whole_k_limit < -1) return fail(LORA_ERR_INVALID_ARG, "options: whole_k_limit = %d", o->whole_k_limit);
    const int32_t sizes[5] = {o->whole_k_max_in, o->heavy_min_tokens, o->heavy_min_batch, o->heavy_k_cut_max_units,
                              o->big_runs_max_units};
    for (int32_t v : sizes)
        if (v < -1) return fail(LORA_ERR_INVALID_ARG, "options: a threshold is %d (-1 = built in)", v);
    if (o->heavy_min_tokens == 0) return fail(LORA_ERR_INVALID_ARG, "options: heavy_min_tokens = 0");
    const int32_t flags[4] = {o->merged_launches, o->side_stream, o->fused_apply, o->decode_single_launch};
    for (int32_t f : flags)
        if (f < -1 || f > 1) return fail(LORA_ERR_INVALID_ARG, "options: a switch is %d, not -1, 0 or 1", f);
    return LORA_OK;
}

extern "C" lora_status_t lora_segments_plan_opts(const lora_pool_t *pool, const int32_t *ta, int32_t T,
                                                 const lora_plan_options_t *options, lora_segments_t **out)
try {
    if (!out) return fail(LORA_ERR_INVALID_ARG, "out is NULL");
    *out = nullptr;
    if (!pool_ok(pool)) return fail(LORA_ERR_INVALID_ARG, "pool is NULL or not a pool");
    if (T < 0) return fail(LORA_ERR_INVALID_ARG, "T = %d", T);
    if (T > 0 && !ta) return fail(LORA_ERR_INVALID_ARG, "token_adapter_host is NULL");
    lora_status_t st = check_options(options);
    if (st != LORA_OK) return st;
    SegmentsGuard g(new_segments());
    if (!g.sg) return fail(LORA_ERR_OOM, "host allocation failed");
    if (options) g.sg->opts = *options;
    st = plan_into(g.sg, pool, ta, T);
    if (st != LORA_OK) return st;
    *out = g.release();
    return LORA_OK;
}
API_CATCH

extern "C" lora_status_t lora_segments_plan(const lora_pool_t *pool, const int32_t *ta, int32_t T,
                                            lora_segments_t **out)
{
    return lora_segments_plan_opts(pool, ta, T, nullptr, out);
}

extern "C" lora_status_t lora_segments_set_options(lora_segments_t *sg, const lora_plan_options_t *options)
try {
    if (!seg_ok(sg)) return fail(LORA_ERR_INVALID_ARG, "seg is NULL or not a segment object");
    lora_status_t st = check_options(options);
    if (st != LORA_OK) return st;
    sg->opts = options ? *options : kDefaultOptions;
    return LORA_OK;
}
API_CATCH

static lora_status_t ranges_to_tokens(const lora_pool_t *pool, const int32_t *start, const int32_t *adapter,
                                      int32_t S, std::vector<int32_t> *ta)
{
    if (!pool_ok(pool)) return fail(LORA_ERR_INVALID_ARG, "pool is NULL or not a pool");
    if (S < 0) return fail(LORA_ERR_INVALID_ARG, "S = %d", S);
    if (!start || (S > 0 && !adapter)) return fail(LORA_ERR_INVALID_ARG, "seg_start_host or seg_adapter_host is NULL");
    if (start[0] != 0) return fail(LORA_ERR_INVALID_ARG, "seg_start_host[0] = %d, must be 0", start[0]);
    for (int32_t i = 0; i < S; ++i)
        if (start[i + 1] < start[i]) return fail(LORA_ERR_INVALID_ARG, "seg_start_host decreases at %d", i + 1);
    ta->assign((size_t)start[S], -1);
    for (int32_t i = 0; i < S; ++i)
        for (int32_t t = start[i]; t < start[i + 1]; ++t) (*ta)[t] = adapter[i];
    return LORA_OK;
}

extern "C" lora_status_t lora_segments_plan_ranges(const lora_pool_t *pool, const int32_t *start,
                                                   const int32_t *adapter, int32_t S, lora_segments_t **out)
try {
    if (!out) return fail(LORA_ERR_INVALID_ARG, "out is NULL");
    *out = nullptr;
    std::vector<int32_t> ta;
    lora_status_t st = ranges_to_tokens(pool, start, adapter, S, &ta);
    if (st != LORA_OK) return st;
    return lora_segments_plan(pool, ta.data(), (int32_t)ta.size(), out);
}
API_CATCH

// Plans every projection on its own, then strings the unit lists together.
static lora_status_t plan_multi_into(lora_segments *sg, const std::vector<const lora_pool *> &pools,
                                     const int32_t *ta, int32_t T)
{
    const lora_pool *p0 = pools[0];
    const uint16_t *base = p0->arena;
    for (const lora_pool *q : pools) {
        if (q->in_features != p0->in_features || q->rank != p0->rank || q->scale != p0->scale)
            return fail(LORA_ERR_SHAPE, "the pools of one multi-projection object must agree in in_features, ranks and scales");
        if (((uintptr_t)q->arena - (uintptr_t)p0->arena) % 2) return fail(LORA_ERR_INVALID_ARG, "arena alignment");
        base = std::min(base, (const uint16_t *)q->arena);
    }
    lora_status_t st = plan_into(sg, p0, ta, T, (int)pools.size());
    if (st != LORA_OK) return st;
    sg->mpools = pools;
    sg->mpool_ids.clear();
    sg->msegs.clear();
    sg->mepochs.clear();
    sg->mouts.clear();
    sg->mdelta.clear();
    const int64_t v_one = sg->v_floats;
    const int sync_one = sg->n_sync;
    auto shift = [](std::vector<Unit> &units, size_t from, uint64_t delta, int64_t vbase, int sync, int col) {
        for (size_t i = from; i < units.size(); ++i) {
            units[i].w_off += delta;
            units[i].v_off += vbase;
            units[i].sync_idx += sync;
            units[i].p0 += col;  // only the expand lists get a column base
        }
    };
    const uint64_t delta0 = (uint64_t)(((uintptr_t)p0->arena - (uintptr_t)base) / 2);
    shift(sg->shrink_units, 0, delta0, 0, 0, 0);
    shift(sg->prefill_units, 0, delta0, 0, 0, 0);
    shift(sg->expand_units, 0, delta0, 0, 0, 0);
    shift(sg->expand_big_units, 0, delta0, 0, 0, 0);
    sg->mpool_ids.push_back(p0->id);
    sg->msegs.push_back(sg->segs);
    sg->mepochs.push_back(sg->seg_epoch);
    sg->mouts.push_back(p0->out_features);
    sg->mdelta.push_back(delta0);
    int col = p0->out_features;
    int64_t weight_bytes = sg->weight_bytes;
    std::unique_ptr<lora_segments> tmp_owner(new (std::nothrow) lora_segments());  // host lists only
    lora_segments *tmp = tmp_owner.get();
    if (!tmp) return fail(LORA_ERR_OOM, "host allocation failed");
    tmp->opts = sg->opts;
    for (size_t q = 1; q < pools.size(); ++q) {
        st = plan_into(tmp, pools[q], ta, T, (int)pools.size());
        if (st != LORA_OK) break;
        const uint64_t delta = (uint64_t)(((uintptr_t)pools[q]->arena - (uintptr_t)base) / 2);
        const size_t n0 = sg->shrink_units.size(), n1 = sg->prefill_units.size(), n2 = sg->expand_units.size(),
                     n3 = sg->expand_big_units.size();
        sg->shrink_units.insert(sg->shrink_units.end(), tmp->shrink_units.begin(), tmp->shrink_units.end());
        sg->prefill_units.insert(sg->prefill_units.end(), tmp->prefill_units.begin(), tmp->prefill_units.end());
        sg->expand_units.insert(sg->expand_units.end(), tmp->expand_units.begin(), tmp->expand_units.end());
        sg->expand_big_units.insert(sg->expand_big_units.end(), tmp->expand_big_units.begin(),
                                    tmp->expand_big_units.end());
        shift(sg->shrink_units, n0, delta, (int64_t)q * v_one, (int)q * sync_one, 0);
        shift(sg->prefill_units, n1, delta, (int64_t)q * v_one, (int)q * sync_one, 0);
        shift(sg->expand_units, n2, delta, (int64_t)q * v_one, (int)q * sync_one, col);
        shift(sg->expand_big_units, n3, delta, (int64_t)q * v_one, (int)q * sync_one, col);
        sg->n_prefill_hi += tmp->n_prefill_hi;
        sg->heavy_small_expand = sg->heavy_small_expand || tmp->heavy_small_expand;
        sg->mpool_ids.push_back(pools[q]->id);
        sg->msegs.push_back(tmp->segs);
        sg->mepochs.push_back(tmp->seg_epoch);
        sg->mouts.push_back(pools[q]->out_features);
        sg->mdelta.push_back(delta);
        col += pools[q]->out_features;
        weight_bytes += tmp->weight_bytes;
    }
    if (st != LORA_OK) return st;
    sg->out_total = col;
    sg->v_floats = v_one * (int64_t)pools.size();
    sg->n_sync = sync_one * (int)pools.size();
    sg->weight_bytes = weight_bytes;
    // (several projections in one launch: the one-launch decode form is planned for single pools only)
    sg->decode_fused = false;
    sg->fused_shrink.clear();
    sg->fused_expand.clear();
    sg->fused_grid = 0;
    sg->lin_rows.clear();
    sg->lin_blocks.clear();
    layout_table(sg);
    return LORA_OK;
}

static lora_status_t check_pool_list(const lora_pool_t *const *pools, int32_t n, std::vector<const lora_pool *> *out)
{
    if (!pools || n < 1 || n > LORA_MAX_PROJECTIONS)
        return fail(LORA_ERR_INVALID_ARG, "pools is NULL or n_pools = %d outside 1..%d", n, LORA_MAX_PROJECTIONS);
    for (int32_t q = 0; q < n; ++q) {
        if (!pool_ok(pools[q])) return fail(LORA_ERR_INVALID_ARG, "pools[%d] is NULL or not a pool", q);
        out->push_back(pools[q]);
    }
    return LORA_OK;
}

extern "C" lora_status_t lora_segments_plan_multi(const lora_pool_t *const *pools, int32_t n_pools,
                                                  const int32_t *ta, int32_t T, lora_segments_t **out)
{
    return lora_segments_plan_multi_opts(pools, n_pools, ta, T, nullptr, out);
}

extern "C" lora_status_t lora_segments_plan_multi_opts(const lora_pool_t *const *pools, int32_t n_pools,
                                                       const int32_t *ta, int32_t T,
                                                       const lora_plan_options_t *options, lora_segments_t **out)
try {
    if (!out) return fail(LORA_ERR_INVALID_ARG, "out is NULL");
    *out = nullptr;
    std::vector<const lora_pool *> list;
    lora_status_t st = check_pool_list(pools, n_pools, &list);
    if (st != LORA_OK) return st;
    if (T < 0) return fail(LORA_ERR_INVALID_ARG, "T = %d", T);
    if (T > 0 && !ta) return fail(LORA_ERR_INVALID_ARG, "token_adapter_host is NULL");
    if ((st = check_options(options)) != LORA_OK) return st;
    SegmentsGuard g(new_segments());
    if (!g.sg) return fail(LORA_ERR_OOM, "host allocation failed");
    if (options) g.sg->opts = *options;
    st = plan_multi_into(g.sg, list, ta, T);
    if (st != LORA_OK) return st;
    *out = g.release();
    return LORA_OK;
}
API_CATCH

// What the library found out about a device at the first upload there: whether it is the chip the
// planner's constants describe (gfx950, at least g_compute_units compute units) and, from one probe
// launch, whether the work groups of one residue mod 8 share an XCD (xcc_map: 4 bits per XCD number, the
// residue found there).  The one-launch decode form needs both; everything else runs without them.
struct DeviceProfile {
    std::atomic<int> state{0};  // 0 unknown, 1 one-launch decode form usable, 2 not usable
    std::atomic<unsigned> xcc_map{0};
};
static DeviceProfile g_profile[lora::kMaxDevices];

static lora_status_t device_profile(hipStream_t s, DeviceProfile **out)
{
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= lora::kMaxDevices) return fail(LORA_ERR_DEVICE, "device %d outside 0..%d", dev, lora::kMaxDevices - 1);
    DeviceProfile &p = g_profile[dev];
    *out = &p;
    if (p.state.load(std::memory_order_acquire)) return LORA_OK;
    hipStreamCaptureStatus capturing = hipStreamCaptureStatusNone;
    HIP_TRY(hipStreamIsCapturing(s, &capturing));
    if (capturing != hipStreamCaptureStatusNone) return LORA_OK;  // no probe under capture: stays unknown
    hipDeviceProp_t prop;
    HIP_TRY(hipGetDeviceProperties(&prop, dev));
    if (strncmp(prop.gcnArchName, "gfx950", 6) != 0)
        return fail(LORA_ERR_DEVICE, "device %d is %s: this library's kernels and planner are for gfx950", dev,
                    prop.gcnArchName);
    bool ok = prop.multiProcessorCount >= g_compute_units;
    unsigned map = 0;
    if (ok) {
        std::vector<unsigned> xcc((size_t)g_compute_units);
        HIP_TRY(lora::probe_xcc(xcc.data(), g_compute_units, s));
        // work groups of one residue mod 8 on one XCD, eight different XCDs numbered 0..7; the map gives
        // each XCD number the residue it had in this launch (launches may start at another XCD)
        bool seen[16] = {false};
        for (int r = 0; r < kXcds && ok; ++r) {
            for (int b = r; b < g_compute_units; b += kXcds) ok = ok && xcc[b] == xcc[r];
            ok = ok && xcc[r] < (unsigned)kXcds && !seen[xcc[r] & 15];
            seen[xcc[r] & 15] = true;
            if (ok) map |= (unsigned)r << (4 * xcc[r]);
        }
    }
    p.xcc_map.store(map, std::memory_order_relaxed);
    p.state.store(ok ? 1 : 2, std::memory_order_release);
    return LORA_OK;
}

static lora_status_t upload_table(lora_segments *sg, hipStream_t s)
{
    DeviceProfile *prof = nullptr;
    lora_status_t pst = device_profile(s, &prof);
    if (pst != LORA_OK) return pst;
    if (!sg->copied) HIP_TRY(hipEventCreateWithFlags(&sg->copied, hipEventDisableTiming));
    // the previous upload may still be reading the staging buffer
    HIP_TRY(hipEventSynchronize(sg->copied));
    if (sg->caller_memory) {
        if (sg->table_bytes > sg->dev_capacity || sg->table_bytes > sg->staging_capacity)
            return fail(LORA_ERR_OOM, "the batch's table needs %zu bytes; the caller's device table holds %zu, its staging %zu",
                        sg->table_bytes, sg->dev_capacity, sg->staging_capacity);
    } else {
        if (sg->table_bytes > sg->staging_capacity) {
            if (sg->staging) HIP_TRY(hipHostFree(sg->staging));
            sg->staging = nullptr;
            sg->staging_capacity = 0;
            const size_t cap = round_up_sz(sg->table_bytes * 2, 4096);
            HIP_TRY(hipHostMalloc((void **)&sg->staging, cap, hipHostMallocDefault));
            sg->staging_capacity = cap;
        }
        if (sg->table_bytes > sg->dev_capacity) {
            if (sg->dev) HIP_TRY(hipFree(sg->dev));
            sg->dev = nullptr;
            sg->dev_capacity = 0;
            const size_t cap = round_up_sz(sg->table_bytes * 2, 4096);
            HIP_TRY(hipMalloc((void **)&sg->dev, cap));
            sg->dev_capacity = cap;
        }
    }
    if (!sg->perm.empty()) memcpy(sg->staging + sg->off_perm, sg->perm.data(), sg->perm.size() * sizeof(int32_t));
    if (!sg->expand_big_units.empty())
        memcpy(sg->staging + sg->off_expand_big, sg->expand_big_units.data(),
               sg->expand_big_units.size() * sizeof(Unit));
    if (!sg->prefill_units.empty())
        memcpy(sg->staging + sg->off_prefill, sg->prefill_units.data(), sg->prefill_units.size() * sizeof(Unit));
    if (!sg->shrink_units.empty())
        memcpy(sg->staging + sg->off_shrink, sg->shrink_units.data(), sg->shrink_units.size() * sizeof(Unit));
    if (!sg->expand_units.empty())
        memcpy(sg->staging + sg->off_expand, sg->expand_units.data(), sg->expand_units.size() * sizeof(Unit));
    if (!sg->fused_shrink.empty())
        memcpy(sg->staging + sg->off_fused_shrink, sg->fused_shrink.data(), sg->fused_shrink.size() * sizeof(Unit));
    if (!sg->fused_expand.empty())
        memcpy(sg->staging + sg->off_fused_expand, sg->fused_expand.data(), sg->fused_expand.size() * sizeof(Unit));
    if (!sg->lin_rows.empty())
        memcpy(sg->staging + sg->off_lin_rows, sg->lin_rows.data(), sg->lin_rows.size() * sizeof(int32_t));
    if (!sg->lin_blocks.empty())
        memcpy(sg->staging + sg->off_lin_blocks, sg->lin_blocks.data(), sg->lin_blocks.size() * sizeof(LinBlock));
    memset(sg->staging + sg->off_sync, 0, sg->table_bytes - sg->off_sync);
    sg->launches = 0;
    if (sg->table_bytes) HIP_TRY(hipMemcpyAsync(sg->dev, sg->staging, sg->table_bytes, hipMemcpyHostToDevice, s));
    HIP_TRY(hipEventRecord(sg->copied, s));
    sg->uploaded = true;
    return LORA_OK;
}

extern "C" lora_status_t lora_segments_upload(lora_segments_t *sg, void *stream)
try {
    if (!seg_ok(sg)) return fail(LORA_ERR_INVALID_ARG, "seg is NULL or not a segment object");
    return upload_table(sg, (hipStream_t)stream);
}
API_CATCH

extern "C" lora_status_t lora_segments_table_bytes(const lora_segments_t *sg, size_t *bytes)
try {
    if (!seg_ok(sg)) return fail(LORA_ERR_INVALID_ARG, "seg is NULL or not a segment object");
    if (!bytes) return fail(LORA_ERR_INVALID_ARG, "bytes is NULL");
    *bytes = sg->table_bytes;
    return LORA_OK;
}
API_CATCH

extern "C" lora_status_t lora_segments_upload_to(lora_segments_t *sg, void *dev_table, size_t dev_bytes,
                                                 void *host_staging, size_t staging_bytes, void *stream)
try {
    if (!seg_ok(sg)) return fail(LORA_ERR_INVALID_ARG, "seg is NULL or not a segment object");
    if (!dev_table || ((uintptr_t)dev_table) % 256) return fail(LORA_ERR_INVALID_ARG, "dev_table is NULL or not 256-byte aligned");
    if (!host_staging || ((uintptr_t)host_staging) % 16) return fail(LORA_ERR_INVALID_ARG, "host_staging is NULL or not 16-byte aligned");
    if (dev_bytes < sg->table_bytes || staging_bytes < sg->table_bytes)
        return fail(LORA_ERR_OOM, "the batch's table needs %zu bytes (lora_segments_table_bytes); dev_table holds %zu, host_staging %zu",
                    sg->table_bytes, dev_bytes, staging_bytes);
    if (sg->copied) HIP_TRY(hipEventSynchronize(sg->copied));  // an upload from the library's own staging may be in flight
    if (!sg->caller_memory) {
        if (sg->dev) HIP_TRY(hipFree(sg->dev));
        sg->dev = nullptr;
        if (sg->staging) HIP_TRY(hipHostFree(sg->staging));
        sg->staging = nullptr;
    }
    sg->caller_memory = true;
    sg->dev = (char *)dev_table;
    sg->dev_capacity = dev_bytes;
    sg->staging = (char *)host_staging;
    sg->staging_capacity = staging_bytes;
    return upload_table(sg, (hipStream_t)stream);
}
API_CATCH

extern "C" lora_status_t lora_segments_build_multi(const lora_pool_t *const *pools, int32_t n_pools,
                                                   const int32_t *ta, int32_t T, void *stream,
                                                   lora_segments_t **out)
{
    return lora_segments_build_multi_opts(pools, n_pools, ta, T, nullptr, stream, out);
}

extern "C" lora_status_t lora_segments_build_multi_opts(const lora_pool_t *const *pools, int32_t n_pools,
                                                        const int32_t *ta, int32_t T,
                                                        const lora_plan_options_t *options, void *stream,
                                                        lora_segments_t **out)
try {
    lora_status_t st = lora_segments_plan_multi_opts(pools, n_pools, ta, T, options, out);
    if (st != LORA_OK) return st;
    st = lora_segments_upload(*out, stream);
    if (st != LORA_OK) {
        lora_segments_destroy(*out);
        *out = nullptr;
    }
    return st;
}
API_CATCH

extern "C" lora_status_t lora_segments_build(const lora_pool_t *pool, const int32_t *ta, int32_t T, void *stream,
                                             lora_segments_t **out)
{
    return lora_segments_build_opts(pool, ta, T, nullptr, stream, out);
}

extern "C" lora_status_t lora_segments_build_opts(const lora_pool_t *pool, const int32_t *ta, int32_t T,
                                                  const lora_plan_options_t *options, void *stream,
                                                  lora_segments_t **out)
try {
    lora_status_t st = lora_segments_plan_opts(pool, ta, T, options, out);
    if (st != LORA_OK) return st;
    st = lora_segments_upload(*out, stream);
    if (st != LORA_OK) {
        lora_segments_destroy(*out);
        *out = nullptr;
    }
    return st;
}
API_CATCH

extern "C" lora_status_t lora_segments_build_ranges(const lora_pool_t *pool, const int32_t *start,
                                                    const int32_t *adapter, int32_t S, void *stream,
                                                    lora_segments_t **out)
try {
    lora_status_t st = lora_segments_plan_ranges(pool, start, adapter, S, out);
    if (st != LORA_OK) return st;
    st = lora_segments_upload(*out, stream);
    if (st != LORA_OK) {
        lora_segments_destroy(*out);
        *out = nullptr;
    }
    return st;
}
API_CATCH

extern "C" lora_status_t lora_segments_rebuild(lora_segments_t *sg, const int32_t *ta, int32_t T, void *stream)
try {
    if (!seg_ok(sg)) return fail(LORA_ERR_INVALID_ARG, "seg is NULL or not a segment object");
    if (!pool_is(sg->pool, sg->pool_id))
        return fail(LORA_ERR_STALE_SEGMENTS, "the pool this segment object was built for no longer exists");
    if (T < 0) return fail(LORA_ERR_INVALID_ARG, "T = %d", T);
    if (T > 0 && !ta) return fail(LORA_ERR_INVALID_ARG, "token_adapter_host is NULL");
    lora_status_t st;
    if (sg->mpools.empty()) {
        st = plan_into(sg, sg->pool, ta, T);
    } else {
        const std::vector<const lora_pool *> pools = sg->mpools;
        for (size_t q = 0; q < pools.size(); ++q)
            if (!pool_is(pools[q], sg->mpool_ids[q]))
                return fail(LORA_ERR_STALE_SEGMENTS, "a pool this segment object was built for no longer exists");
        st = plan_multi_into(sg, pools, ta, T);
    }
    if (st != LORA_OK) {
        sg->uploaded = false;
        return st;
    }
    return upload_table(sg, (hipStream_t)stream);
}
API_CATCH

extern "C" lora_status_t lora_segments_info(const lora_segments_t *sg, lora_segments_info_t *info)
try {
    if (!seg_ok(sg)) return fail(LORA_ERR_INVALID_ARG, "seg is NULL or not a segment object");
    if (!info) return fail(LORA_ERR_INVALID_ARG, "info is NULL");
    info->n_tokens = sg->T;
    info->n_active = sg->n_active;
    info->n_segments = (int32_t)sg->segs.size();
    info->n_shrink_units = (int32_t)(sg->shrink_units.size() + sg->prefill_units.size());
    info->n_expand_units = (int32_t)(sg->expand_units.size() + sg->expand_big_units.size());
    info->n_k_slices = sg->n_k_slices;
    info->v_floats = sg->v_floats;
    info->weight_bytes = sg->weight_bytes;
    info->single_launch = sg->decode_fused ? 1 : 0;
    info->launch_work_groups = sg->decode_fused ? sg->fused_grid : 0;
    return LORA_OK;
}
API_CATCH

extern "C" lora_status_t lora_segments_export(const lora_segments_t *sg, int32_t *perm, int32_t *seg_start,
                                              int32_t *seg_adapter, int64_t *v_offset)
try {
    if (!seg_ok(sg)) return fail(LORA_ERR_INVALID_ARG, "seg is NULL or not a segment object");
    if (perm && !sg->perm.empty()) memcpy(perm, sg->perm.data(), sg->perm.size() * sizeof(int32_t));
    if (seg_start) memcpy(seg_start, sg->seg_start.data(), sg->seg_start.size() * sizeof(int32_t));
    if (seg_adapter && !sg->seg_adapter.empty())
        memcpy(seg_adapter, sg->seg_adapter.data(), sg->seg_adapter.size() * sizeof(int32_t));
    if (v_offset && !sg->v_offset.empty()) memcpy(v_offset, sg->v_offset.data(), sg->v_offset.size() * sizeof(int64_t));
    return LORA_OK;
}
API_CATCH

static void export_units(const std::vector<Unit> &units, int32_t *dst)
{
    for (size_t i = 0; i < units.size(); ++i) {
        const Unit &u = units[i];
        int32_t *d = dst + 6 * i;
        d[0] = u.seg; d[1] = u.tok0; d[2] = u.ntok; d[3] = u.p0; d[4] = u.pn; d[5] = u.ks;
    }
}

extern "C" lora_status_t lora_segments_export_units(const lora_segments_t *sg, int32_t *shrink_units,
                                                    int32_t *expand_units)
try {
    if (!seg_ok(sg)) return fail(LORA_ERR_INVALID_ARG, "seg is NULL or not a segment object");
    if (shrink_units) {
        export_units(sg->shrink_units, shrink_units);
        export_units(sg->prefill_units, shrink_units + 6 * sg->shrink_units.size());
    }
    if (expand_units) {
        export_units(sg->expand_units, expand_units);
        export_units(sg->expand_big_units, expand_units + 6 * sg->expand_units.size());
    }
    return LORA_OK;
}
API_CATCH

extern "C" lora_status_t lora_segments_export_launch_units(const lora_segments_t *sg, int32_t *shrink_units,
                                                           int32_t *expand_units)
try {
    if (!seg_ok(sg)) return fail(LORA_ERR_INVALID_ARG, "seg is NULL or not a segment object");
    if (!sg->decode_fused) return fail(LORA_ERR_INVALID_ARG, "the batch is not planned for the one-launch decode form");
    auto put = [](const std::vector<Unit> &units, int32_t *dst) {
        for (size_t i = 0; i < units.size(); ++i) {
            const Unit &u = units[i];
            int32_t *d = dst + 7 * i;
            d[0] = u.seg; d[1] = u.tok0; d[2] = u.ntok; d[3] = u.p0; d[4] = u.pn; d[5] = u.ks; d[6] = u.sync_idx;
        }
    };
    if (shrink_units) put(sg->fused_shrink, shrink_units);
    if (expand_units) put(sg->fused_expand, expand_units);
    return LORA_OK;
}
API_CATCH

// ------------------------------------------------------------------------------------------------
// hot path
// ------------------------------------------------------------------------------------------------
// A segment object may be launched on the pool it was planned for, or on another pool with the same
// layout (same feature sizes and ranks, hence the same offsets): the layers of a model that share a
// projection shape and an adapter set.  On such a sibling pool every adapter the batch uses must be
// resident.
// The unit records carry each used adapter's place, rank and scale.  An object may be launched on the
// pool it was planned for as long as none of the adapters it uses has been loaded, evicted or moved
// since, whatever happened to other adapters, and on any pool that holds the same adapters at the same
// places (the layers of a model).
static lora_status_t check_adapters(const lora_pool *pool, const lora_segments *sg, const std::vector<SegRec> &segs,
                                    const std::vector<uint64_t> &epochs, uint64_t planned_pool_id)
{
    if (sg->layout_in != pool->in_features)
        return fail(LORA_ERR_STALE_SEGMENTS, "segment object was built for a pool with other feature sizes");
    for (size_t i = 0; i < sg->seg_adapter.size(); ++i) {
        const int32_t a = sg->seg_adapter[i];
        const SegRec &r = segs[i];
        if (a >= pool->n_adapters)
            return fail(LORA_ERR_STALE_SEGMENTS, "segment object uses adapter %d, which this pool does not have", a);
        if (!pool->resident[a])
            return fail(LORA_ERR_NOT_RESIDENT, "adapter %d is used by the batch but not loaded in this pool", a);
        if (pool->rank[a] != r.rank || pool->scale[a] != r.scale || pool->a_off[a] != r.a_off ||
            pool->b_off[a] != r.b_off)
            return fail(LORA_ERR_STALE_SEGMENTS, "adapter %d has another rank, scale or place in this pool", a);
        if (planned_pool_id == pool->id && pool->epoch[a] != epochs[i])
            return fail(LORA_ERR_STALE_SEGMENTS,
                        "adapter %d was loaded, evicted or moved after the segment object was built", a);
    }
    return LORA_OK;
}

static lora_status_t check_launchable(const lora_pool *pool, const lora_segments *sg)
{
    if (!pool_ok(pool)) return fail(LORA_ERR_INVALID_ARG, "pool is NULL or not a pool");
    if (!seg_ok(sg)) return fail(LORA_ERR_INVALID_ARG, "seg is NULL or not a segment object");
    if (!sg->mpools.empty())
        return fail(LORA_ERR_INVALID_ARG, "segment object was built for several pools: use lora_apply_multi");
    if (sg->layout_out != pool->out_features)
        return fail(LORA_ERR_STALE_SEGMENTS, "segment object was built for a pool with other feature sizes");
    lora_status_t st = check_adapters(pool, sg, sg->segs, sg->seg_epoch, sg->pool_id);
    if (st != LORA_OK) return st;
    if (!sg->uploaded) return fail(LORA_ERR_INVALID_ARG, "segment object was planned but not uploaded");
    return LORA_OK;
}

static lora_status_t check_matrix(const void *p, int64_t ld, int cols, const char *name)
{
    if (!p) return fail(LORA_ERR_INVALID_ARG, "%s is NULL", name);
    if (((uintptr_t)p) % 16) return fail(LORA_ERR_INVALID_ARG, "%s is not 16-byte aligned", name);
    if (ld < cols || ld % 8) return fail(LORA_ERR_INVALID_ARG, "row stride of %s (%lld) must be >= %d and a multiple of 8",
                                         name, (long long)ld, cols);
    return LORA_OK;
}

static size_t partial_bytes(const lora_segments *sg)
{
    if (sg->n_k_slices <= 1) return 0;
    return round_up_sz((size_t)sg->n_k_slices * (size_t)sg->v_floats * 4, 256);
}

// lora_apply's workspace: [k-slices' fp32 partial sums of v | v as bf16 hi | v as bf16 lo]
static size_t apply_parts_bytes(const lora_segments *sg)
{
    return round_up_sz((size_t)std::max(1, sg->n_k_slices) * (size_t)sg->v_floats * 4, 256);
}
static size_t apply_packed_bytes(const lora_segments *sg) { return round_up_sz((size_t)sg->v_floats * 2, 256); }

enum UnitKind { kShrink, kPrefill, kExpand, kExpandBig, kFusedShrink, kFusedExpand };

static lora::LaunchCtx ctx_for(const uint16_t *arena, int in_features, int out_features, const lora_segments *sg,
                                UnitKind kind)
{
    lora::LaunchCtx c;
    const size_t off = kind == kShrink        ? sg->off_shrink
                       : kind == kPrefill     ? sg->off_prefill
                       : kind == kExpand      ? sg->off_expand
                       : kind == kExpandBig   ? sg->off_expand_big
                       : kind == kFusedShrink ? sg->off_fused_shrink
                                              : sg->off_fused_expand;
    const std::vector<Unit> &list = kind == kShrink        ? sg->shrink_units
                                    : kind == kPrefill     ? sg->prefill_units
                                    : kind == kExpand      ? sg->expand_units
                                    : kind == kExpandBig   ? sg->expand_big_units
                                    : kind == kFusedShrink ? sg->fused_shrink
                                                           : sg->fused_expand;
    c.units = (const Unit *)(sg->dev + off);
    c.perm = (const int32_t *)(sg->dev + sg->off_perm);
    c.arena = arena;
    c.n_units = (int)list.size();
    c.in_features = in_features;
    c.out_features = out_features;
    return c;
}

static lora::LaunchCtx ctx_for(const lora_pool *pool, const lora_segments *sg, UnitKind kind)
{
    return ctx_for(pool->arena, pool->in_features, pool->out_features, sg, kind);
}

extern "C" lora_status_t lora_workspace_bytes(const lora_pool_t *pool, const lora_segments_t *sg, size_t *bytes)
try {
    if (!pool_ok(pool)) return fail(LORA_ERR_INVALID_ARG, "pool is NULL or not a pool");
    if (!seg_ok(sg)) return fail(LORA_ERR_INVALID_ARG, "seg is NULL or not a segment object");
    if (!bytes) return fail(LORA_ERR_INVALID_ARG, "bytes is NULL");
    *bytes = partial_bytes(sg);
    return LORA_OK;
}
API_CATCH

extern "C" lora_status_t lora_apply_workspace_bytes(const lora_pool_t *pool, const lora_segments_t *sg, size_t *bytes)
try {
    if (!pool_ok(pool)) return fail(LORA_ERR_INVALID_ARG, "pool is NULL or not a pool");
    if (!seg_ok(sg)) return fail(LORA_ERR_INVALID_ARG, "seg is NULL or not a segment object");
    if (!bytes) return fail(LORA_ERR_INVALID_ARG, "bytes is NULL");
    *bytes = apply_parts_bytes(sg) + 2 * apply_packed_bytes(sg);
    return LORA_OK;
}
API_CATCH

static lora_status_t check_workspace(const void *ws, size_t have, size_t need)
{
    if (need == 0) return LORA_OK;
    if (!ws) return fail(LORA_ERR_WORKSPACE, "workspace is NULL but %zu bytes are required", need);
    if (((uintptr_t)ws) % 256) return fail(LORA_ERR_WORKSPACE, "workspace is not 256-byte aligned");
    if (have < need) return fail(LORA_ERR_WORKSPACE, "workspace of %zu bytes is smaller than the %zu required", have, need);
    return LORA_OK;
}

extern "C" lora_status_t lora_shrink(const lora_pool_t *pool, const lora_segments_t *sg, const void *x, int64_t ldx,
                                     float *v, void *workspace, size_t ws_bytes, void *stream)
try {
    lora_status_t st = check_launchable(pool, sg);
    if (st != LORA_OK) return st;
    if (sg->n_active == 0) return LORA_OK;
    if ((st = check_matrix(x, ldx, pool->in_features, "x")) != LORA_OK) return st;
    if (!v || ((uintptr_t)v) % 16) return fail(LORA_ERR_INVALID_ARG, "v is NULL or not 16-byte aligned");
    if ((st = check_workspace(workspace, ws_bytes, partial_bytes(sg))) != LORA_OK) return st;
    hipStream_t s = (hipStream_t)stream;
    const lora::LaunchCtx c = ctx_for(pool, sg, kShrink), cp = ctx_for(pool, sg, kPrefill);
    if (sg->wide) {
        HIP_TRY(lora::launch_shrink_wide(c, c.n_units > g_compute_units, (const uint16_t *)x, ldx, sg->wide_slice_len, sg->wide_slices, v, nullptr,
                                         nullptr, s));
        HIP_TRY(lora::launch_shrink_prefill(cp, sg->n_prefill_hi, (const uint16_t *)x, ldx, nullptr, nullptr, v, 1, 0, nullptr,
                                            nullptr, s));
    } else if (sg->n_k_slices <= 1) {
        HIP_TRY(lora::launch_shrink(c, (const uint16_t *)x, ldx, sg->k_slice_len, v, 1, 0, nullptr, s));
        HIP_TRY(lora::launch_shrink_prefill(cp, sg->n_prefill_hi, (const uint16_t *)x, ldx, nullptr, nullptr, v, 1, 0, nullptr,
                                            nullptr, s));
    } else {
        float *parts = (float *)workspace;
        HIP_TRY(lora::launch_shrink(c, (const uint16_t *)x, ldx, sg->k_slice_len, parts, sg->n_k_slices,
                                    sg->v_floats, nullptr, s));
        HIP_TRY(lora::launch_shrink_prefill(cp, sg->n_prefill_hi, (const uint16_t *)x, ldx, nullptr, nullptr, parts, sg->n_k_slices,
                                            sg->v_floats, nullptr, nullptr, s));
        HIP_TRY(lora::launch_reduce_slices(parts, sg->n_k_slices, sg->v_floats, v, sg->v_floats, s));
    }
    return LORA_OK;
}
API_CATCH

extern "C" lora_status_t lora_expand(const lora_pool_t *pool, const lora_segments_t *sg, const float *v, void *y,
                                     int64_t ldy, void *stream)
try {
    lora_status_t st = check_launchable(pool, sg);
    if (st != LORA_OK) return st;
    if (sg->n_active == 0) return LORA_OK;
    if ((st = check_matrix(y, ldy, pool->out_features, "y")) != LORA_OK) return st;
    if (!v || ((uintptr_t)v) % 16) return fail(LORA_ERR_INVALID_ARG, "v is NULL or not 16-byte aligned");
    HIP_TRY(lora::launch_expand(ctx_for(pool, sg, kExpand), false, v, 1, 0, (uint16_t *)y, ldy, nullptr,
                                (hipStream_t)stream));
    HIP_TRY(lora::launch_expand(ctx_for(pool, sg, kExpandBig), true, v, 1, 0, (uint16_t *)y, ldy, nullptr,
                                (hipStream_t)stream));
    return LORA_OK;
}
API_CATCH

static thread_local hipEvent_t g_prof[3] = {nullptr, nullptr, nullptr};
static const int kSideStreamMinUnits = 32;  // decode shrink units below which a second stream is not worth its events

extern "C" lora_status_t lora_set_fused_apply(int enabled)
try {
    g_fused_apply = enabled ? 1 : 0;
    return LORA_OK;
}
API_CATCH

extern "C" lora_status_t lora_set_decode_single_launch(int enabled)
try {
    g_decode_single_launch = enabled ? 1 : 0;
    return LORA_OK;
}
API_CATCH

extern "C" lora_status_t lora_set_merged_launches(int enabled)
try {
    g_merged_mixed = enabled ? 1 : 0;
    return LORA_OK;
}
API_CATCH

extern "C" lora_status_t lora_set_side_stream(int enabled)
try {
    g_side_stream = enabled ? 1 : 0;
    return LORA_OK;
}
API_CATCH

extern "C" lora_status_t lora_set_fused_wait_limit(uint32_t polls)
{
    g_spin_limit.store(polls ? polls : kSpinLimit);
    return LORA_OK;
}

extern "C" lora_status_t lora_segments_check(const lora_segments_t *sg, void *stream)
try {
    if (!seg_ok(sg)) return fail(LORA_ERR_INVALID_ARG, "seg is NULL or not a segment object");
    if (!sg->uploaded || !sg->dev) return LORA_OK;
    std::vector<unsigned> flags(4 + 2 * 256, 0u);
    HIP_TRY(hipMemcpyAsync(flags.data(), sg->dev + sg->off_sync + (size_t)2 * sg->n_sync * sizeof(unsigned),
                           flags.size() * sizeof(unsigned), hipMemcpyDeviceToHost, (hipStream_t)stream));
    HIP_TRY(hipStreamSynchronize((hipStream_t)stream));
    unsigned flag = flags[0];
    // the last one-launch apply's own record of which places ran on which XCD (earlier ones were looked
    // at by the launch that followed them)
    if (sg->decode_fused && sg->launches > 0) {
        unsigned seen[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        for (int b = 0; b < sg->fused_grid && b < 256; ++b) {
            const unsigned left = flags[4 + 256 * (sg->launches & 1u) + b];
            if ((left >> 8) != (sg->launches & 0xFFFFFFu)) continue;  // the last apply took two launches
            if (left & 0x80u) flag |= 2u;
            seen[(left >> 4) & 7u] |= 1u << (left & 7u);
        }
        for (unsigned q = 0; q < 8; ++q)
            if (seen[q] & (seen[q] - 1u)) {
                flag |= 2u;
                flags[2] = (q << 8) | seen[q];
            }
    }
    if (flag & 2u)
        return fail(LORA_ERR_DEVICE, "in a one-launch lora_apply, work groups of different places mod 8 ran on one XCD (XCD %u, "
                                     "differences seen: bits 0x%x): that apply's y is not valid "
                                     "(lora_set_decode_single_launch(0) selects two launches)", flags[2] >> 8, flags[2] & 255u);
    if (flag) return fail(LORA_ERR_DEVICE, "an expand unit of a one-launch lora_apply gave up waiting for its shrink units");
    return LORA_OK;
}
API_CATCH

extern "C" lora_status_t lora_profile_next_apply(void *before, void *between, void *after)
try {
    g_prof[0] = (hipEvent_t)before;
    g_prof[1] = (hipEvent_t)between;
    g_prof[2] = (hipEvent_t)after;
    return LORA_OK;
}
API_CATCH

// The launches of one apply: `arena` is the base the units' weight offsets count from, `out` the
// width of y that the units' columns lie in.
// may_create: the apply may make the segment object's side stream and events at its first use.
static lora_status_t run_apply(const uint16_t *arena, int in, int out, const lora_segments *sg, const void *x,
                               int64_t ldx, void *y, int64_t ldy, void *workspace, size_t ws_bytes, void *stream,
                               bool may_create = true)
{
    lora_status_t st;
    if ((st = check_matrix(x, ldx, in, "x")) != LORA_OK) return st;
    if ((st = check_matrix(y, ldy, out, "y")) != LORA_OK) return st;
    const size_t need = apply_parts_bytes(sg) + 2 * apply_packed_bytes(sg);
    if ((st = check_workspace(workspace, ws_bytes, need)) != LORA_OK) return st;
    hipStream_t s = (hipStream_t)stream;
    float *parts = (float *)workspace;
    const int nsl = std::max(1, sg->n_k_slices);
    const int64_t stride = nsl > 1 ? sg->v_floats : 0;
    hipEvent_t ev[3] = {g_prof[0], g_prof[1], g_prof[2]};
    g_prof[0] = g_prof[1] = g_prof[2] = nullptr;
    // The arrival counters live in the segment object's device table (and the single-launch form's
    // epoch in the object), so applies that share an object must be issued by one thread at a time and
    // ordered on one stream.
    lora_segments *msg = const_cast<lora_segments *>(sg);
    lora::SyncArgs sa;
    sa.counters = (unsigned *)(sg->dev + sg->off_sync);
    sa.ready = sa.counters + sg->n_sync;
    sa.timeout_flag = sa.counters + 2 * sg->n_sync;
    sa.v_hi = (uint16_t *)((char *)workspace + apply_parts_bytes(sg));
    sa.v_lo = (uint16_t *)((char *)workspace + apply_parts_bytes(sg) + apply_packed_bytes(sg));
    sa.epoch = msg->launches + 1;  // read by the single-launch form only, which also advances it
    sa.spin_limit = opt_spin_limit(sg);
    const lora::LaunchCtx cs = ctx_for(arena, in, out, sg, kShrink), cp = ctx_for(arena, in, out, sg, kPrefill),
                          ce = ctx_for(arena, in, out, sg, kExpand), cb = ctx_for(arena, in, out, sg, kExpandBig);
    if (ev[0]) HIP_TRY(hipEventRecord(ev[0], s));
    // units of more than 16 tokens span several counters, and whole-k shrink units are work groups of
    // another size: such batches always take separate launches
    // The one-launch decode form takes its epoch from the host at launch, which a replayed graph would
    // repeat: under stream capture the batch takes the two launches, which give the same bits.
    // Nor on a device where the probe launch did not find work group b on the XCD of b mod 8.
    hipStreamCaptureStatus capturing = hipStreamCaptureStatusNone;
    const DeviceProfile *prof = nullptr;
    if (opt_decode_single(sg) && sg->decode_fused) {
        HIP_TRY(hipStreamIsCapturing(s, &capturing));
        int dev = -1;
        HIP_TRY(hipGetDevice(&dev));
        if (dev >= 0 && dev < lora::kMaxDevices && g_profile[dev].state.load(std::memory_order_acquire) == 1)
            prof = &g_profile[dev];
    }
    if (prof && capturing == hipStreamCaptureStatusNone) {
        ++msg->launches;
        HIP_TRY(lora::launch_decode_fused(ctx_for(arena, in, out, sg, kFusedShrink), ctx_for(arena, in, out, sg, kFusedExpand),
                                          sg->fused_grid, (const uint16_t *)x, ldx, sg->wide_slice_len, sg->wide_slices,
                                          (uint16_t *)y, ldy, prof->xcc_map.load(std::memory_order_relaxed), &sa, s));
        if (ev[1]) HIP_TRY(hipEventRecord(ev[1], s));
    } else if (opt_fused_apply(sg) && !sg->has_big_units && !sg->wide) {
        ++msg->launches;
        HIP_TRY(lora::launch_apply_fused(cs, ce, (const uint16_t *)x, ldx, sg->k_slice_len, parts, nsl, stride,
                                         (uint16_t *)y, ldy, &sa, s));
        if (ev[1]) HIP_TRY(hipEventRecord(ev[1], s));
    } else {
        // A mixed batch: the decode-sized groups' two launches are short, latency-bound and touch
        // other tokens (rows of v and y) than the token-heavy groups' two, so they go to a stream of
        // the segment object's own and run beside them; the caller's stream waits for them at the end.
        if (opt_merged(sg) && sg->has_big_units && !sg->wide && cs.n_units > 0) {
            HIP_TRY(lora::launch_shrink_mixed(cp, sg->n_prefill_hi, cs, (const uint16_t *)x, ldx, sg->k_slice_len, parts,
                                              nsl, stride, &sa, s));
            if (ev[1]) HIP_TRY(hipEventRecord(ev[1], s));
            HIP_TRY(lora::launch_expand_mixed(cb, ce, parts, nsl, stride, (uint16_t *)y, ldy, &sa, s));
            if (ev[2]) HIP_TRY(hipEventRecord(ev[2], s));
            return LORA_OK;
        }
        hipStream_t sd = s;
        // not when a token-heavy group's v is read by 16-token expand units (groups above kBigExpandMaxRank):
        // those would sit on the side stream, which does not wait for the token-heavy shrink launch
        const bool split = opt_side_stream(sg) && sg->has_big_units && !sg->heavy_small_expand &&
                           cs.n_units >= kSideStreamMinUnits && (may_create || (sg->side && sg->fork && sg->join));
        if (split) {
            if (!msg->side) HIP_TRY(hipStreamCreateWithFlags(&msg->side, hipStreamNonBlocking));
            // the two events order launches of this device among themselves and nothing reads them on
            // the host: created without the system-scope fence an event otherwise carries (whole layer
            // of the mixed batch 865 -> 803 us)
            const unsigned ev_flags = hipEventDisableTiming | hipEventDisableSystemFence;
            if (!msg->fork) HIP_TRY(hipEventCreateWithFlags(&msg->fork, ev_flags));
            if (!msg->join) HIP_TRY(hipEventCreateWithFlags(&msg->join, ev_flags));
            sd = msg->side;
            HIP_TRY(hipEventRecord(msg->fork, s));
            HIP_TRY(hipStreamWaitEvent(sd, msg->fork, 0));
        }
        HIP_TRY(lora::launch_shrink_prefill(cp, sg->n_prefill_hi, (const uint16_t *)x, ldx, sa.v_hi, sa.v_lo, nullptr,
                                            nsl, stride, parts, &sa, s));
        if (sg->wide)
            HIP_TRY(lora::launch_shrink_wide(cs, cs.n_units > g_compute_units, (const uint16_t *)x, ldx, sg->wide_slice_len, sg->wide_slices, nullptr,
                                             sa.v_hi, sa.v_lo, sd));
        else
            HIP_TRY(lora::launch_shrink(cs, (const uint16_t *)x, ldx, sg->k_slice_len, parts, nsl, stride, &sa, sd));
        if (ev[1]) HIP_TRY(hipEventRecord(ev[1], s));
        HIP_TRY(lora::launch_expand(ce, false, parts, nsl, stride, (uint16_t *)y, ldy, &sa, sd));
        HIP_TRY(lora::launch_expand(cb, true, parts, nsl, stride, (uint16_t *)y, ldy, &sa, s));
        if (split) {
            HIP_TRY(hipEventRecord(msg->join, sd));
            HIP_TRY(hipStreamWaitEvent(s, msg->join, 0));
        }
    }
    if (ev[2]) HIP_TRY(hipEventRecord(ev[2], s));
    return LORA_OK;
}

extern "C" lora_status_t lora_apply(const lora_pool_t *pool, const lora_segments_t *sg, const void *x, int64_t ldx,
                                    void *y, int64_t ldy, void *workspace, size_t ws_bytes, void *stream)
try {
    lora_status_t st = check_launchable(pool, sg);
    if (st != LORA_OK) return st;
    if (sg->n_active == 0) return LORA_OK;
    return run_apply(pool->arena, pool->in_features, pool->out_features, sg, x, ldx, y, ldy, workspace, ws_bytes,
                     stream);
}
API_CATCH

// ---- the adapted layer as one pass over y: base GEMM with the delta in its epilogue ----
extern "C" lora_status_t lora_linear_pack_weight(const void *wt_out_by_in, int32_t in_features, int32_t out_features,
                                                 void *dev_packed, void *stream)
try {
    if (!wt_out_by_in || !dev_packed) return fail(LORA_ERR_INVALID_ARG, "wt_out_by_in or dev_packed is NULL");
    if (((uintptr_t)dev_packed) % 256) return fail(LORA_ERR_INVALID_ARG, "dev_packed is not 256-byte aligned");
    if (in_features <= 0 || out_features <= 0 || in_features % 64 || out_features % 128)
        return fail(LORA_ERR_SHAPE, "in_features (%d) must be a positive multiple of 64 and out_features (%d) of 128",
                    in_features, out_features);
    HIP_TRY(lora::launch_pack_weight((const uint16_t *)wt_out_by_in, in_features, out_features, (uint16_t *)dev_packed,
                                     (hipStream_t)stream));
    return LORA_OK;
}
API_CATCH

extern "C" lora_status_t lora_linear(const lora_pool_t *pool, const lora_segments_t *sg, const void *x, int64_t ldx,
                                     const void *w_packed, void *y, int64_t ldy, void *workspace, size_t ws_bytes,
                                     void *stream)
try {
    lora_status_t st = check_launchable(pool, sg);
    if (st != LORA_OK) return st;
    if (sg->T == 0) return LORA_OK;
    if (!w_packed || ((uintptr_t)w_packed) % 16) return fail(LORA_ERR_INVALID_ARG, "w_packed is NULL or not 16-byte aligned");
    const int in = pool->in_features, out = pool->out_features;
    if ((st = check_matrix(x, ldx, in, "x")) != LORA_OK) return st;
    if ((st = check_matrix(y, ldy, out, "y")) != LORA_OK) return st;
    const size_t need = apply_parts_bytes(sg) + 2 * apply_packed_bytes(sg);
    if (sg->n_active > 0 && (st = check_workspace(workspace, ws_bytes, need)) != LORA_OK) return st;
    hipStream_t s = (hipStream_t)stream;
    float *parts = (float *)workspace;
    const int nsl = std::max(1, sg->n_k_slices);
    const int64_t stride = nsl > 1 ? sg->v_floats : 0;
    lora::SyncArgs sa;
    sa.counters = (unsigned *)(sg->dev + sg->off_sync);
    sa.ready = sa.counters + sg->n_sync;
    sa.timeout_flag = sa.counters + 2 * sg->n_sync;
    sa.v_hi = (uint16_t *)((char *)workspace + apply_parts_bytes(sg));
    sa.v_lo = (uint16_t *)((char *)workspace + apply_parts_bytes(sg) + apply_packed_bytes(sg));
    sa.epoch = 0;
    sa.spin_limit = opt_spin_limit(sg);
    if (sg->n_active > 0) {
        // the shrink half of lora_apply's separate-launch forms: v complete as bf16 hi + lo in the workspace
        const lora::LaunchCtx cs = ctx_for(pool, sg, kShrink), cp = ctx_for(pool, sg, kPrefill);
        if (opt_merged(sg) && sg->has_big_units && !sg->wide && cs.n_units > 0) {
            HIP_TRY(lora::launch_shrink_mixed(cp, sg->n_prefill_hi, cs, (const uint16_t *)x, ldx, sg->k_slice_len, parts, nsl,
                                              stride, &sa, s));
        } else {
            HIP_TRY(lora::launch_shrink_prefill(cp, sg->n_prefill_hi, (const uint16_t *)x, ldx, sa.v_hi, sa.v_lo, nullptr, nsl,
                                                stride, parts, &sa, s));
            if (sg->wide)
                HIP_TRY(lora::launch_shrink_wide(cs, cs.n_units > g_compute_units, (const uint16_t *)x, ldx, sg->wide_slice_len, sg->wide_slices, nullptr,
                                                 sa.v_hi, sa.v_lo, s));
            else
                HIP_TRY(lora::launch_shrink(cs, (const uint16_t *)x, ldx, sg->k_slice_len, parts, nsl, stride, &sa, s));
        }
    }
    HIP_TRY(lora::launch_linear_lora((const int32_t *)(sg->dev + sg->off_lin_rows),
                                     (const LinBlock *)(sg->dev + sg->off_lin_blocks), (int)sg->lin_rows.size(), pool->arena,
                                     (const uint16_t *)w_packed, (const uint16_t *)x, ldx, in, out, sa.v_hi, sa.v_lo,
                                     (uint16_t *)y, ldy, s));
    return LORA_OK;
}
API_CATCH

// lora_apply with the library's own workspace: nothing is allocated here, neither device memory nor a
// stream or an event (a mixed batch planned for four launches keeps them on `stream` unless the
// object's side stream already exists).
extern "C" lora_status_t lora_apply_static(const lora_pool_t *pool, const lora_segments_t *sg, const void *x,
                                           int64_t ldx, void *y, int64_t ldy, void *stream)
try {
    lora_status_t st = check_launchable(pool, sg);
    if (st != LORA_OK) return st;
    if (sg->n_active == 0) return LORA_OK;
    const size_t need = apply_parts_bytes(sg) + 2 * apply_packed_bytes(sg);
    if (need > lora::kStaticScratchBytes)
        return fail(LORA_ERR_WORKSPACE,
                    "this batch needs a workspace of %zu bytes, the library's own holds LORA_STATIC_WORKSPACE_BYTES = "
                    "%zu: use lora_apply with a workspace of the caller's",
                    need, (size_t)lora::kStaticScratchBytes);
    void *ws = nullptr;
    HIP_TRY(lora::static_scratch(&ws));
    return run_apply(pool->arena, pool->in_features, pool->out_features, sg, x, ldx, y, ldy, ws,
                     lora::kStaticScratchBytes, stream, false);
}
API_CATCH

extern "C" lora_status_t lora_apply_multi(const lora_pool_t *const *pools, int32_t n_pools,
                                          const lora_segments_t *sg, const void *x, int64_t ldx, void *y,
                                          int64_t ldy, void *workspace, size_t ws_bytes, void *stream)
try {
    std::vector<const lora_pool *> list;
    lora_status_t st = check_pool_list(pools, n_pools, &list);
    if (st != LORA_OK) return st;
    if (!seg_ok(sg)) return fail(LORA_ERR_INVALID_ARG, "seg is NULL or not a segment object");
    if (sg->mpools.size() != list.size())
        return fail(LORA_ERR_INVALID_ARG, "segment object was built for %zu pools, %zu given", sg->mpools.size(),
                    list.size());
    const uint16_t *base = list[0]->arena;
    for (const lora_pool *q : list) base = std::min(base, (const uint16_t *)q->arena);
    for (size_t q = 0; q < list.size(); ++q) {
        if (list[q]->out_features != sg->mouts[q])
            return fail(LORA_ERR_STALE_SEGMENTS, "pools[%zu] has another out_features than the pool planned for", q);
        if ((uint64_t)(((uintptr_t)list[q]->arena - (uintptr_t)base) / 2) != sg->mdelta[q])
            return fail(LORA_ERR_STALE_SEGMENTS,
                        "the arenas of the given pools are not spaced as those the object was planned for");
        if ((st = check_adapters(list[q], sg, sg->msegs[q], sg->mepochs[q], sg->mpool_ids[q])) != LORA_OK) return st;
    }
    if (!sg->uploaded) return fail(LORA_ERR_INVALID_ARG, "segment object was planned but not uploaded");
    if (sg->n_active == 0) return LORA_OK;
    return run_apply(base, list[0]->in_features, sg->out_total, sg, x, ldx, y, ldy, workspace, ws_bytes, stream);
}
API_CATCH

extern "C" const char *lora_status_string(lora_status_t status)
{
    switch (status) {
    case LORA_OK: return "LORA_OK";
    case LORA_ERR_INVALID_ARG: return "LORA_ERR_INVALID_ARG";
    case LORA_ERR_SHAPE: return "LORA_ERR_SHAPE";
    case LORA_ERR_OOM: return "LORA_ERR_OOM";
    case LORA_ERR_NOT_RESIDENT: return "LORA_ERR_NOT_RESIDENT";
    case LORA_ERR_STALE_SEGMENTS: return "LORA_ERR_STALE_SEGMENTS";
    case LORA_ERR_WORKSPACE: return "LORA_ERR_WORKSPACE";
    case LORA_ERR_DEVICE: return "LORA_ERR_DEVICE";
    }
    return "LORA_ERR_UNKNOWN";
}

extern "C" const char *lora_last_error(void) { return g_err; }
