/*
 * liblora_gfx950 -- co-batched heterogeneous-rank LoRA delta for one MI355X (gfx950).
 *
 *     v[t, :] = x[t, :] * A_a          (shrink,  A_a is in x r_a)
 *     y[t, :] += s_a * v[t, :] * B_a   (expand,  B_a is r_a x out)
 *
 * for every token t of a batch, where a = token_adapter[t] may differ from token to token and the
 * ranks r_a of the adapters that share the batch differ too.  This is the operation behind the
 * paper's problem statement: LoRA adds a pair of low-rank matrices to a frozen layer, the rank
 * being the adapter's size (Background, "Low-Rank Adaptation"); serving systems run requests of
 * different adapters and ranks in one batched kernel (Background, "Kernel Optimizations"); and
 * kernels that size their tiles to the largest rank in the batch make low-rank requests pay for
 * the high-rank ones (Motivation, "Effect of Co-serving Adapters of Different Ranks").  Here every
 * unit of work is sized by the bytes of its own adapter, never by the largest rank present.
 *
 * Conventions
 *   - bf16 storage (x, y, adapter weights), fp32 accumulation, one round-to-nearest-even to bf16
 *     when y is written.  lora_shrink returns v as fp32.  Between the two halves of lora_apply, and
 *     when lora_expand takes the caller's fp32 v, v enters the expand MFMAs as two bf16 terms hi + lo
 *     (hi = nearest bf16 of v, lo = nearest bf16 of v - hi): 16 significant bits, relative error at
 *     most 2^-16 per element, far inside the one rounding of y to bf16 (2^-8).
 *   - "device" pointers are HIP device memory of the current device; "host" pointers are ordinary
 *     host memory.  The caller owns every device buffer it passes in (arena, x, y, v, workspace).
 *     The library owns its opaque host objects.  Two conveniences allocate on the caller's behalf:
 *     lora_segments_upload (the object's device table and its pinned host copy) and lora_pool_load
 *     from a host source (a device staging buffer for the duration of the call); callers that want
 *     every byte of device memory to be their own use lora_segments_upload_to and
 *     lora_pool_load_staged instead, which allocate nothing.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Kernel launches and
 *     copies are asynchronous on it unless a function says otherwise.
 *   - Every function validates its arguments on the host before touching the device and returns a
 *     status; nothing throws, aborts or exits.  lora_last_error() gives a thread-local detail line
 *     for the last non-OK status returned on this thread.
 *   - in_features must be a multiple of 64 and out_features of 128; ranks are 1..LORA_MAX_RANK.
 *   - Threads: the objects are not locked.  Calls that touch one pool, or a segment object and the
 *     pools it was planned for, must come from one thread at a time; unrelated objects may be used
 *     from different threads at once.  Plan settings are per segment object (lora_plan_options_t);
 *     the lora_set_* calls set the process-wide defaults that fields left at "default" fall back to
 *     (atomic variables: a setter may run beside planning threads, which see the old or the new value).  A failed host allocation comes back as LORA_ERR_OOM like any other
 *     status (no C++ exception leaves the library).
 */
#ifndef LORA_GFX950_H
#define LORA_GFX950_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LORA_MAX_RANK 256
#define LORA_MAX_PROJECTIONS 8 /* pools per multi-projection segment object */
#define LORA_BF16 1

typedef enum {
    LORA_OK = 0,
    LORA_ERR_INVALID_ARG = 1,    /* NULL pointer, negative count, id out of range, bad flag        */
    LORA_ERR_SHAPE = 2,          /* feature size or rank outside what the kernels support         */
    LORA_ERR_OOM = 3,            /* arena / host / device allocation too small or failed          */
    LORA_ERR_NOT_RESIDENT = 4,   /* a token is routed to an adapter that is not loaded            */
    LORA_ERR_STALE_SEGMENTS = 5, /* an adapter the segment object uses was reloaded, moved or differs */
    LORA_ERR_WORKSPACE = 6,      /* workspace missing, misaligned or smaller than required        */
    LORA_ERR_DEVICE = 7          /* a HIP call failed (no device, launch error, copy error)       */
} lora_status_t;

typedef struct lora_pool lora_pool_t;         /* opaque: ragged adapter pool of one projection */
typedef struct lora_segments lora_segments_t; /* opaque: one batch's token grouping + work units */

/* Adapters of one projection (one weight matrix of one layer).  `ranks` and `scales` are host
 * arrays of n_adapters entries, copied by lora_pool_create. */
typedef struct {
    int32_t in_features;
    int32_t out_features;
    int32_t n_adapters;
    const int32_t *ranks;
    const float *scales;
    int32_t dtype; /* LORA_BF16 */
} lora_pool_desc_t;

/* Where one adapter lives inside the arena (element = one bf16): A^T (rank_padded x in_features) at
 * a_offset, B^T (out_features x rank_padded) at b_offset, rank_padded = rank rounded up to a multiple of
 * 8, padding rows / columns zero.  An adapter costs 2*rank_padded*(in+out) bytes whatever the other
 * adapters' ranks are.  Inside a matrix the elements are in the order in which a 16x16x32 bf16 MFMA
 * reads its weight operand (lane l: 8 consecutive values of the contracted index, chunk l>>4, of row
 * l&15), so that one wavefront load of an operand is 1 KB of consecutive bytes:
 *   A^T element (row j, k):   block jb = j/16 of h rows (h = 16, or 8 for the last block when
 *        rank_padded mod 16 == 8), n = j mod 16, step s = k/32, kq = (k mod 32)/8, e = k mod 8:
 *        a_offset + 16*jb*in + s*32*h + (kq*h + n)*8 + e
 *   B^T element (column c, j): strip = c/128, within it c' = c mod 128, b = c' mod 8, n = c'/8,
 *        kp = j/8, e = j mod 8:
 *        b_offset + 128*strip*rank_padded + ((b*(rank_padded/8) + kp)*16 + n)*8 + e
 * Callers never build this form themselves: lora_pool_load takes row-major A and B. */
typedef struct {
    uint64_t a_offset;
    uint64_t b_offset;
    int32_t rank;
    int32_t rank_padded;
    float scale;
    int32_t resident;
} lora_adapter_info_t;

/* Sizes of a built segment object. */
typedef struct {
    int32_t n_tokens;        /* T as passed in                                          */
    int32_t n_active;        /* tokens with an adapter (token_adapter >= 0)             */
    int32_t n_segments;      /* distinct adapters used by the batch                     */
    int32_t n_shrink_units;  /* work groups of the shrink launch                        */
    int32_t n_expand_units;  /* work groups of the expand launch                        */
    int32_t n_k_slices;      /* split-K partial sums per v element (1 = none)           */
    int64_t v_floats;        /* length of v in floats: sum over active tokens of rank_padded */
    int64_t weight_bytes;    /* packed bytes of the distinct adapters the batch touches */
    int32_t single_launch;   /* 1: planned for the one-launch decode form (see lora_set_decode_single_launch) */
    int32_t launch_work_groups; /* work groups of that launch (a multiple of 8, at most 256), else 0 */
} lora_segments_info_t;

/* ---- pool: the ragged, rank-packed adapter arena (set-up time, not on the per-step path) ---- */

/* Bytes of device memory the arena needs for this description.  Host only. */
lora_status_t lora_pool_bytes(const lora_pool_desc_t *desc, size_t *arena_bytes);

/* Lay the adapters of `desc` out in `dev_arena` (device memory, 256-byte aligned, at least
 * lora_pool_bytes() long, owned by the caller and alive as long as the pool).  Host only: it
 * records offsets; no adapter is resident until lora_pool_load.  LORA_ERR_SHAPE for unsupported
 * feature sizes or ranks, LORA_ERR_OOM if arena_bytes is too small. */
lora_status_t lora_pool_create(const lora_pool_desc_t *desc, void *dev_arena, size_t arena_bytes,
                               lora_pool_t **out);

/* A live pool: the same object over an arena of any size (256-byte aligned), smaller than the sum of
 * the adapters if wanted.  No adapter has a place until it is loaded (or reserved); lora_pool_load
 * takes the first free piece that is large enough (adapters occupy 2*rank_padded*(in+out) bytes
 * rounded up to 256), lora_pool_evict gives the piece back, lora_pool_compact closes the gaps.  This
 * is one GPU's share of the adapter store that the paper keeps across servers (System Design,
 * "Distributed Adapter Pool"): which adapters are present changes while batches run.  Host only. */
lora_status_t lora_pool_create_live(const lora_pool_desc_t *desc, void *dev_arena, size_t arena_bytes,
                                    lora_pool_t **out);

/* Copy adapter `adapter` into the pool and mark it resident.  A is [in][rank] and B is [rank][out],
 * row-major bf16, in host memory (src_is_device = 0) or device memory (1).  The packed, transposed
 * form is written by a device kernel on `stream`.  With a host source the call allocates a device
 * staging buffer and returns after the copy has completed; with a device source it is asynchronous
 * and the source must stay valid until the stream reaches it.  In a live pool the adapter is given a
 * place first: LORA_ERR_OOM if no free piece is large enough (the message says whether compaction
 * would help).  The adapter gets a new stamp: segment objects that use it become stale, others stay
 * valid, so adapters can be loaded on a copy stream while batches that do not use them run on
 * another; the caller orders the load before the first launch that uses the adapter (an event). */
lora_status_t lora_pool_load(lora_pool_t *pool, int32_t adapter, const void *A_in_by_r,
                             const void *B_r_by_out, int src_is_device, void *stream);

/* Mark an adapter non-resident.  Fixed pool: its bytes stay where they are.  Live pool: its piece
 * returns to the free list, so the caller makes sure no launch that reads it is still running.
 * Segment objects that use the adapter are refused from now on (LORA_ERR_NOT_RESIDENT). */
/* lora_pool_load from host memory without any allocation or wait of the library's: A and B are copied
 * into dev_staging (device memory of the caller, 16-byte aligned, at least
 * lora_pool_load_staging_bytes(pool, adapter) long) and packed from there, all asynchronous on
 * `stream`.  A, B (pinned host memory if the copies are to overlap anything) and dev_staging must stay
 * valid and untouched until the stream has passed the call. */
lora_status_t lora_pool_load_staging_bytes(const lora_pool_t *pool, int32_t adapter, size_t *bytes);
lora_status_t lora_pool_load_staged(lora_pool_t *pool, int32_t adapter, const void *A_in_by_r, const void *B_r_by_out,
                                    void *dev_staging, size_t staging_bytes, void *stream);

lora_status_t lora_pool_evict(lora_pool_t *pool, int32_t adapter);

/* Live pool: give the adapter a place without copying anything (no-op in a fixed pool, or if it has
 * one).  Host only.  LORA_ERR_OOM as for lora_pool_load. */
lora_status_t lora_pool_reserve(lora_pool_t *pool, int32_t adapter);

/* Declare an adapter resident without copying: for callers that wrote its packed form into the
 * arena themselves (a device-to-device copy of another pool's arena, a restored snapshot).  Host
 * only.  In a live pool the adapter must have a place (lora_pool_reserve).  New stamp as for load. */
lora_status_t lora_pool_mark_resident(lora_pool_t *pool, int32_t adapter);

/* Live pool: free bytes in total and in the largest single piece (0, 0 for a fixed pool).  Host only. */
lora_status_t lora_pool_space(const lora_pool_t *pool, size_t *free_bytes, size_t *largest_free_bytes);

/* Live pool: slide every placed adapter towards the start of the arena, in address order, with
 * device-to-device copies on `stream` (asynchronous), leaving one free piece at the end.  A move that
 * overlaps its own source goes through dev_scratch (device memory, may be NULL) when scratch_bytes
 * covers the adapter, else in pieces no longer than the gap.  Moved adapters get a new stamp (segment
 * objects that use them become stale); *n_moved (may be NULL) counts them.  The caller makes sure no
 * launch that reads a moved adapter is still running on another stream. */
lora_status_t lora_pool_compact(lora_pool_t *pool, void *dev_scratch, size_t scratch_bytes, void *stream,
                                int32_t *n_moved);

/* Host only: layout and residency of one adapter. */
lora_status_t lora_pool_adapter_info(const lora_pool_t *pool, int32_t adapter, lora_adapter_info_t *info);

lora_status_t lora_pool_destroy(lora_pool_t *pool);

/* ---- segments: per-batch grouping of tokens by adapter and the byte-balanced work-unit lists ---- */

/* Plan settings of one segment object, given to the *_opts calls (NULL = all defaults) and kept by the
 * object: they govern its planning (also every later lora_segments_rebuild) and how lora_apply
 * launches it.  A switch left at -1 (fused_wait_limit: 0) takes the process-wide default, the value of
 * the lora_set_* call of the same name, read at the time of use.  The meaning of each setting is
 * described at that call, further down. */
typedef struct {
    int32_t whole_k_limit;        /* -1 or as lora_set_whole_k_limit                  */
    int32_t merged_launches;      /* -1, 0, 1: lora_set_merged_launches              */
    int32_t side_stream;          /* -1, 0, 1: lora_set_side_stream                  */
    int32_t fused_apply;          /* -1, 0, 1: lora_set_fused_apply                  */
    int32_t decode_single_launch; /* -1, 0, 1: lora_set_decode_single_launch         */
    uint32_t fused_wait_limit;    /* 0 or polls: lora_set_fused_wait_limit           */
    /* The planner's size thresholds, each found by a sweep on one MI355X (the measured points are listed
     * beside the built-in values in the host source); -1 = built in.  They exist so that a caller, or a
     * bench, can measure a plan on either side of a threshold; results do not depend on them beyond the
     * order of fp32 sums. */
    int32_t whole_k_max_in;        /* largest in_features planned without k-slices (built in: 18432)      */
    int32_t heavy_min_tokens;      /* a group of at least this many tokens is token-heavy (32) ...        */
    int32_t heavy_min_batch;       /* ... in a batch of at least this many active tokens (1024)           */
    int32_t heavy_k_cut_max_units; /* token-heavy shrink units are cut along k while the cut units stay    *
                                    * within this count (320; 750 beyond in_features 8192)                 */
    int32_t big_runs_max_units;    /* 64-token expand units take their columns in 8 runs, not 4, while     *
                                    * the launch stays within this many of them (two per compute unit: 512) */
} lora_plan_options_t;
#define LORA_PLAN_OPTIONS_DEFAULT {-1, -1, -1, -1, -1, 0u, -1, -1, -1, -1, -1}

/* Host-only half of lora_segments_build: group the T tokens by adapter (stable: tokens of one
 * adapter keep their order), and cut every group into work units whose cost follows that adapter's
 * own bytes.  token_adapter_host[t] in [0, n_adapters) or -1 for "no adapter" (row left untouched).
 * LORA_ERR_INVALID_ARG for ids out of range, LORA_ERR_NOT_RESIDENT for an id that is not loaded.
 * T = 0 and batches without any active token are valid.  The result cannot be launched until
 * lora_segments_upload has run. */
lora_status_t lora_segments_plan(const lora_pool_t *pool, const int32_t *token_adapter_host, int32_t T,
                                 lora_segments_t **out);

lora_status_t lora_segments_plan_opts(const lora_pool_t *pool, const int32_t *token_adapter_host, int32_t T,
                                      const lora_plan_options_t *options, lora_segments_t **out);

/* Replaces the object's settings (NULL: all defaults); takes effect at the next rebuild and apply. */
lora_status_t lora_segments_set_options(lora_segments_t *seg, const lora_plan_options_t *options);

/* Same, from contiguous ranges: tokens seg_start_host[i] .. seg_start_host[i+1]-1 use adapter
 * seg_adapter_host[i] (or none if it is -1); seg_start_host has S+1 non-decreasing entries starting
 * at 0 and T = seg_start_host[S].  Ranges that name the same adapter are merged into one group. */
lora_status_t lora_segments_plan_ranges(const lora_pool_t *pool, const int32_t *seg_start_host,
                                        const int32_t *seg_adapter_host, int32_t S, lora_segments_t **out);

/* Allocate the segment object's device table (library-owned, freed by lora_segments_destroy) and
 * enqueue one host-to-device copy of it on `stream`. */
lora_status_t lora_segments_upload(lora_segments_t *seg, void *stream);

/* The same with memory of the caller's: the table goes into dev_table (device memory, 256-byte aligned)
 * through host_staging (host memory, pinned if the copy is to be asynchronous, 16-byte aligned), each
 * at least lora_segments_table_bytes(seg) long (known after planning).  The object uses both from now
 * on, for lora_segments_rebuild too (LORA_ERR_OOM, with the sizes, if a later batch needs more), and
 * never frees them; the caller keeps them alive as long as the object and leaves them alone while
 * launches that use the object may run.  No allocation is made. */
lora_status_t lora_segments_table_bytes(const lora_segments_t *seg, size_t *bytes);
lora_status_t lora_segments_upload_to(lora_segments_t *seg, void *dev_table, size_t dev_bytes, void *host_staging,
                                      size_t staging_bytes, void *stream);

/* plan + upload. */
lora_status_t lora_segments_build(const lora_pool_t *pool, const int32_t *token_adapter_host, int32_t T,
                                  void *stream, lora_segments_t **out);
lora_status_t lora_segments_build_opts(const lora_pool_t *pool, const int32_t *token_adapter_host, int32_t T,
                                       const lora_plan_options_t *options, void *stream, lora_segments_t **out);
lora_status_t lora_segments_build_ranges(const lora_pool_t *pool, const int32_t *seg_start_host,
                                         const int32_t *seg_adapter_host, int32_t S, void *stream,
                                         lora_segments_t **out);

/* Re-plan an existing object for a new batch of the same pool and upload it, re-using its host and
 * device storage when it is large enough (the per-step call of a decode loop).  The previous
 * table must no longer be in use by work enqueued on another stream. */
lora_status_t lora_segments_rebuild(lora_segments_t *seg, const int32_t *token_adapter_host, int32_t T,
                                    void *stream);
/* (A segment object remembers its pool by handle and id and looks both up among the live pools before
 * it touches the pool: after lora_pool_destroy, rebuild returns LORA_ERR_STALE_SEGMENTS, and any call
 * given a destroyed pool handle returns LORA_ERR_INVALID_ARG; no freed memory is read.) */

lora_status_t lora_segments_info(const lora_segments_t *seg, lora_segments_info_t *info);

/* Host copies of the grouping, for callers that want to read v and for tests.  Any output may be
 * NULL.  perm[n_active]: token index at each sorted position; seg_start[n_segments+1]: sorted
 * positions where each group starts; seg_adapter[n_segments]; v_offset[T]: float offset of token
 * t's row inside v (rank_padded floats long), -1 for tokens without adapter. */
lora_status_t lora_segments_export(const lora_segments_t *seg, int32_t *perm, int32_t *seg_start,
                                   int32_t *seg_adapter, int64_t *v_offset);

/* Host copies of the work-unit lists, 6 int32 per unit: {segment, first token (relative to the
 * group), token count, first row (shrink) or first column (expand), row or column count,
 * k-slice (shrink) or 0}.  Groups of fewer than 32 tokens are cut into shrink units of <= 16 tokens x
 * 16 rank rows x one k-slice (in a whole-k plan of at most 256 units, the units of the most tokens
 * come as two units of 8 rank rows each, as many token counts as fit 256 units); token-heavy groups
 * into shrink units of up to 32 tokens (64 for ranks 65..192) x all rank
 * rows x all of k (listed after the others, k-slice 0; in a batch planned in k-slices with few such
 * units, two or four k-slices each) and into expand units of up to 64 tokens.
 * The order is the launch order: the decode shrink units of one group take places of one residue
 * mod 8 where the counts allow it (the launch's work groups go to the chip's 8 XCDs in turn, and the
 * group's rows of x then stay in one XCD's L2); the token-heavy shrink units of one adapter likewise
 * (its A^T then enters one L2), the eight lists filled to equal bytes and the shorter ones padded at
 * their end with places that hold no work: segment -1, token count 0; the 64-token expand units (listed after the others)
 * of one group (its columns in 4 runs, 8 in a launch of few such units) come in rows of 8, each
 * column run with 8 / (column runs) consecutive token tiles, so that a column run's part of B^T is
 * fetched by that many XCDs instead of all 8.  Either output may be NULL. */
lora_status_t lora_segments_export_units(const lora_segments_t *seg, int32_t *shrink_units,
                                         int32_t *expand_units);

/* Host copies of the one-launch decode form's lists (info.single_launch == 1), by place in the launch:
 * shrink_units holds launch_work_groups records, expand_units four times as many (work group b runs
 * shrink unit b, then expand units 4b .. 4b+3), 7 int32 each: the six of lora_segments_export_units
 * and the index of the (group, token tile) whose v the unit writes or reads.  Empty places have a
 * token count of 0.  Either output may be NULL. */
lora_status_t lora_segments_export_launch_units(const lora_segments_t *seg, int32_t *shrink_units,
                                                int32_t *expand_units);

lora_status_t lora_segments_destroy(lora_segments_t *seg);

/* ---- the hot path ---- */

/* Bytes of device workspace lora_shrink / lora_apply need for this batch (split-K partial sums of
 * v; 0 is possible).  The workspace must be 256-byte aligned. */
lora_status_t lora_workspace_bytes(const lora_pool_t *pool, const lora_segments_t *seg, size_t *bytes);

/* A segment object can be launched on the pool it was built for, and on any other pool with the same
 * feature sizes that holds every adapter the batch uses, resident, with the same rank and scale at the
 * same place in its arena (pools created from the same description: the layers of a model share one
 * token->adapter map, so one object serves all layers of one projection shape).  On its own pool it
 * is refused with LORA_ERR_STALE_SEGMENTS once an adapter it uses has been loaded again or moved, and
 * with LORA_ERR_NOT_RESIDENT once one has been evicted; changes to other adapters do not touch it. */

/* Shrink: v[t, j] = sum_k x[t, k] * A_a(t)[k, j] for every active token.
 * x: device, bf16, [T][in] with row stride ldx elements (ldx >= in, ldx % 8 == 0, 16-byte aligned).
 * v: device, fp32, info.v_floats long, 16-byte aligned; token t's row starts at v_offset[t] and is
 *    rank_padded long (entries beyond the rank are written as 0).
 * LORA_ERR_STALE_SEGMENTS / LORA_ERR_NOT_RESIDENT as described above, LORA_ERR_WORKSPACE if the
 * workspace is too small. */
lora_status_t lora_shrink(const lora_pool_t *pool, const lora_segments_t *seg, const void *x, int64_t ldx,
                          float *v, void *workspace, size_t ws_bytes, void *stream);

/* Expand: y[t, o] = bf16(y[t, o] + s_a(t) * sum_j v[t, j] * B_a(t)[j, o]) for every active token,
 * in place.  y: device, bf16, [T][out] with row stride ldy (ldy >= out, ldy % 8 == 0, 16-byte
 * aligned).  Rows of tokens without adapter are neither read nor written. */
lora_status_t lora_expand(const lora_pool_t *pool, const lora_segments_t *seg, const float *v, void *y,
                          int64_t ldy, void *stream);

/* Shrink then expand on one stream.  x, y, the workspace and the pool's arena must not overlap one
 * another (the launches read x and the arena while they write the workspace and y; nothing checks
 * this).  v never leaves the workspace, whose size
 * lora_apply_workspace_bytes gives (the k-slices' partial sums of v; the expand adds them up, in
 * slice order, while it loads them). */
lora_status_t lora_apply_workspace_bytes(const lora_pool_t *pool, const lora_segments_t *seg, size_t *bytes);
lora_status_t lora_apply(const lora_pool_t *pool, const lora_segments_t *seg, const void *x, int64_t ldx,
                         void *y, int64_t ldy, void *workspace, size_t ws_bytes, void *stream);

/* The adapted layer in one pass over y: y[t, :] = bf16(x[t, :] W + s_a v[t, :] B_a) for EVERY token of the
 * batch (tokens without adapter get x W alone): the base projection with the delta in its epilogue, the
 * frozen layer plus the low-rank pair of Background, "Low-Rank Adaptation", computed together as a
 * serving system does for each adapted projection (Motivation, Fig. 3).  y is written once and never
 * read, where lora_apply reads and re-writes what a separate base GEMM wrote.  Launches: the shrink of
 * lora_apply (v into the workspace), then one GEMM kernel over 256 x 128 tiles of y whose rows follow
 * the segment object's grouping (x is gathered and y scattered through it; no copy of either).
 *   w_packed: the base weight in the kernel's operand order, made once by lora_linear_pack_weight from
 *             W^T [out][in] row-major bf16 (the layout of a linear layer's weight), in_features *
 *             out_features * 2 bytes of device memory, 256-byte aligned, owned by the caller;
 *   x, y, workspace, stream: as for lora_apply (workspace size: lora_apply_workspace_bytes); y need not be
 *             initialised.  Single-pool segment objects only.
 * fp32 accumulation of x W and of the delta (each in one accumulator, the delta scaled once), one
 * rounding to bf16. */
lora_status_t lora_linear_pack_weight(const void *wt_out_by_in, int32_t in_features, int32_t out_features,
                                      void *dev_packed, void *stream);
lora_status_t lora_linear(const lora_pool_t *pool, const lora_segments_t *seg, const void *x, int64_t ldx,
                          const void *w_packed, void *y, int64_t ldy, void *workspace, size_t ws_bytes, void *stream);

/* For callers that cannot allocate device memory: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  lora_apply with a workspace of the library's own, a file-scope
 * device array of LORA_STATIC_WORKSPACE_BYTES that every GPU the library runs on holds until the
 * process ends (its address is looked up once per device, at the first call there).  The call makes
 * no device allocation, no stream and no event; x, y, the pool's arena and the segment object's table
 * are still the caller's / the object's, made beforehand.  LORA_ERR_WORKSPACE, with both sizes in the
 * message, if lora_apply_workspace_bytes(pool, seg) exceeds LORA_STATIC_WORKSPACE_BYTES (cfg1's 256
 * decode tokens need 0.1 MB, 9.5 k mixed tokens 9.5 MB).  Same launches and bitwise the same y as
 * lora_apply.  Nothing in the workspace has to start at zero (every element read by a launch was
 * written earlier in the same apply).  All such calls on one GPU share the one array: calls whose
 * launches may overlap there (different streams, different threads) race; order them on one stream.
 * A mixed batch planned for four launches keeps them on `stream` unless an earlier lora_apply on the
 * object has already made its side stream. */
#define LORA_STATIC_WORKSPACE_BYTES ((size_t)32 << 20)
lora_status_t lora_apply_static(const lora_pool_t *pool, const lora_segments_t *seg, const void *x, int64_t ldx,
                                void *y, int64_t ldy, void *stream);

/* Several projections that read the same x (q, k and v of a layer; gate and up) in one pass: their
 * pools (same in_features, same ranks and scales, each with its own out_features and arena) are
 * planned together and every launch of lora_apply_multi covers all of them, so x is fetched once per
 * launch rather than once per projection and the fixed cost of a launch is paid once.  y is one
 * matrix [T][out_0 + out_1 + ...], row stride ldy: projection q's columns follow those of q - 1, the
 * layout of a fused q|k|v or gate|up output.  Each row gets bitwise what separate lora_apply calls on
 * the column blocks would give it.  lora_segments_plan_multi is host only; build = plan + upload;
 * lora_segments_rebuild, info, export, check and destroy work on such objects, the single-pool
 * launch calls refuse them.  The object can be launched on other pools (the next layer's) with the
 * same adapters at the same places whose arenas lie at the same distances from each other
 * (LORA_ERR_STALE_SEGMENTS otherwise).  Workspace: lora_apply_workspace_bytes(pools[0], seg). */
lora_status_t lora_segments_plan_multi(const lora_pool_t *const *pools, int32_t n_pools,
                                       const int32_t *token_adapter_host, int32_t T, lora_segments_t **out);
lora_status_t lora_segments_build_multi(const lora_pool_t *const *pools, int32_t n_pools,
                                        const int32_t *token_adapter_host, int32_t T, void *stream,
                                        lora_segments_t **out);
lora_status_t lora_segments_plan_multi_opts(const lora_pool_t *const *pools, int32_t n_pools,
                                            const int32_t *token_adapter_host, int32_t T,
                                            const lora_plan_options_t *options, lora_segments_t **out);
lora_status_t lora_segments_build_multi_opts(const lora_pool_t *const *pools, int32_t n_pools,
                                             const int32_t *token_adapter_host, int32_t T,
                                             const lora_plan_options_t *options, void *stream,
                                             lora_segments_t **out);
lora_status_t lora_apply_multi(const lora_pool_t *const *pools, int32_t n_pools, const lora_segments_t *seg,
                               const void *x, int64_t ldx, void *y, int64_t ldy, void *workspace,
                               size_t ws_bytes, void *stream);

/* Planning knob: the process-wide default of lora_plan_options_t.whole_k_limit, read by the
 * lora_segments_plan / build / rebuild calls that follow for objects that leave the field at -1.
 * A batch whose decode-sized groups make between 64 and `max_units` shrink units when a unit takes
 * the whole of k (16 rank rows x up to 16 tokens each) is planned that way, if in_features is at most
 * 18432 and the batch is not a mixed one run as merged launches (below): work groups of 16
 * wavefronts, v complete when the unit ends.  Other batches cut k into up to 4 slices per unit (more,
 * smaller units spread a small batch over the chip and fill the last round of a large one better) and
 * add the slices up through counters.  Both plans give bitwise the same v for these groups
 * (token-heavy groups, whose units a k-slice plan may also cut along k, get another grouping of
 * their sums).  Default 1024 (four rounds of one work group per compute unit); 0 = always k-slices. */
lora_status_t lora_set_whole_k_limit(int32_t max_units);

/* lora_apply is two launches by default (shrink units, then expand units).  With k-slices the shrink
 * unit that completes a token tile (found through per-tile counters in the segment object's device
 * table) adds the k-slices up and leaves the tile's v for the expand units.
 * lora_set_fused_apply(1) selects, for batches planned with k-slices and without token-heavy groups,
 * a single launch in which shrink and expand units share the grid and the expand units poll, with a
 * bounded number of polls, until their tile's v is complete.  Applies that share one segment object
 * share its counters, so they must be issued by one thread at a time and ordered on one stream.
 * In the forms of separate shrink and expand launches every counter is back at zero when the launch
 * that used it ends, so such an apply may be captured into a graph and replayed (the form of a mixed
 * batch that uses the object's own stream makes that stream and its two events at the object's
 * first such apply, which has to come before the capture).  A captured apply holds the launch sizes
 * and the table address of the plan it was captured with: after lora_segments_rebuild on the
 * object, capture again.  The single-launch form takes an epoch from
 * host state of the segment object at launch: it must not be captured, and not be used on an object
 * that a captured graph replays.  The setting is process-wide. */
lora_status_t lora_set_fused_apply(int enabled);

/* A mixed batch holds token-heavy groups and decode-sized groups, whose units are of different kinds.
 * By default (lora_set_merged_launches(1)) such a batch is planned with the decode-sized groups in
 * k-slices, whose work groups have the size of the token-heavy ones', and lora_apply /
 * lora_apply_multi run it as two launches on `stream`: one shrink launch and one expand launch that
 * each hold both kinds of unit, the token-heavy ones first.  The setting is read when a batch is
 * planned (build / rebuild) and again when it is applied; a batch planned under one setting and
 * applied under the other still gives the same y, through the four launches below.  Process-wide.
 *
 * With lora_set_merged_launches(0) a mixed batch is four launches: the token-heavy groups' shrink
 * and expand, the decode-sized groups' shrink and expand.  The two pairs touch different tokens
 * (other rows of v and y), and the decode-sized pair is short and bound by latency, so with
 * lora_set_side_stream(1) (the default) it is issued onto a stream that belongs to the segment object
 * (created at the first such apply, default priority, non-blocking), between an event recorded on
 * `stream` at the start of the apply and one that `stream` waits for at its end: the pairs run side
 * by side and everything later on `stream` is ordered behind both.  lora_set_side_stream(0) keeps all
 * four launches on `stream`.  y is bitwise the same in all three forms, except where the merged
 * form's plan also cuts the token-heavy shrink units along k (launches of few such units: at most
 * 160 of them, 375 beyond 8192 input features; the sums of v are then grouped differently, within
 * the same tolerance).
 * Process-wide. */
lora_status_t lora_set_merged_launches(int enabled);

/* A decode-sized batch on the whole-k plan (no token-heavy groups, one pool) whose units fit one round of
 * the chip (at most 256 shrink units, 1024 expand units) is planned for, and run as, ONE launch of at
 * most one work group per compute unit: work group b does one shrink unit and then four expand
 * units, and the expand units' loads of B^T follow the shrink units' loads of A^T without the tail,
 * the pause and the ramp of a launch boundary.  v goes from the shrink units to the expand units of a
 * (group, token tile) through the L2 of one XCD: the planner puts all of a tile's units at places of
 * one residue mod 8, which the hardware's dispatch order (work group b to the XCD of b mod 8) turns
 * into one XCD.  The library checks that order with one probe launch per device (at the first
 * lora_segments_upload there; on a device where it does not hold, batches keep their two launches)
 * and every work group of the launch checks its own XCD: a mismatch, like a wait that ran out, is
 * reported by lora_segments_check.  y is bitwise what the two launches give.
 * The launch takes an epoch from host state of the segment object, so under stream capture lora_apply
 * issues the two launches instead (same bits), and applies that share an object must be ordered on
 * one stream, as ever.  Two such launches that run at the same time on one GPU (different objects on
 * different streams) can hold each other's compute units while they wait: their waits are bounded and
 * reported, but callers that overlap applies should select two launches.
 * lora_set_decode_single_launch(0): always two launches.  Read when a batch is planned and again when it
 * is applied.  Process-wide; default 1. */
lora_status_t lora_set_decode_single_launch(int enabled);
lora_status_t lora_set_side_stream(int enabled);

/* Polls an expand unit of the single-launch apply makes before it gives up waiting, flags the object
 * and goes on with whatever v holds (default 2^18; 0 restores the default).  Process-wide.  A small
 * value makes the give-up path reachable on a healthy machine, which is what it is for: every
 * wavefront still ends, lora_segments_check then reports the apply as failed. */
lora_status_t lora_set_fused_wait_limit(uint32_t polls);

/* Synchronises `stream` and reports LORA_ERR_DEVICE if an expand unit of an earlier fused lora_apply
 * on this object ran into its (bounded) wait limit, in which case that apply's y is not valid.  The
 * flag stays until the object's table is uploaded again (lora_segments_rebuild / _upload). */
lora_status_t lora_segments_check(const lora_segments_t *seg, void *stream);

/* Measurement hook.  The next lora_apply on the calling thread records the given hipEvent_t handles
 * (passed as void*, any may be NULL) on its stream: `before` ahead of the shrink launch, `between`
 * after it, `after` behind the expand launch (a fused apply records `between` and `after` together,
 * behind its single launch; in a mixed batch with the side stream on, `between` follows the token-heavy
 * groups' shrink launch and `after` the join of both streams).  The hook clears itself after that call. */
lora_status_t lora_profile_next_apply(void *before, void *between, void *after);

const char *lora_status_string(lora_status_t status);
const char *lora_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* LORA_GFX950_H */
