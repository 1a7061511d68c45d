// Records shared by the host planner and the gfx950 kernels, and the launch entry points the host
// side calls.  Not part of the public boundary (that is include/lora.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lora {

// One group of tokens that share an adapter (host-side planning record).
struct SegRec {
    uint64_t a_off;     // element offset of A^T [r8][in] in the arena
    uint64_t b_off;     // element offset of B^T [out][r8] in the arena
    int64_t v_off;      // float offset of the group's first v row
    int32_t rank;
    int32_t r8;         // rank rounded up to a multiple of 8 (row length of v and of B^T)
    float scale;
    int32_t tok_start;  // first sorted position of the group in perm
    int32_t ntok;
    int32_t pad[5];
};
static_assert(sizeof(SegRec) == 64, "SegRec is 64 bytes");

// One work group's share, self-contained so that a work group needs a single round trip to memory
// before it can issue its weight loads.  128 bytes: the first 64 are read with scalar loads, the
// token list with one vector load.
struct Unit {
    uint64_t w_off;   // element offset of the unit's first weight row (A^T row p0 / B^T row p0)
    int64_t v_off;    // float offset of the unit's first v element (shrink: row tok0, column p0;
                      // expand: row tok0, column 0)
    int32_t r8;       // padded rank = row length of v and of B^T
    int32_t ntok;     // tokens in this unit: 1..16 (decode units), up to 64 (expand, prefill shrink above rank 64) or 32 (prefill shrink)
    int32_t p0;       // shrink: first rank row; expand: first output column
    int32_t pn;       // shrink: valid rank rows (1..16, multiple of 8 except the tail); expand: columns
    int32_t ks;       // shrink: k-slice index
    float scale;
    int32_t seg;
    int32_t tok0;     // first token, relative to the group
    int32_t sync_idx; // counter of this unit's (group, token tile) in a fused launch
    int32_t sync_n;   // shrink units that feed that counter per launch
    int32_t perm_off; // position of the unit's first token in the device copy of perm
    int32_t pad[1];
    int32_t tok[16];  // batch row index of each token; entries >= ntok repeat tok[0] (units of <= 16
                      // tokens; larger units read perm[perm_off + i])
};
static_assert(sizeof(Unit) == 128, "Unit is 128 bytes");

// One block of 16 consecutive places of the adapted layer's row order (lora_linear): tokens grouped by
// adapter, every group padded to a multiple of 16 places, tokens without adapter last.
struct LinBlock {
    uint64_t b_off;  // element offset of the group's B^T in the arena
    int64_t v_off;   // element offset of the v row of the block's first token
    int32_t r8;      // padded rank; 0 = tokens without adapter (or an empty block)
    int32_t ntok;    // tokens in the block, 0..16
    float scale;
    int32_t pad;
};
static_assert(sizeof(LinBlock) == 32, "LinBlock is 32 bytes");
constexpr int kLinTileM = 256;  // rows of a work group's output tile (the row order is padded to a multiple)
constexpr int kLinTileN = 256;  // columns of it: two 128-column strips of B^T (the last tile of a row may hold one)

#define LORA_MAX_RANK_PADDED 256
constexpr int kTokTile = 16;   // tokens per MFMA tile (the N of a 16x16x32 MFMA)
constexpr int kRowTile = 16;   // rank rows / output columns per MFMA tile (the M)
constexpr int kThreads = 256;  // 4 wavefronts per work group

struct LaunchCtx {
    const Unit *units;
    const int32_t *perm;
    const uint16_t *arena;
    int n_units;
    int in_features;
    int out_features;
};

// Hand-over of v through the segment table's counters (see the kernels): arrivals and ready counters
// per (group, token tile), the complete v as bf16 hi + lo, the launch epoch and the poll limit.
struct SyncArgs {
    unsigned *counters;
    unsigned *ready;
    unsigned *timeout_flag;
    uint16_t *v_hi;
    uint16_t *v_lo;
    unsigned epoch;
    unsigned spin_limit;
};

// v_out[ks * slice_stride + ...] receives k-slice ks's partial sums (slice_stride = 0 when there is
// a single slice).  With `sync`, the unit that completes a token tile also writes the tile's summed v
// as bf16 hi + lo.
hipError_t launch_shrink(const LaunchCtx &c, const uint16_t *x, int64_t ldx, int k_slice_len, float *v_out,
                         int n_slices, int64_t slice_stride, const SyncArgs *sync, hipStream_t stream);

// Whole-k shrink units: work groups of 16 wavefronts, four per k-slice of k_slice_len (n_slices <= 4
// slices cover in_features); v written complete, either as fp32 into v_f32 or (v_hi != NULL) as bf16
// hi + lo, bitwise what the k-slice units of launch_shrink give.  more_than_one_round: the launch has more
// units than the chip has compute units; it then runs as work groups of 8 wavefronts, two per compute unit
// (same bits).
hipError_t launch_shrink_wide(const LaunchCtx &c, bool more_than_one_round, const uint16_t *x, int64_t ldx,
                              int k_slice_len, int n_slices, float *v_f32, uint16_t *v_hi, uint16_t *v_lo,
                              hipStream_t stream);

// Without `sync`: v_in holds n_slices fp32 partial sums slice_stride floats apart (n_slices = 1: v
// itself).  With `sync`: v comes from sync->v_hi / v_lo (written by a shrink launch of the same epoch).
// `big`: the list holds units of up to 64 tokens (token indices through perm).
hipError_t launch_expand(const LaunchCtx &c, bool big, const float *v_in, int n_slices, int64_t slice_stride,
                         uint16_t *y, int64_t ldy, const SyncArgs *sync, hipStream_t stream);

// Shrink of token-heavy groups: one unit = (group, up to 32 tokens, all rank rows, the whole of k).
// n_hi = how many of the units are above rank 64: with none, the launch takes the kernel that fits four
// work groups on a compute unit, otherwise the one for any rank (two per compute unit).
// Writes complete v: as bf16 hi + lo into v_hi / v_lo, or (v_f32 != NULL) as fp32 into v_f32 with the
// other n_slices - 1 slices of the same rows set to zero.  Units cut by k (sync_n = slices of the unit's
// tokens, ks = which) put their sums into slices of `parts` and complete v through `sync`'s counters
// (apply), or into slices of v_f32 for the caller to add up (stand-alone shrink, sync = NULL).
hipError_t launch_shrink_prefill(const LaunchCtx &c, int n_hi, const uint16_t *x, int64_t ldx, uint16_t *v_hi,
                                 uint16_t *v_lo, float *v_f32, int n_slices, int64_t slice_stride, float *parts,
                                 const SyncArgs *sync, hipStream_t stream);

// A mixed batch's shrink in one launch: the token-heavy units of `heavy` (n_hi of them above rank 64),
// then the k-slice units of `c`, which leave partial sums in `parts` and complete v through `sync` as
// launch_shrink does.  Likewise the expand: the 64-token units of `big`, then the units of `c`; both
// read v from sync->v_hi / v_lo.
hipError_t launch_shrink_mixed(const LaunchCtx &heavy, int n_hi, const LaunchCtx &c, const uint16_t *x, int64_t ldx,
                               int k_slice_len, float *parts, int n_slices, int64_t slice_stride,
                               const SyncArgs *sync, hipStream_t stream);
hipError_t launch_expand_mixed(const LaunchCtx &big, const LaunchCtx &c, const float *parts, int n_slices,
                               int64_t slice_stride, uint16_t *y, int64_t ldy, const SyncArgs *sync,
                               hipStream_t stream);

// Both halves in one launch (shrink units first); the expand units poll `ready` of their token tile,
// at most spin_limit times each.
hipError_t launch_apply_fused(const LaunchCtx &shrink, const LaunchCtx &expand, const uint16_t *x, int64_t ldx,
                              int k_slice_len, float *parts, int n_slices, int64_t slice_stride, uint16_t *y,
                              int64_t ldy, const SyncArgs *sync, hipStream_t stream);

// A decode-sized batch on the whole-k plan in one launch of `grid` work groups of 16 wavefronts (at most
// one per compute unit): work group b runs shrink.units[b], then its four groups of four wavefronts run
// expand.units[4b .. 4b+3]; places with ntok == 0 are empty.  All units of one (group, token tile) sit
// at places of one residue mod 8, i.e. on one XCD, through whose L2 v (sync->v_hi / v_lo) and the
// tile's `ready` counter are handed over; the counter grows by an expand unit's sync_n per launch and
// sync->epoch is the number of such launches since the table was uploaded, this one included.
// xcc_map: 4 bits per XCD number (0..7), its position in the order in which a launch's work groups are
// dealt to the XCDs, as a probe launch found it (probe_xcc).  sync->timeout_flag is followed by 3 words
// of detail and 2 x 256 words the launches' own check of that order uses (see the kernel).  Expand units must be a single
// column pass (pn <= 512 / 256 / 128 columns up to rank 32 / 64 / beyond).
hipError_t launch_decode_fused(const LaunchCtx &shrink, const LaunchCtx &expand, int grid, const uint16_t *x,
                               int64_t ldx, int k_slice_len, int n_slices, uint16_t *y, int64_t ldy,
                               unsigned xcc_map, const SyncArgs *sync, hipStream_t stream);

// host_out[b] = XCD number (0..15) that work group b of an n-work-group launch ran on (n <= 1024).
// Synchronises the stream.
hipError_t probe_xcc(unsigned *host_out, int n_work_groups, hipStream_t stream);

// The adapted layer in one pass over y: y[row] = bf16(x[row] W + s_a v[row] B_a), W in operand order
// (launch_pack_weight), v as bf16 hi + lo from a shrink launch, rows[m] = batch row of place m (-1: none),
// blocks[m / 16] the adapter of places 16 (m / 16) .. +15.  m_pad places, a multiple of kLinTileM.
hipError_t launch_linear_lora(const int32_t *rows, const LinBlock *blocks, int m_pad, const uint16_t *arena,
                              const uint16_t *w_packed, const uint16_t *x, int64_t ldx, int in, int out,
                              const uint16_t *v_hi, const uint16_t *v_lo, uint16_t *y, int64_t ldy,
                              hipStream_t stream);

// W^T [out][in] row-major bf16 (the layout of a linear layer's weight) -> operand order: for every
// 128-column strip and every 32-wide k step, eight 1 KB pieces (sub-block b = columns 8n + b), piece
// (kq, n) holding k = 32 step + 8 kq .. +7 of column 128 strip + 8 n + b.
hipError_t launch_pack_weight(const uint16_t *wt, int in, int out, uint16_t *dst, hipStream_t stream);

// v[i] = sum over slices, in slice order.
hipError_t launch_reduce_slices(const float *parts, int n_slices, int64_t slice_stride, float *v,
                                int64_t n, hipStream_t stream);

// Writes adapter (A [in][r], B [r][out], row-major bf16, device memory) in the pool's packed,
// MFMA-operand-major form: dst_a gets r8*in elements, dst_b out*r8.
hipError_t launch_pack_adapter(const uint16_t *A, const uint16_t *B, int in, int out, int r, int r8,
                               uint16_t *dst_a, uint16_t *dst_b, hipStream_t stream);

// The library's own workspace for callers that cannot allocate: a file-scope device array of
// kStaticScratchBytes in the kernels' source file.  Gives that array's address on the current device
// (looked up once per device, then kept); the host must use this address, never the array's name.
constexpr size_t kStaticScratchBytes = (size_t)32 << 20;
constexpr int kMaxDevices = 64;
hipError_t static_scratch(void **ptr);

}  // namespace lora
