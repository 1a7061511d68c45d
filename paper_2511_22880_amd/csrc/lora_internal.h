// Records shared by the host planner and the gfx950 kernels, and the launch entry points the host
// side calls.  Not part of the public boundary (that is include/lora.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lora {

// One group of tokens that share an adapter.  64 bytes, read with scalar loads.
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

// One work group's share.  32 bytes.
struct Unit {
    int32_t seg;
    int32_t tok0;  // first token, relative to the group
    int32_t ntok;  // tokens in this unit
    int32_t p0;    // shrink: first rank row; expand: first output column
    int32_t pn;    // shrink: rank rows;      expand: output columns
    int32_t ks;    // shrink: k-slice index
    int32_t pad[2];
};
static_assert(sizeof(Unit) == 32, "Unit is 32 bytes");

constexpr int kTokTile = 16;   // tokens per MFMA tile (the N of a 16x16x32 MFMA)
constexpr int kRowTile = 16;   // rank rows / output columns per MFMA tile (the M)
constexpr int kThreads = 256;  // 4 wavefronts per work group

struct LaunchCtx {
    const Unit *units;
    const SegRec *segs;
    const int32_t *perm;
    const uint16_t *arena;
    int n_units;
    int in_features;
    int out_features;
};

// v_out[ks * slice_stride + ...] receives k-slice ks's partial sums (slice_stride = 0 when there is
// a single slice and v_out is v itself).
hipError_t launch_shrink(const LaunchCtx &c, const uint16_t *x, int64_t ldx, int k_slice_len,
                         float *v_out, int64_t slice_stride, hipStream_t stream);

// v_in holds n_slices partial sums slice_stride floats apart (n_slices = 1: v itself).
hipError_t launch_expand(const LaunchCtx &c, const float *v_in, int n_slices, int64_t slice_stride,
                         uint16_t *y, int64_t ldy, hipStream_t stream);

// v[i] = sum over slices, in slice order.
hipError_t launch_reduce_slices(const float *parts, int n_slices, int64_t slice_stride, float *v,
                                int64_t n, hipStream_t stream);

// dst[p][q] = q_src_valid ? src[q * src_ld + p] : 0 for p < P, q < Q; used to write A^T (P = r8,
// Q = in, src = A [in][r], rows p >= r zero) and B^T (P = out, Q = r8, src = B [r][out], columns
// q >= r zero).
hipError_t launch_pack_transpose(const uint16_t *src, int src_rows, int src_cols, uint16_t *dst, int P,
                                 int Q, hipStream_t stream);

}  // namespace lora
