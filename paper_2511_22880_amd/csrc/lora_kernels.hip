// gfx950 kernels of the co-batched LoRA delta (shrink: v = x A_a, expand: y += s_a v B_a).
//
// Both adapter matrices are stored with the contracted index contiguous (A^T [r8][in],
// B^T [out][r8]), so a 16x16x32 bf16 MFMA can take its weight operand straight from 16-byte global
// loads: lane l supplies row (l & 15) of a 16-row weight tile and the 8 consecutive k values
// 8*(l >> 4) .. +7 of a 32-wide k step.  The token operand uses the same lane->k mapping, so the
// order of k inside a step is irrelevant to the result.  The 16x16 fp32 result tile has
// D[4*(l >> 4) + i][l & 15] in register i of lane l: weight row down, token across.
//
// Work is cut on the host into units of roughly equal adapter bytes; one work group (4 wavefronts)
// takes one unit.  No unit ever depends on another adapter's rank.
#include "lora_internal.h"

namespace lora {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

static __device__ __forceinline__ bf16x8 as_bf16x8(uint4 u) { return __builtin_bit_cast(bf16x8, u); }

static __device__ __forceinline__ uint4 ld16(const uint16_t *p) { return *reinterpret_cast<const uint4 *>(p); }

static __device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

// ------------------------------------------------------------------------------------------------
// shrink: one unit = (group, <=16 tokens, 16 rank rows, one k-slice).  The four wavefronts split the
// k-slice, each accumulates a 16x16 tile, the tiles are summed through LDS in wavefront order.
// ------------------------------------------------------------------------------------------------
constexpr int kShrinkUnroll = 8;

__global__ __launch_bounds__(kThreads) void k_shrink(const Unit *__restrict__ units,
                                                     const uint16_t *__restrict__ arena,
                                                     const uint16_t *__restrict__ x, int64_t ldx, int in,
                                                     int k_slice_len, float *__restrict__ v_out,
                                                     int64_t slice_stride)
{
    __shared__ f32x4 red[4][64];
    const Unit &u = units[blockIdx.x];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int i = lane & 15;
    const int kq = lane >> 4;

    const int token = u.tok[i];
    const int ntok = u.ntok, pn = u.pn, ks = u.ks;
    const bool w_ok = i < pn;
    const bool x_ok = i < ntok;
    const uint16_t *wrow = arena + u.w_off + (int64_t)(w_ok ? i : 0) * in;
    const uint16_t *xrow = x + (int64_t)token * ldx;

    const int kw = k_slice_len >> 2;
    const int kbeg = ks * k_slice_len + wave * kw;
    int kend = kbeg + kw;
    if (kend > in) kend = in;

    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    const uint4 zero = {0u, 0u, 0u, 0u};
    for (int k0 = kbeg; k0 < kend; k0 += 32 * kShrinkUnroll) {
        uint4 a[kShrinkUnroll], b[kShrinkUnroll];
#pragma unroll
        for (int q = 0; q < kShrinkUnroll; ++q) {
            const int k = k0 + 32 * q;
            if (k < kend) {
                a[q] = ld16(wrow + k + 8 * kq);
#ifndef EXP_NO_X
                b[q] = ld16(xrow + k + 8 * kq);
#else
                b[q] = make_uint4(kq, k, 3u, 4u);
#endif
            } else {
                a[q] = zero;
                b[q] = zero;
            }
        }
#pragma unroll
        for (int q = 0; q < kShrinkUnroll; ++q) {
            const uint4 aa = w_ok ? a[q] : zero;
            const uint4 bb = x_ok ? b[q] : zero;
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(aa), as_bf16x8(bb), acc, 0, 0, 0);
        }
    }
#ifdef EXP_NO_RED
    if (acc[0] == 1.2345f) v_out[blockIdx.x] = acc[1];
    return;
#endif
    red[wave][lane] = acc;
    __syncthreads();
    if (wave == 0) {
        f32x4 t = red[0][lane];
        t += red[1][lane];
        t += red[2][lane];
        t += red[3][lane];
        if (x_ok && 4 * kq < pn) {
            float *dst = v_out + (int64_t)ks * slice_stride + u.v_off + (int64_t)i * u.r8 + 4 * kq;
            *reinterpret_cast<f32x4 *>(dst) = t;
        }
    }
}

// ------------------------------------------------------------------------------------------------
// expand: one unit = (group, <=16 tokens, a run of output columns).  Each wavefront keeps the
// tokens' v rows in registers as two bf16 terms (hi + lo, so v keeps ~16 mantissa bits), walks
// 16-column tiles of B^T and updates y in place.
// ------------------------------------------------------------------------------------------------
static __device__ __forceinline__ uint32_t pack_bf16_rne(float a, float b)
{
    typedef __attribute__((ext_vector_type(2))) float f32x2;
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
    const f32x2 f = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));
}

constexpr int kMaxSlices = 4;               // upper bound of the shrink's k-slices
constexpr int kVRow = LORA_MAX_RANK_PADDED + 8;  // LDS row length of the staged v (bf16), padded against bank conflicts

template <int KSTEPS, int TILES>
static __device__ __forceinline__ void expand_body(const Unit &u, const uint16_t *__restrict__ arena,
                                                   const float *__restrict__ v_in, int n_slices,
                                                   int64_t slice_stride, uint16_t *__restrict__ y,
                                                   int64_t ldy, uint16_t (*__restrict__ s_hi)[kVRow],
                                                   uint16_t (*__restrict__ s_lo)[kVRow])
{
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int i = lane & 15;
    const int kq = lane >> 4;
    const int r8 = u.r8;
    const int ntok = u.ntok;
    const bool t_ok = i < ntok;
    const uint4 zero = {0u, 0u, 0u, 0u};
    const int token = u.tok[i];
    uint16_t *yrow = y + (int64_t)token * ldy + u.p0 + 4 * kq;
    const uint16_t *bbase = arena + u.w_off + (int64_t)i * r8;
    const float scale = u.scale;
    const int ncols = u.pn;

    int jc[KSTEPS];
    bool j_ok[KSTEPS];
#pragma unroll
    for (int st = 0; st < KSTEPS; ++st) {
        const int j = 32 * st + 8 * kq;
        j_ok[st] = j < r8;
        jc[st] = j_ok[st] ? j : 0;
    }

    // first batch of weight tiles goes out before anything waits on v
    uint4 w[TILES][KSTEPS];
    uint2 yv[TILES];
    auto load_batch = [&](int c0) {
#pragma unroll
        for (int tl = 0; tl < TILES; ++tl) {
            const int c = c0 + 64 * tl;
            if (c < ncols) {
                const uint16_t *brow = bbase + (int64_t)c * r8;
#pragma unroll
                for (int st = 0; st < KSTEPS; ++st) w[tl][st] = ld16(brow + jc[st]);
#ifndef EXP_NO_YLOAD
                yv[tl] = t_ok ? *reinterpret_cast<const uint2 *>(yrow + c) : make_uint2(0u, 0u);
#else
                yv[tl] = make_uint2(0u, 0u);
#endif
            } else {
#pragma unroll
                for (int st = 0; st < KSTEPS; ++st) w[tl][st] = zero;
                yv[tl] = make_uint2(0u, 0u);
            }
        }
    };
    load_batch(16 * wave);

    // stage v once per work group: every thread sums the k-slices of some 8-float pieces (all slice
    // loads in flight together, added in slice order) and leaves them in LDS as bf16 hi + lo
    const int groups = r8 >> 3;  // 8-float pieces per token row
#ifdef EXP_NO_V
    for (int task = threadIdx.x; task < 0; task += kThreads) {
#else
    for (int task = threadIdx.x; task < ntok * groups; task += kThreads) {
#endif
        const int t = task / groups, g = task - t * groups;
        const float *src = v_in + u.v_off + (int64_t)t * r8 + 8 * g;
        f32x4 p0[kMaxSlices], p1[kMaxSlices];
#pragma unroll
        for (int sl = 0; sl < kMaxSlices; ++sl) {
            const int64_t off = (int64_t)(sl < n_slices ? sl : 0) * slice_stride;
            p0[sl] = *reinterpret_cast<const f32x4 *>(src + off);
            p1[sl] = *reinterpret_cast<const f32x4 *>(src + off + 4);
        }
        f32x4 f0 = p0[0], f1 = p1[0];
#pragma unroll
        for (int sl = 1; sl < kMaxSlices; ++sl)
            if (sl < n_slices) {
                f0 += p0[sl];
                f1 += p1[sl];
            }
        uint4 ph, pl;
        ph.x = pack_bf16_rne(f0[0], f0[1]);
        ph.y = pack_bf16_rne(f0[2], f0[3]);
        ph.z = pack_bf16_rne(f1[0], f1[1]);
        ph.w = pack_bf16_rne(f1[2], f1[3]);
        pl.x = pack_bf16_rne(f0[0] - bf16_bits_to_f32(ph.x & 0xFFFFu), f0[1] - __uint_as_float(ph.x & 0xFFFF0000u));
        pl.y = pack_bf16_rne(f0[2] - bf16_bits_to_f32(ph.y & 0xFFFFu), f0[3] - __uint_as_float(ph.y & 0xFFFF0000u));
        pl.z = pack_bf16_rne(f1[0] - bf16_bits_to_f32(ph.z & 0xFFFFu), f1[1] - __uint_as_float(ph.z & 0xFFFF0000u));
        pl.w = pack_bf16_rne(f1[2] - bf16_bits_to_f32(ph.w & 0xFFFFu), f1[3] - __uint_as_float(ph.w & 0xFFFF0000u));
        *reinterpret_cast<uint4 *>(&s_hi[t][8 * g]) = ph;
        *reinterpret_cast<uint4 *>(&s_lo[t][8 * g]) = pl;
    }
    __syncthreads();

    bf16x8 vhi[KSTEPS], vlo[KSTEPS];
#pragma unroll
    for (int st = 0; st < KSTEPS; ++st) {
        uint4 ph = zero, pl = zero;
        if (t_ok && j_ok[st]) {
            ph = *reinterpret_cast<const uint4 *>(&s_hi[i][32 * st + 8 * kq]);
            pl = *reinterpret_cast<const uint4 *>(&s_lo[i][32 * st + 8 * kq]);
        }
        vhi[st] = as_bf16x8(ph);
        vlo[st] = as_bf16x8(pl);
    }

    for (int c0 = 16 * wave; c0 < ncols; c0 += 64 * TILES) {
        f32x4 acc[TILES];
#pragma unroll
        for (int tl = 0; tl < TILES; ++tl) {
            acc[tl] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int st = 0; st < KSTEPS; ++st) {
                const bf16x8 ww = as_bf16x8(j_ok[st] ? w[tl][st] : zero);
                acc[tl] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ww, vhi[st], acc[tl], 0, 0, 0);
                acc[tl] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ww, vlo[st], acc[tl], 0, 0, 0);
            }
        }
        uint2 o[TILES];
#pragma unroll
        for (int tl = 0; tl < TILES; ++tl) {
            const float y0 = bf16_bits_to_f32(yv[tl].x & 0xFFFFu) + scale * acc[tl][0];
            const float y1 = __uint_as_float(yv[tl].x & 0xFFFF0000u) + scale * acc[tl][1];
            const float y2 = bf16_bits_to_f32(yv[tl].y & 0xFFFFu) + scale * acc[tl][2];
            const float y3 = __uint_as_float(yv[tl].y & 0xFFFF0000u) + scale * acc[tl][3];
            o[tl].x = pack_bf16_rne(y0, y1);
            o[tl].y = pack_bf16_rne(y2, y3);
        }
        const int cnext = c0 + 64 * TILES;
#pragma unroll
        for (int tl = 0; tl < TILES; ++tl) {
            const int c = c0 + 64 * tl;
#ifndef EXP_NO_YSTORE
            if (t_ok && c < ncols) *reinterpret_cast<uint2 *>(yrow + c) = o[tl];
#else
            if (t_ok && c < ncols && o[tl].x == 0x12345678u) *reinterpret_cast<uint2 *>(yrow + c) = o[tl];
#endif
        }
        if (cnext < ncols) load_batch(cnext);
    }
}

__global__ __launch_bounds__(kThreads) void k_expand(const Unit *__restrict__ units,
                                                     const uint16_t *__restrict__ arena,
                                                     const float *__restrict__ v_in, int n_slices,
                                                     int64_t slice_stride, uint16_t *__restrict__ y,
                                                     int64_t ldy)
{
    __shared__ __attribute__((aligned(16))) uint16_t s_hi[kTokTile][kVRow];
    __shared__ __attribute__((aligned(16))) uint16_t s_lo[kTokTile][kVRow];
    const Unit &u = units[blockIdx.x];
    const int r8 = u.r8;
    if (r8 <= 32)
        expand_body<1, 8>(u, arena, v_in, n_slices, slice_stride, y, ldy, s_hi, s_lo);
    else if (r8 <= 64)
        expand_body<2, 4>(u, arena, v_in, n_slices, slice_stride, y, ldy, s_hi, s_lo);
    else if (r8 <= 128)
        expand_body<4, 2>(u, arena, v_in, n_slices, slice_stride, y, ldy, s_hi, s_lo);
    else
        expand_body<8, 1>(u, arena, v_in, n_slices, slice_stride, y, ldy, s_hi, s_lo);
}

__global__ __launch_bounds__(256) void k_reduce_slices(const float *__restrict__ parts, int n_slices,
                                                       int64_t slice_stride, float *__restrict__ v, int64_t n)
{
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= n) return;
    float acc = parts[idx];
    for (int sl = 1; sl < n_slices; ++sl) acc += parts[idx + (int64_t)sl * slice_stride];
    v[idx] = acc;
}

__global__ __launch_bounds__(256) void k_pack_transpose(const uint16_t *__restrict__ src, int src_rows,
                                                        int src_cols, uint16_t *__restrict__ dst, int P, int Q)
{
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (int64_t)P * Q) return;
    const int p = (int)(idx / Q);
    const int q = (int)(idx % Q);
    uint16_t val = 0;
    if (q < src_rows && p < src_cols) val = src[(int64_t)q * src_cols + p];
    dst[idx] = val;
}

// ------------------------------------------------------------------------------------------------
// launchers
// ------------------------------------------------------------------------------------------------
hipError_t launch_shrink(const LaunchCtx &c, const uint16_t *x, int64_t ldx, int k_slice_len, float *v_out,
                         int64_t slice_stride, hipStream_t stream)
{
    if (c.n_units <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_shrink, dim3(c.n_units), dim3(kThreads), 0, stream, c.units, c.arena, x, ldx,
                       c.in_features, k_slice_len, v_out, slice_stride);
    return hipGetLastError();
}

hipError_t launch_expand(const LaunchCtx &c, const float *v_in, int n_slices, int64_t slice_stride, uint16_t *y,
                         int64_t ldy, hipStream_t stream)
{
    if (c.n_units <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_expand, dim3(c.n_units), dim3(kThreads), 0, stream, c.units, c.arena, v_in, n_slices,
                       slice_stride, y, ldy);
    return hipGetLastError();
}

hipError_t launch_reduce_slices(const float *parts, int n_slices, int64_t slice_stride, float *v, int64_t n,
                                hipStream_t stream)
{
    if (n <= 0) return hipSuccess;
    const int64_t blocks = (n + 255) / 256;
    hipLaunchKernelGGL(k_reduce_slices, dim3((unsigned)blocks), dim3(256), 0, stream, parts, n_slices,
                       slice_stride, v, n);
    return hipGetLastError();
}

hipError_t launch_pack_transpose(const uint16_t *src, int src_rows, int src_cols, uint16_t *dst, int P, int Q,
                                 hipStream_t stream)
{
    const int64_t n = (int64_t)P * Q;
    if (n <= 0) return hipSuccess;
    const int64_t blocks = (n + 255) / 256;
    hipLaunchKernelGGL(k_pack_transpose, dim3((unsigned)blocks), dim3(256), 0, stream, src, src_rows, src_cols,
                       dst, P, Q);
    return hipGetLastError();
}

}  // namespace lora
