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

// round-to-nearest-even fp32 -> bf16 bits (finite inputs)
static __device__ __forceinline__ uint32_t f32_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// ------------------------------------------------------------------------------------------------
// shrink: one unit = (group, <=16 tokens, 16 rank rows, one k-slice).  The four wavefronts split the
// k-slice, each accumulates a 16x16 tile, the tiles are summed through LDS in wavefront order.
// ------------------------------------------------------------------------------------------------
constexpr int kShrinkUnroll = 8;

__global__ __launch_bounds__(kThreads) void k_shrink(const Unit *__restrict__ units,
                                                     const SegRec *__restrict__ segs,
                                                     const int32_t *__restrict__ perm,
                                                     const uint16_t *__restrict__ arena,
                                                     const uint16_t *__restrict__ x, int64_t ldx, int in,
                                                     int k_slice_len, float *__restrict__ v_out,
                                                     int64_t slice_stride)
{
    __shared__ f32x4 red[4][64];
    const Unit u = units[blockIdx.x];
    const SegRec s = segs[u.seg];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int i = lane & 15;
    const int kq = lane >> 4;

    const bool w_ok = (u.p0 + i) < s.r8;
    const bool x_ok = i < u.ntok;
    const uint16_t *wrow = arena + s.a_off + (int64_t)(w_ok ? u.p0 + i : u.p0) * in;
    const int token = perm[s.tok_start + u.tok0 + (x_ok ? i : 0)];
    const uint16_t *xrow = x + (int64_t)token * ldx;

    const int kw = k_slice_len >> 2;
    const int kbeg = u.ks * k_slice_len + wave * kw;
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
                b[q] = ld16(xrow + k + 8 * kq);
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
    red[wave][lane] = acc;
    __syncthreads();
    if (wave == 0) {
        f32x4 t = red[0][lane];
        t += red[1][lane];
        t += red[2][lane];
        t += red[3][lane];
        const int row = u.p0 + 4 * kq;
        if (x_ok && row < s.r8) {
            float *dst = v_out + (int64_t)u.ks * slice_stride + s.v_off + (int64_t)(u.tok0 + i) * s.r8 + row;
            *reinterpret_cast<f32x4 *>(dst) = t;
        }
    }
}

// ------------------------------------------------------------------------------------------------
// expand: one unit = (group, <=16 tokens, a run of output columns).  Each wavefront keeps the
// tokens' v rows in registers as two bf16 terms (hi + lo, so v keeps ~16 mantissa bits), walks
// 16-column tiles of B^T and updates y in place.
// ------------------------------------------------------------------------------------------------
template <int KSTEPS, int TILES>
static __device__ __forceinline__ void expand_body(const Unit &u, const SegRec &s,
                                                   const int32_t *__restrict__ perm,
                                                   const uint16_t *__restrict__ arena,
                                                   const float *__restrict__ v_in, int n_slices,
                                                   int64_t slice_stride, uint16_t *__restrict__ y,
                                                   int64_t ldy)
{
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int i = lane & 15;
    const int kq = lane >> 4;
    const int r8 = s.r8;
    const bool t_ok = i < u.ntok;
    const uint4 zero = {0u, 0u, 0u, 0u};

    bf16x8 vhi[KSTEPS], vlo[KSTEPS];
    int jc[KSTEPS];
    bool j_ok[KSTEPS];
#pragma unroll
    for (int st = 0; st < KSTEPS; ++st) {
        const int j = 32 * st + 8 * kq;
        j_ok[st] = j < r8;
        jc[st] = j_ok[st] ? j : 0;
        float f[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) f[e] = 0.f;
        if (t_ok && j_ok[st]) {
            const float *src = v_in + s.v_off + (int64_t)(u.tok0 + i) * r8 + j;
            for (int sl = 0; sl < n_slices; ++sl) {
                const f32x4 lo4 = *reinterpret_cast<const f32x4 *>(src + (int64_t)sl * slice_stride);
                const f32x4 hi4 = *reinterpret_cast<const f32x4 *>(src + (int64_t)sl * slice_stride + 4);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    f[e] += lo4[e];
                    f[4 + e] += hi4[e];
                }
            }
        }
        uint32_t h[8], l[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            h[e] = f32_to_bf16_bits(f[e]);
            l[e] = f32_to_bf16_bits(f[e] - bf16_bits_to_f32(h[e]));
        }
        uint4 ph = {h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16)};
        uint4 pl = {l[0] | (l[1] << 16), l[2] | (l[3] << 16), l[4] | (l[5] << 16), l[6] | (l[7] << 16)};
        vhi[st] = as_bf16x8(ph);
        vlo[st] = as_bf16x8(pl);
    }

    const int token = perm[s.tok_start + u.tok0 + (t_ok ? i : 0)];
    uint16_t *yrow = y + (int64_t)token * ldy;
    const uint16_t *bbase = arena + s.b_off;
    const float scale = s.scale;
    const int cend = u.p0 + u.pn;

    for (int c0 = u.p0 + 16 * wave; c0 < cend; c0 += 64 * TILES) {
        uint4 w[TILES][KSTEPS];
        uint2 yv[TILES];
#pragma unroll
        for (int tl = 0; tl < TILES; ++tl) {
            const int c = c0 + 64 * tl;
            if (c < cend) {
                const uint16_t *brow = bbase + (int64_t)(c + i) * r8;
#pragma unroll
                for (int st = 0; st < KSTEPS; ++st) w[tl][st] = ld16(brow + jc[st]);
                yv[tl] = t_ok ? *reinterpret_cast<const uint2 *>(yrow + c + 4 * kq) : make_uint2(0u, 0u);
            } else {
#pragma unroll
                for (int st = 0; st < KSTEPS; ++st) w[tl][st] = zero;
                yv[tl] = make_uint2(0u, 0u);
            }
        }
#pragma unroll
        for (int tl = 0; tl < TILES; ++tl) {
            const int c = c0 + 64 * tl;
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int st = 0; st < KSTEPS; ++st) {
                const bf16x8 ww = as_bf16x8(j_ok[st] ? w[tl][st] : zero);
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ww, vhi[st], acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ww, vlo[st], acc, 0, 0, 0);
            }
            if (t_ok && c < cend) {
                const float y0 = bf16_bits_to_f32(yv[tl].x & 0xFFFFu) + scale * acc[0];
                const float y1 = bf16_bits_to_f32(yv[tl].x >> 16) + scale * acc[1];
                const float y2 = bf16_bits_to_f32(yv[tl].y & 0xFFFFu) + scale * acc[2];
                const float y3 = bf16_bits_to_f32(yv[tl].y >> 16) + scale * acc[3];
                uint2 o;
                o.x = f32_to_bf16_bits(y0) | (f32_to_bf16_bits(y1) << 16);
                o.y = f32_to_bf16_bits(y2) | (f32_to_bf16_bits(y3) << 16);
                *reinterpret_cast<uint2 *>(yrow + c + 4 * kq) = o;
            }
        }
    }
}

__global__ __launch_bounds__(kThreads) void k_expand(const Unit *__restrict__ units,
                                                     const SegRec *__restrict__ segs,
                                                     const int32_t *__restrict__ perm,
                                                     const uint16_t *__restrict__ arena,
                                                     const float *__restrict__ v_in, int n_slices,
                                                     int64_t slice_stride, uint16_t *__restrict__ y,
                                                     int64_t ldy)
{
    const Unit u = units[blockIdx.x];
    const SegRec s = segs[u.seg];
    if (s.r8 <= 32)
        expand_body<1, 8>(u, s, perm, arena, v_in, n_slices, slice_stride, y, ldy);
    else if (s.r8 <= 64)
        expand_body<2, 4>(u, s, perm, arena, v_in, n_slices, slice_stride, y, ldy);
    else if (s.r8 <= 128)
        expand_body<4, 2>(u, s, perm, arena, v_in, n_slices, slice_stride, y, ldy);
    else
        expand_body<8, 1>(u, s, perm, arena, v_in, n_slices, slice_stride, y, ldy);
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
    hipLaunchKernelGGL(k_shrink, dim3(c.n_units), dim3(kThreads), 0, stream, c.units, c.segs, c.perm, c.arena, x,
                       ldx, c.in_features, k_slice_len, v_out, slice_stride);
    return hipGetLastError();
}

hipError_t launch_expand(const LaunchCtx &c, const float *v_in, int n_slices, int64_t slice_stride, uint16_t *y,
                         int64_t ldy, hipStream_t stream)
{
    if (c.n_units <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_expand, dim3(c.n_units), dim3(kThreads), 0, stream, c.units, c.segs, c.perm, c.arena,
                       v_in, n_slices, slice_stride, y, ldy);
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
