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
// Hand-over of v between the two halves of a fused launch.  The L2 caches of the chip's eight XCDs
// are not coherent with each other, and a device-scope fence (write back / invalidate a whole L2)
// costs far more than the data is worth.  So the partial sums of v never live in a cache: they are
// stored and loaded with device-scope relaxed atomics (64 bits at a time), which go through to
// memory.  A shrink work group waits until its stores have completed, then bumps the counter of its
// (group, token tile); an expand work group polls that counter until it has reached
// epoch * (shrink units of the tile).  Counters only grow: epoch is the number of fused launches
// the table has seen, so nothing is cleared between launches.  The wait is bounded: at the limit
// the work group records it in *timeout_flag and goes on, so every wavefront reaches its end.
// Shrink units come first in the grid and never wait, and work groups are dispatched in grid order,
// so a waiting expand unit never keeps a shrink unit from running.
// ------------------------------------------------------------------------------------------------
struct Sync {
    unsigned *counters;       // arrivals, one per (group, token tile); NULL = no hand-over through counters
    unsigned *ready;          // one per tile: bumped once per launch when the tile's v is complete
    unsigned *timeout_flag;
    uint16_t *v_hi;           // complete v as two bf16 terms, same indexing as the fp32 partial sums
    uint16_t *v_lo;
    unsigned epoch;
    unsigned spin_limit;
    int wait;                 // expand units poll `ready` (single launch) or not (expand launched after shrink)
};

static __device__ __forceinline__ void st_through_f32x4(float *p, f32x4 v)
{
    typedef __attribute__((ext_vector_type(2))) float f32x2;
    uint64_t *q = reinterpret_cast<uint64_t *>(p);
    const f32x2 lo = {v[0], v[1]}, hi = {v[2], v[3]};
    __hip_atomic_store(q, __builtin_bit_cast(uint64_t, lo), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(q + 1, __builtin_bit_cast(uint64_t, hi), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

static __device__ __forceinline__ f32x4 ld_through_f32x4(const float *p)
{
    typedef __attribute__((ext_vector_type(2))) float f32x2;
    const uint64_t *q = reinterpret_cast<const uint64_t *>(p);
    const f32x2 lo = __builtin_bit_cast(f32x2, __hip_atomic_load(q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
    const f32x2 hi = __builtin_bit_cast(f32x2, __hip_atomic_load(q + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
    return f32x4{lo[0], lo[1], hi[0], hi[1]};
}

static __device__ __forceinline__ void stores_done()
{
    __atomic_signal_fence(__ATOMIC_SEQ_CST);
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wavefront's stores have completed
    __atomic_signal_fence(__ATOMIC_SEQ_CST);
}

static __device__ __forceinline__ void st_through_u16x8(uint16_t *p, uint4 v)
{
    uint64_t *q = reinterpret_cast<uint64_t *>(p);
    __hip_atomic_store(q, (uint64_t)v.x | ((uint64_t)v.y << 32), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(q + 1, (uint64_t)v.z | ((uint64_t)v.w << 32), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

static __device__ __forceinline__ uint4 ld_through_u16x8(const uint16_t *p)
{
    const uint64_t *q = reinterpret_cast<const uint64_t *>(p);
    const uint64_t a = __hip_atomic_load(q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const uint64_t b = __hip_atomic_load(q + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return make_uint4((uint32_t)a, (uint32_t)(a >> 32), (uint32_t)b, (uint32_t)(b >> 32));
}

static __device__ __forceinline__ void wait_for(const Sync &sy, int idx)
{
    if (threadIdx.x == 0) {
        const unsigned target = sy.epoch;
        unsigned spins = 0;
        while (__hip_atomic_load(sy.ready + idx, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
            if (++spins > sy.spin_limit) {
                atomicOr(sy.timeout_flag, 1u);
                break;
            }
            __builtin_amdgcn_s_sleep(8);
        }
    }
    __syncthreads();
    __atomic_signal_fence(__ATOMIC_SEQ_CST);
}

static __device__ __forceinline__ uint32_t pack_bf16_rne(float a, float b)
{
    typedef __attribute__((ext_vector_type(2))) float f32x2;
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
    const f32x2 f = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));
}

// 8 floats -> bf16 hi (nearest) and bf16 lo (nearest of the remainder): hi + lo keeps ~16 mantissa bits
static __device__ __forceinline__ void split_bf16(f32x4 f0, f32x4 f1, uint4 &ph, uint4 &pl)
{
    ph.x = pack_bf16_rne(f0[0], f0[1]);
    ph.y = pack_bf16_rne(f0[2], f0[3]);
    ph.z = pack_bf16_rne(f1[0], f1[1]);
    ph.w = pack_bf16_rne(f1[2], f1[3]);
    pl.x = pack_bf16_rne(f0[0] - bf16_bits_to_f32(ph.x & 0xFFFFu), f0[1] - __uint_as_float(ph.x & 0xFFFF0000u));
    pl.y = pack_bf16_rne(f0[2] - bf16_bits_to_f32(ph.y & 0xFFFFu), f0[3] - __uint_as_float(ph.y & 0xFFFF0000u));
    pl.z = pack_bf16_rne(f1[0] - bf16_bits_to_f32(ph.z & 0xFFFFu), f1[1] - __uint_as_float(ph.z & 0xFFFF0000u));
    pl.w = pack_bf16_rne(f1[2] - bf16_bits_to_f32(ph.w & 0xFFFFu), f1[3] - __uint_as_float(ph.w & 0xFFFF0000u));
}

constexpr int kMaxSlices = 4;  // upper bound of the shrink's k-slices

// sum of the k-slices' partial sums of 8 consecutive v elements, in slice order
static __device__ __forceinline__ void sum_slices(const float *__restrict__ src, int n_slices, int64_t slice_stride,
                                                  f32x4 &f0, f32x4 &f1)
{
    f32x4 p0[kMaxSlices], p1[kMaxSlices];
#pragma unroll
    for (int sl = 0; sl < kMaxSlices; ++sl) {
        const int64_t off = (int64_t)(sl < n_slices ? sl : 0) * slice_stride;
        p0[sl] = ld_through_f32x4(src + off);
        p1[sl] = ld_through_f32x4(src + off + 4);
    }
    f0 = p0[0];
    f1 = p1[0];
#pragma unroll
    for (int sl = 1; sl < kMaxSlices; ++sl)
        if (sl < n_slices) {
            f0 += p0[sl];
            f1 += p1[sl];
        }
}

// ------------------------------------------------------------------------------------------------
// shrink: one unit = (group, <=16 tokens, 16 rank rows, one k-slice).  The four wavefronts split the
// k-slice.  Each issues its 16-byte weight loads up front (rows of A^T straight into the MFMA's
// row operand); meanwhile the work group stages the tokens' x slab for this k-slice in LDS with
// coalesced loads, from which every wavefront reads its token operand.  Each wavefront accumulates
// a 16x16 tile (rank row x token); the four tiles are summed through LDS in wavefront order.
// ------------------------------------------------------------------------------------------------
constexpr int kShrinkSteps = 8;                   // 32-wide k steps per wavefront per pass
constexpr int kSlabK = 4 * 32 * kShrinkSteps;     // k range staged per pass (all four wavefronts)
constexpr int kSlabRow = kSlabK + 8;              // LDS row length in bf16, padded by 16 bytes
constexpr int kShrinkLds = kTokTile * kSlabRow * 2 + 4 * 64 * 16;

static __device__ __forceinline__ void shrink_body(const Unit &u, const uint16_t *__restrict__ arena,
                                                   const uint16_t *__restrict__ x, int64_t ldx, int in,
                                                   int k_slice_len, float *__restrict__ v_out, int n_slices,
                                                   int64_t slice_stride, char *lds, const Sync &sy)
{
    uint16_t(*slab)[kSlabRow] = reinterpret_cast<uint16_t(*)[kSlabRow]>(lds);
    f32x4(*red)[64] = reinterpret_cast<f32x4(*)[64]>(lds + kTokTile * kSlabRow * 2);
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int i = lane & 15;
    const int kq = lane >> 4;

    const int ntok = u.ntok, pn = u.pn, ks = u.ks;
    const bool w_ok = i < pn;
    const bool x_ok = i < ntok;
    const uint16_t *wrow = arena + u.w_off + (int64_t)(w_ok ? i : 0) * in;
    // slab staging: thread tid copies 16-byte chunk (tid & 127) of tokens (tid >> 7), +2, +4, ...
    const int s_chunk = tid & 127;
    const int s_tok0 = __builtin_amdgcn_readfirstlane(tid >> 7);  // wavefront-uniform

    const int kslice_beg = ks * k_slice_len;
    int kslice_end = kslice_beg + k_slice_len;
    if (kslice_end > in) kslice_end = in;

    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    const uint4 zero = {0u, 0u, 0u, 0u};
    for (int kp = kslice_beg; kp < kslice_end; kp += kSlabK) {
        // this wavefront's k range inside the pass
        const int kbeg = kp + wave * (32 * kShrinkSteps);
        uint4 a[kShrinkSteps];
#pragma unroll
        for (int q = 0; q < kShrinkSteps; ++q) {
            const int k = kbeg + 32 * q;
            a[q] = (k < kslice_end) ? ld16(wrow + k + 8 * kq) : zero;
        }
        if (kp != kslice_beg) __syncthreads();  // previous pass's slab is no longer being read
        {
            const int k = kp + 8 * s_chunk;
            if (k < kslice_end) {
                uint4 xs[kTokTile / 2];
#pragma unroll
                for (int t = 0; t < kTokTile / 2; ++t) {
                    const int tok = s_tok0 + 2 * t;
                    xs[t] = (tok < ntok) ? ld16(x + (int64_t)u.tok[tok] * ldx + k) : zero;
                }
#pragma unroll
                for (int t = 0; t < kTokTile / 2; ++t) {
                    const int tok = s_tok0 + 2 * t;
                    if (tok < ntok) *reinterpret_cast<uint4 *>(&slab[tok][8 * s_chunk]) = xs[t];
                }
            }
        }
        __syncthreads();
#pragma unroll
        for (int q = 0; q < kShrinkSteps; ++q) {
            const int k = kbeg + 32 * q;
            if (k < kslice_end) {
                const uint4 aa = w_ok ? a[q] : zero;
                const uint4 bb = x_ok ? *reinterpret_cast<const uint4 *>(&slab[i][k - kp + 8 * kq]) : zero;
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(aa), as_bf16x8(bb), acc, 0, 0, 0);
            }
        }
    }
    red[wave][lane] = acc;
    __syncthreads();
    if (wave == 0) {
        f32x4 t = red[0][lane];
        t += red[1][lane];
        t += red[2][lane];
        t += red[3][lane];
        if (x_ok && 4 * kq < pn) {
            float *dst = v_out + (int64_t)ks * slice_stride + u.v_off + (int64_t)i * u.r8 + 4 * kq;
            st_through_f32x4(dst, t);
        }
        if (sy.counters) {
            // count this unit in; the unit that completes its token tile adds the k-slices up and
            // leaves the tile's v as bf16 hi + lo for the expand units
            stores_done();
            unsigned old = 0;
            if (lane == 0) old = atomicAdd(sy.counters + u.sync_idx, 1u);
            old = __builtin_amdgcn_readfirstlane(old);
            if (old + 1u == sy.epoch * (unsigned)u.sync_n) {
                const int64_t tile_off = u.v_off - u.p0;
                const int tasks = ntok * (u.r8 >> 3);
                for (int task = lane; task < tasks; task += 64) {
                    f32x4 f0, f1;
                    sum_slices(v_out + tile_off + 8 * task, n_slices, slice_stride, f0, f1);
                    uint4 ph, pl;
                    split_bf16(f0, f1, ph, pl);
                    st_through_u16x8(sy.v_hi + tile_off + 8 * task, ph);
                    st_through_u16x8(sy.v_lo + tile_off + 8 * task, pl);
                }
                stores_done();
                if (lane == 0) atomicAdd(sy.ready + u.sync_idx, 1u);
            }
        }
    }
}

// ------------------------------------------------------------------------------------------------
// expand: one unit = (group, <=16 tokens, a run of output columns made of 128-column strips).
// MFMA orientation: tokens down (operand from v), output columns across (operand straight from
// 16-byte loads of B^T rows).  Inside a strip, MFMA b (0..7) takes column 8*n + b for its column
// slot n, so that after the eight MFMAs lane n holds 8 consecutive columns of up to 4 tokens: y is
// then read and written 16 bytes per lane.  The four wavefronts of a work group split the unit by
// strip and by k step (rank >= 128: one strip, one 32-wide slice of the rank each); partial tiles
// meet in LDS and are added in wavefront order by the y update, which all 256 threads share.
// v enters as two bf16 terms (hi + lo), so it keeps about 16 mantissa bits.
// ------------------------------------------------------------------------------------------------
constexpr int kStrip = 128;           // output columns per strip
constexpr int kPartRow = kStrip + 4;  // LDS row length of a partial tile in floats (padded)
constexpr int kExpandLds = 4 * kTokTile * kPartRow * 4;

// v operand of one 32-wide k step from fp32 v: token n, 8 values, k-slices added in slice order,
// split into bf16 hi + lo.
static __device__ __forceinline__ void load_v_operand(const float *__restrict__ src, bool ok, int n_slices,
                                                      int64_t slice_stride, bf16x8 &vhi, bf16x8 &vlo)
{
    f32x4 f0, f1;
    sum_slices(src, n_slices, slice_stride, f0, f1);
    if (!ok) {
        f0 = f32x4{0.f, 0.f, 0.f, 0.f};
        f1 = f0;
    }
    uint4 ph, pl;
    split_bf16(f0, f1, ph, pl);
    vhi = as_bf16x8(ph);
    vlo = as_bf16x8(pl);
}

// KSTEPS: 32-wide steps that cover the padded rank (1, 2, 4 or 8).
template <int KSTEPS>
static __device__ __forceinline__ void expand_body(const Unit &u, const uint16_t *__restrict__ arena,
                                                   const float *__restrict__ v_in, int n_slices,
                                                   int64_t slice_stride, uint16_t *__restrict__ y,
                                                   int64_t ldy, char *lds, const Sync &sy)
{
    constexpr int P = KSTEPS < 4 ? KSTEPS : 4;  // wavefronts that share one strip (each a part of the rank)
    constexpr int S = 4 / P;                    // strips per pass of the work group
    constexpr int ITEMS = KSTEPS / P;           // k steps per wavefront (1, or 2 for rank > 128)
    float(*part)[kTokTile][kPartRow] = reinterpret_cast<float(*)[kTokTile][kPartRow]>(lds);
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int n = lane & 15;
    const int kq = lane >> 4;
    const int r8 = u.r8;
    const int ntok = u.ntok;
    const int ncols = u.pn;
    const uint4 zero = {0u, 0u, 0u, 0u};
    const int my_strip = wave / P;
    const int my_part = wave % P;

    // epilogue role of this thread: token e_tok, 8 columns starting at 8*e_cg of every strip
    const int e_tok = tid >> 4;
    const int e_cg = tid & 15;
    const bool e_ok = e_tok < ntok;
    uint16_t *e_y = y + (int64_t)u.tok[e_ok ? e_tok : 0] * ldy + u.p0 + 8 * e_cg;
    const float scale = u.scale;

    int jc[ITEMS];
    bool j_ok[ITEMS];
#pragma unroll
    for (int it = 0; it < ITEMS; ++it) {
        const int j = 32 * (my_part + P * it) + 8 * kq;
        j_ok[it] = j < r8;
        jc[it] = j_ok[it] ? j : 0;
    }
    bf16x8 vhi[ITEMS], vlo[ITEMS];

    for (int c0 = 0; c0 < ncols; c0 += S * kStrip) {
        const int cs = c0 + my_strip * kStrip;  // this wavefront's strip
        const bool strip_ok = cs < ncols;
        const uint16_t *brow = arena + u.w_off + (int64_t)((strip_ok ? cs : 0) + 8 * n) * r8;
        // first k step's weights: row (column of y) cs + 8*n + b, 16 bytes at jc
        uint4 w[8];
#pragma unroll
        for (int b = 0; b < 8; ++b) w[b] = ld16(brow + (int64_t)b * r8 + jc[0]);
        // y of this thread's epilogue share
        uint4 yv[S];
#pragma unroll
        for (int s = 0; s < S; ++s)
            yv[s] = (e_ok && c0 + s * kStrip < ncols) ? *reinterpret_cast<const uint4 *>(e_y + c0 + s * kStrip) : zero;

        if (c0 == 0) {
            // the weights above are in flight; now v has to be there
            if (sy.counters && sy.wait) wait_for(sy, u.sync_idx);
#pragma unroll
            for (int it = 0; it < ITEMS; ++it) {
                const bool ok = (n < ntok) && j_ok[it];
                const int64_t off = u.v_off + (int64_t)(ok ? n : 0) * r8 + jc[it];
                if (sy.counters) {
                    const uint4 ph = ld_through_u16x8(sy.v_hi + off);
                    const uint4 pl = ld_through_u16x8(sy.v_lo + off);
                    vhi[it] = as_bf16x8(ok ? ph : zero);
                    vlo[it] = as_bf16x8(ok ? pl : zero);
                } else {
                    load_v_operand(v_in + off, ok, n_slices, slice_stride, vhi[it], vlo[it]);
                }
            }
        } else {
            __syncthreads();  // the previous pass's partial tiles have been consumed
        }

        f32x4 acc[8];
#pragma unroll
        for (int b = 0; b < 8; ++b) acc[b] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int it = 0; it < ITEMS; ++it) {
            uint4 wn[8];
            if (it + 1 < ITEMS) {
#pragma unroll
                for (int b = 0; b < 8; ++b) wn[b] = ld16(brow + (int64_t)b * r8 + jc[it + 1 < ITEMS ? it + 1 : 0]);
            }
#pragma unroll
            for (int b = 0; b < 8; ++b) {
                const bf16x8 ww = as_bf16x8(j_ok[it] ? w[b] : zero);
                acc[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vhi[it], ww, acc[b], 0, 0, 0);
                acc[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vlo[it], ww, acc[b], 0, 0, 0);
            }
            if (it + 1 < ITEMS) {
#pragma unroll
                for (int b = 0; b < 8; ++b) w[b] = wn[b];
            }
        }
        if (strip_ok) {
            // lane (n, kq) holds tokens 4*kq + e, columns 8*n + b
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int tok = 4 * kq + e;
                if (tok < ntok) {
                    const f32x4 lo = {acc[0][e], acc[1][e], acc[2][e], acc[3][e]};
                    const f32x4 hi = {acc[4][e], acc[5][e], acc[6][e], acc[7][e]};
                    *reinterpret_cast<f32x4 *>(&part[wave][tok][8 * n]) = lo;
                    *reinterpret_cast<f32x4 *>(&part[wave][tok][8 * n + 4]) = hi;
                }
            }
        }
        __syncthreads();
        if (e_ok) {
#pragma unroll
            for (int s = 0; s < S; ++s) {
                if (c0 + s * kStrip < ncols) {
                    f32x4 d0 = *reinterpret_cast<const f32x4 *>(&part[s * P][e_tok][8 * e_cg]);
                    f32x4 d1 = *reinterpret_cast<const f32x4 *>(&part[s * P][e_tok][8 * e_cg + 4]);
#pragma unroll
                    for (int p = 1; p < P; ++p) {
                        d0 += *reinterpret_cast<const f32x4 *>(&part[s * P + p][e_tok][8 * e_cg]);
                        d1 += *reinterpret_cast<const f32x4 *>(&part[s * P + p][e_tok][8 * e_cg + 4]);
                    }
                    const uint4 yy = yv[s];
                    uint4 o;
                    o.x = pack_bf16_rne(bf16_bits_to_f32(yy.x & 0xFFFFu) + scale * d0[0],
                                        __uint_as_float(yy.x & 0xFFFF0000u) + scale * d0[1]);
                    o.y = pack_bf16_rne(bf16_bits_to_f32(yy.y & 0xFFFFu) + scale * d0[2],
                                        __uint_as_float(yy.y & 0xFFFF0000u) + scale * d0[3]);
                    o.z = pack_bf16_rne(bf16_bits_to_f32(yy.z & 0xFFFFu) + scale * d1[0],
                                        __uint_as_float(yy.z & 0xFFFF0000u) + scale * d1[1]);
                    o.w = pack_bf16_rne(bf16_bits_to_f32(yy.w & 0xFFFFu) + scale * d1[2],
                                        __uint_as_float(yy.w & 0xFFFF0000u) + scale * d1[3]);
                    *reinterpret_cast<uint4 *>(e_y + c0 + s * kStrip) = o;
                }
            }
        }
    }
}

static __device__ __forceinline__ void expand_dispatch(const Unit &u, const uint16_t *__restrict__ arena,
                                                       const float *__restrict__ v_in, int n_slices,
                                                       int64_t slice_stride, uint16_t *__restrict__ y,
                                                       int64_t ldy, char *lds, const Sync &sy)
{
    const int r8 = u.r8;
    if (r8 <= 32)
        expand_body<1>(u, arena, v_in, n_slices, slice_stride, y, ldy, lds, sy);
    else if (r8 <= 64)
        expand_body<2>(u, arena, v_in, n_slices, slice_stride, y, ldy, lds, sy);
    else if (r8 <= 128)
        expand_body<4>(u, arena, v_in, n_slices, slice_stride, y, ldy, lds, sy);
    else
        expand_body<8>(u, arena, v_in, n_slices, slice_stride, y, ldy, lds, sy);
}

constexpr int kFusedLds = kShrinkLds > kExpandLds ? kShrinkLds : kExpandLds;

__global__ __launch_bounds__(kThreads) void k_shrink(const Unit *__restrict__ units,
                                                     const uint16_t *__restrict__ arena,
                                                     const uint16_t *__restrict__ x, int64_t ldx, int in,
                                                     int k_slice_len, float *__restrict__ v_out, int n_slices,
                                                     int64_t slice_stride, Sync sy)
{
    __shared__ __attribute__((aligned(16))) char lds[kShrinkLds];
    shrink_body(units[blockIdx.x], arena, x, ldx, in, k_slice_len, v_out, n_slices, slice_stride, lds, sy);
}

__global__ __launch_bounds__(kThreads, 4) void k_expand(const Unit *__restrict__ units,
                                                     const uint16_t *__restrict__ arena,
                                                     const float *__restrict__ v_in, int n_slices,
                                                     int64_t slice_stride, uint16_t *__restrict__ y,
                                                     int64_t ldy, Sync sy)
{
    __shared__ __attribute__((aligned(16))) char lds[kExpandLds];
    expand_dispatch(units[blockIdx.x], arena, v_in, n_slices, slice_stride, y, ldy, lds, sy);
}

// Both halves in one launch: blocks [0, n_shrink) are shrink units, the rest expand units that wait
// for their tokens' v through the counters.
__global__ __launch_bounds__(kThreads, 4) void k_apply_fused(const Unit *__restrict__ shrink_units, int n_shrink,
                                                          const Unit *__restrict__ expand_units,
                                                          const uint16_t *__restrict__ arena,
                                                          const uint16_t *__restrict__ x, int64_t ldx, int in,
                                                          int k_slice_len, float *__restrict__ parts, int n_slices,
                                                          int64_t slice_stride, uint16_t *__restrict__ y,
                                                          int64_t ldy, Sync sy)
{
    __shared__ __attribute__((aligned(16))) char lds[kFusedLds];
    const int b = blockIdx.x;
    if (b < n_shrink)
        shrink_body(shrink_units[b], arena, x, ldx, in, k_slice_len, parts, n_slices, slice_stride, lds, sy);
    else
        expand_dispatch(expand_units[b - n_shrink], arena, parts, n_slices, slice_stride, y, ldy, lds, sy);
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
static Sync make_sync(const SyncArgs *a, int wait)
{
    Sync sy;
    if (!a) {
        sy = Sync{nullptr, nullptr, nullptr, nullptr, nullptr, 0u, 0u, 0};
    } else {
        sy = Sync{a->counters, a->ready, a->timeout_flag, a->v_hi, a->v_lo, a->epoch, a->spin_limit, wait};
    }
    return sy;
}

hipError_t launch_shrink(const LaunchCtx &c, const uint16_t *x, int64_t ldx, int k_slice_len, float *v_out,
                         int n_slices, int64_t slice_stride, const SyncArgs *sync, hipStream_t stream)
{
    if (c.n_units <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_shrink, dim3(c.n_units), dim3(kThreads), 0, stream, c.units, c.arena, x, ldx,
                       c.in_features, k_slice_len, v_out, n_slices, slice_stride, make_sync(sync, 0));
    return hipGetLastError();
}

hipError_t launch_expand(const LaunchCtx &c, const float *v_in, int n_slices, int64_t slice_stride, uint16_t *y,
                         int64_t ldy, const SyncArgs *sync, hipStream_t stream)
{
    if (c.n_units <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_expand, dim3(c.n_units), dim3(kThreads), 0, stream, c.units, c.arena, v_in, n_slices,
                       slice_stride, y, ldy, make_sync(sync, 0));
    return hipGetLastError();
}

hipError_t launch_apply_fused(const LaunchCtx &cs, const LaunchCtx &ce, const uint16_t *x, int64_t ldx,
                              int k_slice_len, float *parts, int n_slices, int64_t slice_stride, uint16_t *y,
                              int64_t ldy, const SyncArgs *sync, hipStream_t stream)
{
    const int total = cs.n_units + ce.n_units;
    if (total <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_apply_fused, dim3(total), dim3(kThreads), 0, stream, cs.units, cs.n_units, ce.units,
                       cs.arena, x, ldx, cs.in_features, k_slice_len, parts, n_slices, slice_stride, y, ldy,
                       make_sync(sync, 1));
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
