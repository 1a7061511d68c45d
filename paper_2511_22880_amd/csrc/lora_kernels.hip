// gfx950 kernels of the co-batched LoRA delta (shrink: v = x A_a, expand: y += s_a v B_a).
//
// Both adapter matrices are stored the way a 16x16x32 bf16 MFMA reads its weight operand: lane l
// supplies row (l & 15) of a 16-row weight tile and the 8 consecutive k values 8*(l >> 4) .. +7 of a
// 32-wide k step, so the pool keeps, for every 16-row tile and every k step, the 64 lanes' 16-byte
// pieces back to back.  One wavefront load of an operand is then 1 KB of consecutive bytes (a
// row-major matrix would make it 16 pieces of 64 bytes, which costs the address path of a CU about
// 3.7 times as many cycles):
//   A^T: 16-row block jb (the last block has 8 rows when the padded rank is 8 mod 16), k step s,
//        piece (kq, row n): element offset  16*jb*in + s*(32*h) + (kq*h + n)*8,  h = rows in the block
//   B^T: 128-column strip, sub-block b (the 16 columns 8*n + b), rank piece kp (8 values), column
//        slot n: element offset  128*strip*r8 + ((b*(r8/8) + kp)*16 + n)*8
// The token operand uses the same lane->k mapping, so the order of k inside a step is irrelevant to
// the result.  The 16x16 fp32 result tile has D[4*(l >> 4) + i][l & 15] in register i of lane l.
//
// Work is cut on the host into units of roughly equal adapter bytes; one work group (4 wavefronts)
// takes one unit.  No unit ever depends on another adapter's rank.
#include "lora_internal.h"

#include <atomic>

namespace lora {

// Per-work-group device clocks, in builds with -DLORA_WG_CLOCKS only (the measurement build of the
// library; see lora_debug_clock_buffer): wavefront 0 of a work group writes the 100 MHz wall clock at a
// few points of its unit into slot (work group, point) of a caller's buffer.  Ordinary builds compile
// the macro to nothing.
#ifdef LORA_WG_CLOCKS
__device__ unsigned long long *g_clock_buf = nullptr;
__device__ unsigned g_clock_slots = 0;
#define LORA_CLOCK_AT(base, point)                                                                     \
    do {                                                                                               \
        if (g_clock_buf && threadIdx.x == 0 && (base) + blockIdx.x < g_clock_slots)                    \
            g_clock_buf[((size_t)(base) + blockIdx.x) * 8 + (point)] = wall_clock64();                 \
    } while (0)
#else
#define LORA_CLOCK_AT(base, point) do { } while (0)
#endif
#define LORA_CLOCK(point) LORA_CLOCK_AT(0, point)
// expand launches keep their clocks behind those of the shrink launch of the same apply
[[maybe_unused]] constexpr unsigned kClockExpandBase = 32768;
#define LORA_CLOCK_E(point) LORA_CLOCK_AT(kClockExpandBase, point)

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

static __device__ __forceinline__ bf16x8 as_bf16x8(uint4 u) { return __builtin_bit_cast(bf16x8, u); }

static __device__ __forceinline__ uint4 ld16(const uint16_t *p) { return *reinterpret_cast<const uint4 *>(p); }

// 16-byte load of data that is read exactly once per launch (a decode batch's adapter weights, the
// x rows of a token-heavy shrink): marked non-temporal, so it is not kept in the caches on its way.
// A plain read of 2 GB runs at 6.2 TB/s on this chip with ordinary loads and at 7.0 TB/s with these.
static __device__ __forceinline__ uint4 ld16_stream(const uint16_t *p)
{
    typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
    const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
    return uint4{v.x, v.y, v.z, v.w};
}

// 16-byte store of data this launch will not read again (y).
static __device__ __forceinline__ void st16_stream(uint16_t *p, uint4 v)
{
    typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
    __builtin_nontemporal_store(u32x4{v.x, v.y, v.z, v.w}, reinterpret_cast<u32x4 *>(p));
}

static __device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

// ------------------------------------------------------------------------------------------------
// Hand-over of v between the two halves of a fused launch.  The L2 caches of the chip's eight XCDs
// are not coherent with each other, and a device-scope fence (write back / invalidate a whole L2)
// costs far more than the data is worth.  So the partial sums of v never live in a cache: they are
// stored and loaded with device-scope relaxed atomics (64 bits at a time), which go through to
// memory.  A shrink work group waits until its stores have completed, then bumps the arrival counter
// of its (group, token tile); the one whose bump completes the tile's count for this launch adds the
// slices up, sets the arrival counter back to zero (a launch leaves the table as it found it, so a
// launch replayed from a captured graph finds what the first one found) and bumps the tile's ready
// counter.  Only the single-launch form reads the ready counters: an expand work group polls its
// tile's until it has reached epoch, the number of such launches the table has seen (they only
// grow, so nothing is cleared between launches).  The wait is bounded: at the limit
// the work group records it in *timeout_flag and goes on, so every wavefront reaches its end.
// Shrink units come first in the grid and never wait, and work groups are dispatched in grid order,
// so a waiting expand unit never keeps a shrink unit from running.
// ------------------------------------------------------------------------------------------------
struct Sync {
    unsigned *counters;       // arrivals, one per (group, token tile); NULL = no hand-over through counters
    unsigned *ready;          // one per tile: bumped once per single-launch apply when the tile's v is complete
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

// The s_waitcnt immediate of the gfx9 family (gfx950 included): vmcnt in bits 3:0 and 15:14, expcnt in
// bits 6:4, lgkmcnt in bits 11:8; a field at its maximum waits for nothing.
#if defined(__HIP_DEVICE_COMPILE__) && !defined(__gfx950__)
#error "the hand-built s_waitcnt immediate below is the gfx9 encoding: this file is for gfx950"
#endif
constexpr unsigned kWaitcntVmcnt0 = (0u << 0) | (7u << 4) | (15u << 8) | (0u << 14);  // vmcnt(0), nothing else
static_assert(kWaitcntVmcnt0 == 0x0F70, "vmcnt(0) expcnt(7) lgkmcnt(15)");

// This wavefront's vector memory operations (its stores among them) have completed.  The two signal
// fences keep the compiler from moving memory operations across the wait in either direction.
static __device__ __forceinline__ void stores_done()
{
    __atomic_signal_fence(__ATOMIC_SEQ_CST);
    __builtin_amdgcn_s_waitcnt(kWaitcntVmcnt0);
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
    // this lane's 16-byte piece of a k step of the unit's row block (pn = rows in the block: 16 or 8)
    const uint16_t *wrow = arena + u.w_off + (kq * pn + (w_ok ? i : 0)) * 8;
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
            a[q] = (k < kslice_end) ? ld16_stream(wrow + (int64_t)k * pn) : zero;
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
                // rows of tokens beyond ntok hold whatever LDS held: they only reach accumulator columns
                // that are never stored, and an unconditional 16-byte read stays one instruction
                const uint4 bb = *reinterpret_cast<const uint4 *>(&slab[i][k - kp + 8 * kq]);
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
            // nothing below (the loads of the other units' partial sums) moves up in front of the arrival
            __atomic_signal_fence(__ATOMIC_SEQ_CST);
            if (old + 1u == (unsigned)u.sync_n) {
                // the last of this launch's arrivals at the tile: the counter goes back to zero for the
                // next launch (nothing else touches it before this launch ends)
                if (lane == 0) atomicExch(sy.counters + u.sync_idx, 0u);
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
                if (sy.wait && lane == 0) atomicAdd(sy.ready + u.sync_idx, 1u);  // polled by the single-launch form only
            }
        }
    }
}

// A unit record read with one 128-byte request per wavefront: word w of the record in lane w (and w + 32).
// Its fields are then taken from that register (unit_word), so that a unit's operand loads are one trip to
// memory behind the start of its work group, not two (the token list after the token count).  Used by the
// one-launch decode kernel for its shrink units, every one of which is on the launch's critical path (15.4 ->
// 15.0 us on a 256-token batch; for its expand units' records, which are read while the shrink units run,
// 15.0 -> 15.2 us); in the launches of several rounds (k_shrink_wide, k_expand) it changed nothing or
// cost a little (28.9 -> 29.3 us for 2,560 expand units), so they read the record field by field.
static_assert(offsetof(Unit, w_off) == 0 && offsetof(Unit, v_off) == 8 && offsetof(Unit, r8) == 16 &&
                  offsetof(Unit, ntok) == 20 && offsetof(Unit, p0) == 24 && offsetof(Unit, pn) == 28 &&
                  offsetof(Unit, sync_idx) == 48 && offsetof(Unit, tok) == 64,
              "the words of a unit record as unit_word's callers number them");
static __device__ __forceinline__ uint32_t load_unit_words(const Unit *u)
{
    return reinterpret_cast<const uint32_t *>(u)[threadIdx.x & 31];
}
static __device__ __forceinline__ uint32_t unit_word(uint32_t rec, int w)
{
    return (uint32_t)__builtin_amdgcn_readlane((int)rec, w);
}

// ------------------------------------------------------------------------------------------------
// shrink, whole-k units: one unit = (group, <=16 tokens, 16 rank rows or one half of them, all of k), one work group of
// 16 wavefronts.  Used when the batch's units fit the chip in one round: each compute unit then
// streams one row block of one adapter with 128 KB of loads in flight, and v leaves complete (no
// partial sums in memory, no counters).  The work group is four k-slice units in one: wavefronts
// 4j .. 4j+3 do exactly the arithmetic of the four wavefronts of a k-slice unit for slice j, and the
// tiles are added in the same order (inside a slice by wavefront, then the slices), so the result
// is bitwise the one the k-slice path gives.  Every wavefront requests its 8 weight operands and its
// own piece of the tokens' x rows (coalesced, two tokens per load), turns the x piece into MFMA
// operand order through a private LDS region (no work-group barrier), and runs its 8 MFMAs.
// ------------------------------------------------------------------------------------------------
constexpr int kWideWaves = 4 * kMaxSlices;
constexpr int kWideThreads = 64 * kWideWaves;
constexpr int kWideK = 32 * kShrinkSteps;  // k range of one wavefront per pass
constexpr int kWideRow = kWideK + 8;       // LDS row length in bf16, padded by 16 bytes
constexpr int kWideSlab = kTokTile * kWideRow * 2;
constexpr int kWideLds = kWideWaves * kWideSlab + kWideWaves * 64 * 16;
constexpr int kWideHalfWaves = kWideWaves / 2;  // the same unit by 8 wavefronts, two of the 16 roles each

// WAVES = 16: one work group per compute unit.  WAVES = 8: every wavefront takes two of the sixteen roles
// in turn (role = wavefront, then wavefront + 8: the same place in another k-slice), and two work groups
// share a compute unit: for launches of more units than the chip has compute units, where one unit's
// record fetch, ramp and reduction then run beside the other's loads instead of between two units'
// (544 units of 8192 input features: 32.7 -> 29.9 us; four wavefronts in four roles, four work groups per
// compute unit: 32.4 us).
template <int WAVES>
__global__ __launch_bounds__(64 * WAVES, kWideWaves / WAVES) void k_shrink_wide(const Unit *__restrict__ units,
                                                              const uint16_t *__restrict__ arena,
                                                              const uint16_t *__restrict__ x, int64_t ldx, int in,
                                                              int k_slice_len, int n_slices,
                                                              float *__restrict__ v_f32,
                                                              uint16_t *__restrict__ v_hi,
                                                              uint16_t *__restrict__ v_lo)
{
    constexpr int ROLES = kWideWaves / WAVES;
    // the sixteen partial tiles: behind the x regions, or (8 wavefronts, so that two work groups fit the
    // compute unit's LDS) at the start of the x region of the wavefront that computed them
    constexpr bool kRedInSlab = WAVES < kWideWaves;
    __shared__ __attribute__((aligned(16))) char lds[kRedInSlab ? WAVES * kWideSlab : kWideLds];
    static_assert(ROLES * 64 * 16 <= kWideSlab, "a wavefront's partial tiles fit its x region");
    LORA_CLOCK(0);
    const Unit &u = units[blockIdx.x];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wq = wave & 3;      // its place among a slice's four wavefronts
    const int i = lane & 15;
    const int kq = lane >> 4;
    uint16_t(*slab)[kWideRow] = reinterpret_cast<uint16_t(*)[kWideRow]>(lds + wave * kWideSlab);
    auto red = [&](int role) __attribute__((always_inline)) -> f32x4 * {
        char *at = kRedInSlab ? lds + (role % WAVES) * kWideSlab + (role / WAVES) * (64 * 16)
                              : lds + kWideWaves * kWideSlab + role * (64 * 16);
        return reinterpret_cast<f32x4 *>(at);
    };

    const int ntok = u.ntok, pn = u.pn;
    const bool w_ok = i < pn;
    const bool x_ok = i < ntok;
    // the unit's rows are rows row0 .. row0 + pn - 1 of a block of blk_rows rows of A^T (all of the
    // block, or one half of a 16-row block), which starts at w_off
    const int blk_rows = min(kRowTile, u.r8 - (u.p0 & ~(kRowTile - 1)));
    const int row0 = u.p0 & (kRowTile - 1);
    const uint16_t *wrow = arena + u.w_off + (kq * blk_rows + row0 + (w_ok ? i : 0)) * 8;
    // x staging: lane -> token 2t + half, 16-byte chunk s_chunk of the wavefront's 256 k.  The unit's
    // token list repeats its first token beyond ntok, so every listed row is a valid row of x.
    const int half = lane >> 5;
    const int s_chunk = lane & 31;
    const uint16_t *xrow[kTokTile / 2];
#pragma unroll
    for (int t = 0; t < kTokTile / 2; ++t) xrow[t] = x + (int64_t)(half ? u.tok[2 * t + 1] : u.tok[2 * t]) * ldx;

    f32x4 accs[ROLES];
    const uint4 zero = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int ro = 0; ro < ROLES; ++ro) {
    const int slice = (wave + WAVES * ro) >> 2;  // the k-slice this role works on
    const int kslice_beg = slice * k_slice_len;
    int kslice_end = kslice_beg + k_slice_len;
    if (kslice_end > in) kslice_end = in;
    if (slice >= n_slices) kslice_end = kslice_beg;

    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int kp = kslice_beg; kp < kslice_end; kp += 4 * kWideK) {
        const int kbeg = kp + wq * kWideK;  // wavefront-uniform
        if (kbeg >= kslice_end) break;
        uint4 a[kShrinkSteps];
#pragma unroll
        for (int q = 0; q < kShrinkSteps; ++q) {
            const int k = kbeg + 32 * q;
            a[q] = (k < kslice_end) ? ld16_stream(wrow + (int64_t)k * blk_rows) : zero;
        }
        // in is a multiple of 64, so a 16-byte chunk is either inside the row or wholly beyond it;
        // chunks beyond it are fetched from the row's last chunk instead and never enter an MFMA
        int kx = kbeg + 8 * s_chunk;
        if (kx > in - 8) kx = in - 8;
        uint4 xs[kTokTile / 2];
#pragma unroll
        for (int t = 0; t < kTokTile / 2; ++t)
            if (2 * t < ntok) xs[t] = ld16(xrow[t] + kx);
#pragma unroll
        for (int t = 0; t < kTokTile / 2; ++t)
            if (2 * t < ntok) *reinterpret_cast<uint4 *>(&slab[2 * t + half][8 * s_chunk]) = xs[t];
        // the region is private to this wavefront and LDS operations of a wavefront complete in order
        __atomic_signal_fence(__ATOMIC_SEQ_CST);
        __builtin_amdgcn_wave_barrier();
        __atomic_signal_fence(__ATOMIC_SEQ_CST);
#pragma unroll
        for (int q = 0; q < kShrinkSteps; ++q) {
            const int k = kbeg + 32 * q;
            if (k < kslice_end) {
                const uint4 aa = w_ok ? a[q] : zero;
                // rows of tokens beyond ntok hold whatever LDS held: they only reach accumulator columns
                // that are never stored, and an unconditional 16-byte read stays one instruction
                const uint4 bb = *reinterpret_cast<const uint4 *>(&slab[i][32 * q + 8 * kq]);
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(aa), as_bf16x8(bb), acc, 0, 0, 0);
            }
        }
        __atomic_signal_fence(__ATOMIC_SEQ_CST);
        __builtin_amdgcn_wave_barrier();
        __atomic_signal_fence(__ATOMIC_SEQ_CST);
    }
    accs[ro] = acc;
    }
    // (the x region is this wavefront's own, and its LDS operations complete in order)
#pragma unroll
    for (int ro = 0; ro < ROLES; ++ro) red(wave + WAVES * ro)[lane] = accs[ro];
    __syncthreads();
    // the first wavefront of every slice adds the slice's four tiles (in wavefront order), then
    // wavefront 0 adds the slices (in slice order): the order of the k-slice plan, two short steps
    // instead of sixteen reads by one wavefront
#pragma unroll
    for (int ro = 0; ro < ROLES; ++ro) {
        const int role = wave + WAVES * ro;
        if (wq == 0 && (role >> 2) < n_slices) {
            f32x4 ts = red(role)[lane];
            ts += red(role + 1)[lane];
            ts += red(role + 2)[lane];
            ts += red(role + 3)[lane];
            red(role)[lane] = ts;
        }
    }
    __syncthreads();
    if (wave == 0) {
        f32x4 t = red(0)[lane];
#pragma unroll
        for (int sl = 1; sl < kMaxSlices; ++sl)
            if (sl < n_slices) t += red(4 * sl)[lane];
        // register r of lane (i, kq) is rank row 4*kq + r of the block for token i
        if (x_ok && 4 * kq < pn) {
            const int64_t off = u.v_off + (int64_t)i * u.r8 + 4 * kq;
            if (v_hi) {
                uint2 h, l;
                h.x = pack_bf16_rne(t[0], t[1]);
                h.y = pack_bf16_rne(t[2], t[3]);
                l.x = pack_bf16_rne(t[0] - bf16_bits_to_f32(h.x & 0xFFFFu), t[1] - __uint_as_float(h.x & 0xFFFF0000u));
                l.y = pack_bf16_rne(t[2] - bf16_bits_to_f32(h.y & 0xFFFFu), t[3] - __uint_as_float(h.y & 0xFFFF0000u));
                *reinterpret_cast<uint2 *>(v_hi + off) = h;
                *reinterpret_cast<uint2 *>(v_lo + off) = l;
            } else {
                *reinterpret_cast<f32x4 *>(v_f32 + off) = t;
            }
        }
        LORA_CLOCK(4);
    }
}

// ------------------------------------------------------------------------------------------------
// shrink of token-heavy groups (prefill) up to rank 64: one unit = (group, 32 tokens, all rank
// rows, all of k).  The four wavefronts split k into quarters; each streams its quarter of the
// tokens' x rows exactly once.  x comes from HBM with coalesced loads (a wavefront load covers 256
// bytes of each of 4 tokens), XD passes of 128 k ahead, and is turned into MFMA operand order through
// an LDS region private to the wavefront, so no work-group barrier sits in the k loop.  (Loading the
// token operand straight from memory, 16 rows x 64 bytes per load, costs the address path 3.7 times
// as much per byte.)  The rows of A^T come from L2 (every token tile of the group re-reads them),
// requested WD k steps ahead because a step of a low rank is far shorter than a round trip to L2,
// and are shared by the TB token blocks in registers.  The four partial tiles are summed through
// LDS (re-using the x regions) in a fixed order (3+1, 2+0, then 1+0) and v leaves complete: as bf16
// hi + lo for the expand, or as fp32.  JB = 16-row blocks of A^T (1, 2, 4).
// ------------------------------------------------------------------------------------------------
constexpr int kPfTokens = 32;
constexpr int kPfPassK = 128;                 // k per pass of a wavefront
constexpr int kPfRow = kPfPassK + 8;          // LDS row length in bf16, padded by 16 bytes
constexpr int kPfSlab = kPfTokens * kPfRow * 2;
constexpr int kPrefillLds = 4 * kPfSlab;

// lane (n, kq) holds v[token][j .. j+3] of a tile; `at` is the element's index in v
static __device__ __forceinline__ void store_v4(f32x4 f, int64_t at, uint16_t *__restrict__ v_hi,
                                                uint16_t *__restrict__ v_lo, float *__restrict__ v_f32,
                                                int n_slices, int64_t slice_stride)
{
    if (v_f32) {
        *reinterpret_cast<f32x4 *>(v_f32 + at) = f;
        for (int sl = 1; sl < n_slices; ++sl)
            *reinterpret_cast<f32x4 *>(v_f32 + (int64_t)sl * slice_stride + at) = f32x4{0.f, 0.f, 0.f, 0.f};
    } else {
        uint2 h, l;
        h.x = pack_bf16_rne(f[0], f[1]);
        h.y = pack_bf16_rne(f[2], f[3]);
        l.x = pack_bf16_rne(f[0] - bf16_bits_to_f32(h.x & 0xFFFFu), f[1] - __uint_as_float(h.x & 0xFFFF0000u));
        l.y = pack_bf16_rne(f[2] - bf16_bits_to_f32(h.y & 0xFFFFu), f[3] - __uint_as_float(h.y & 0xFFFF0000u));
        *reinterpret_cast<uint2 *>(v_hi + at) = h;
        *reinterpret_cast<uint2 *>(v_lo + at) = l;
    }
}

template <int JB, int TB, int WD, int XD = 1>
static __device__ __forceinline__ void shrink_prefill_ksplit(const Unit &u, const int32_t *__restrict__ perm,
                                                             const uint16_t *__restrict__ arena,
                                                             const uint16_t *__restrict__ x, int64_t ldx, int in,
                                                             uint16_t *__restrict__ v_hi,
                                                             uint16_t *__restrict__ v_lo, float *__restrict__ v_f32,
                                                             int n_slices, int64_t slice_stride, char *lds,
                                                             float *__restrict__ parts, const Sync &sy)
{
    constexpr int NT = JB * TB;
    constexpr int NL = 4 * TB;  // x loads of a wavefront per pass: 4 tokens each
    static_assert(16 * TB <= kPfTokens, "tokens of a unit");
    static_assert(2 * NT * 64 * 16 <= kPrefillLds, "the partial tiles of two wavefronts fit the LDS");
    static_assert(WD == 1 || WD == 2 || WD == 4, "the weight ring must divide the 4 steps of a pass");
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    uint16_t(*slab)[kPfRow] = reinterpret_cast<uint16_t(*)[kPfRow]>(lds + wave * kPfSlab);
    f32x4(*red)[NT][64] = reinterpret_cast<f32x4(*)[NT][64]>(lds);  // re-uses the x regions after the k loop
    const int n = lane & 15;
    const int kq = lane >> 4;
    const int r8 = u.r8;
    const int ntok = u.ntok;

    // staging: load t of a pass takes tokens 4t .. 4t+3, this lane token 4t + kq, 16-byte chunk n
    const uint16_t *xrow[NL];
#pragma unroll
    for (int t = 0; t < NL; ++t) {
        const int tok = min(4 * t + kq, ntok - 1);
        xrow[t] = x + (int64_t)perm[u.perm_off + tok] * ldx;
    }
    // The caller picks JB from the rank; telling the compiler so removes the branches around the row
    // blocks that always exist (with a branch per block the same loop ran 2.4 times slower).
    __builtin_assume(r8 <= 16 * JB && (JB == 1 ? r8 >= 8 : r8 > 8 * JB));
    const uint16_t *wbase = arena + u.w_off;
    int woff[JB];  // element offset of this lane's 16-byte piece in k step 0 of row block jb
    int wh[JB];    // rows in block jb (16, or 8 for the last block of a padded rank that is 8 mod 16)
    // The loop below has no branch: a block beyond the padded rank (ranks 33..48 of the bucket up to 64) is
    // worked as a copy of the last block that exists, and its sums are never stored.
    static_assert(JB <= 4, "ranks above 64 take the row-split body");
    const int nblk = (r8 + 15) >> 4;
#pragma unroll
    for (int jb = 0; jb < JB; ++jb) {
        const int jbc = min(jb, nblk - 1);
        const int h = min(16, r8 - 16 * jbc);
        wh[jb] = h > 0 ? h : 16;
        // lanes n >= 8 of an 8-row block read the piece of row n - 8: they only reach accumulator rows
        // beyond the padded rank, which are never stored
        woff[jb] = 16 * jbc * in + (kq * wh[jb] + (n & (wh[jb] - 1))) * 8;
    }

    f32x4 acc[JB][TB];
#pragma unroll
    for (int jb = 0; jb < JB; ++jb)
#pragma unroll
        for (int tb = 0; tb < TB; ++tb) acc[jb][tb] = f32x4{0.f, 0.f, 0.f, 0.f};

    // this wavefront's quarter of the unit's k range: all of k, or (in launches of few units, which
    // last as long as a unit's walk through k) k-slice u.ks of u.sync_n, multiples of 128 long
    const int n_ks = u.sync_n > 1 ? u.sync_n : 1;
    const int ks_len = n_ks > 1 ? ((in / n_ks + 127) / 128) * 128 : in;
    const int ks_beg = min(in, u.ks * ks_len);
    const int ks_end = min(in, ks_beg + ks_len);
    const int kquarter = ((ks_end - ks_beg + 3) / 4 + 31) & ~31;
    const int kbeg = ks_beg + wave * kquarter;
    const int kend = min(ks_end, kbeg + kquarter);

    {
        // Loads without conditions (rows of tokens beyond ntok are the last token's, see xrow; a chunk beyond
        // the row is fetched from the row's last chunk and a k step beyond the row from its last step; none
        // of them enters an MFMA whose sums are stored): with a branch around a load the compiler no
        // longer counts the loads in flight and waits for all of them at every wait, the x of the passes
        // ahead included, so that every pass of 128 of k took a whole trip to memory.
        const int npass = kend > kbeg ? (kend - kbeg + kPfPassK - 1) / kPfPassK : 0;
        const int nfull = kend > kbeg ? (kend - kbeg) / kPfPassK : 0;
        auto x_all = [&](int k0, uint4(&xq)[NL]) __attribute__((always_inline)) {
            const int kx = min(k0 + 8 * n, in - 8);
#pragma unroll
            for (int t = 0; t < NL; ++t) xq[t] = ld16_stream(xrow[t] + kx);
        };
        auto w_step = [&](int k, int jb) __attribute__((always_inline)) {
            return ld16(wbase + woff[jb] + (int64_t)min(k, in - 32) * wh[jb]);
        };
        auto stage = [&](const uint4(&xq)[NL]) __attribute__((always_inline)) {
#pragma unroll
            for (int t = 0; t < NL; ++t) *reinterpret_cast<uint4 *>(&slab[4 * t + kq][8 * n]) = xq[t];
        };
        auto k_step = [&](int d, const uint4(&wd)[JB]) __attribute__((always_inline)) {
            bf16x8 xo[TB];
#pragma unroll
            for (int tb = 0; tb < TB; ++tb)
                xo[tb] = as_bf16x8(*reinterpret_cast<const uint4 *>(&slab[16 * tb + n][32 * d + 8 * kq]));
#pragma unroll
            for (int jb = 0; jb < JB; ++jb) {
                const bf16x8 ww = as_bf16x8(wd[jb]);
#pragma unroll
                for (int tb = 0; tb < TB; ++tb)
                    acc[jb][tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ww, xo[tb], acc[jb][tb], 0, 0, 0);
            }
        };
        auto wave_sync = [&]() __attribute__((always_inline)) {
            // the region is private to this wavefront and LDS operations of a wavefront complete in order
            __atomic_signal_fence(__ATOMIC_SEQ_CST);
            __builtin_amdgcn_wave_barrier();
            __atomic_signal_fence(__ATOMIC_SEQ_CST);
        };
        // XD passes of x and WD k steps of A^T are in flight per wavefront (registers)
        uint4 xq[XD][NL], w[WD][JB];
#pragma unroll
        for (int q = 0; q < XD; ++q) x_all(kbeg + min(q, max(npass - 1, 0)) * kPfPassK, xq[q]);
#pragma unroll
        for (int d = 0; d < WD; ++d)
#pragma unroll
            for (int jb = 0; jb < JB; ++jb) w[d][jb] = w_step(kbeg + 32 * d, jb);
        int i0 = 0;
        for (; i0 + 2 * XD <= nfull; i0 += XD) {
#pragma unroll
            for (int q = 0; q < XD; ++q) {
                const int k0 = kbeg + (i0 + q) * kPfPassK;
                stage(xq[q]);
                x_all(k0 + XD * kPfPassK, xq[q]);
                wave_sync();
#pragma unroll
                for (int d = 0; d < kPfPassK / 32; ++d) {
                    k_step(d, w[d % WD]);
#pragma unroll
                    for (int jb = 0; jb < JB; ++jb) w[d % WD][jb] = w_step(k0 + 32 * (d + WD), jb);
                }
                wave_sync();
            }
        }
        // the last passes (fewer than 2 XD full ones and maybe a shorter one): the same under conditions
        for (; i0 < npass; i0 += XD) {
#pragma unroll
        for (int q = 0; q < XD; ++q) {
            const int i = i0 + q;
            if (i < npass) {
                const int k0 = kbeg + i * kPfPassK;
                stage(xq[q]);
                if (i + XD < npass) x_all(k0 + XD * kPfPassK, xq[q]);
                wave_sync();
#pragma unroll
                for (int d = 0; d < kPfPassK / 32; ++d) {
                    const int k = k0 + 32 * d;
                    if (k < kend) {
                        k_step(d, w[d % WD]);
                        if (k + 32 * WD < kend) {
#pragma unroll
                            for (int jb = 0; jb < JB; ++jb) w[d % WD][jb] = w_step(k + 32 * WD, jb);
                        }
                    }
                }
                wave_sync();
            }
        }
        }
    }

    // sum the four k-quarters: (wave 2 -> 0, wave 3 -> 1), then (wave 1 -> 0)
    __syncthreads();  // every wavefront has finished with its x region
    if (wave >= 2) {
#pragma unroll
        for (int jb = 0; jb < JB; ++jb)
#pragma unroll
            for (int tb = 0; tb < TB; ++tb) red[wave - 2][jb * TB + tb][lane] = acc[jb][tb];
    }
    __syncthreads();
    if (wave < 2) {
#pragma unroll
        for (int jb = 0; jb < JB; ++jb)
#pragma unroll
            for (int tb = 0; tb < TB; ++tb) acc[jb][tb] += red[wave][jb * TB + tb][lane];
    }
    __syncthreads();
    if (wave == 1) {
#pragma unroll
        for (int jb = 0; jb < JB; ++jb)
#pragma unroll
            for (int tb = 0; tb < TB; ++tb) red[0][jb * TB + tb][lane] = acc[jb][tb];
    }
    __syncthreads();
    if (wave != 0) return;

    // lane (n, kq) holds, for token block tb and row block jb, v[token n][16*jb + 4*kq + e]
    if (n_ks == 1) {
#pragma unroll
        for (int tb = 0; tb < TB; ++tb) {
            if (16 * tb + n >= ntok) continue;
            const int64_t row = u.v_off + (int64_t)(16 * tb + n) * r8;
#pragma unroll
            for (int jb = 0; jb < JB; ++jb) {
                const int j = 16 * jb + 4 * kq;
                if (j < r8)
                    store_v4(acc[jb][tb] + red[0][jb * TB + tb][lane], row + j, v_hi, v_lo, v_f32, n_slices,
                             slice_stride);
            }
        }
        return;
    }
    // A k-slice of the unit's tokens: the sums go to slice u.ks of the fp32 partial sums.  Stand-alone
    // shrink (v_f32): the caller adds the slices up afterwards, so slice 0's unit clears the slices
    // this group does not use.  Apply: stores that go through to memory, then the tile's counter; the
    // unit that completes the tile adds the slices in slice order and leaves v as bf16 hi + lo.
    float *dst = v_f32 ? v_f32 : parts;
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) {
        if (16 * tb + n >= ntok) continue;
        const int64_t row = u.v_off + (int64_t)(16 * tb + n) * r8;
#pragma unroll
        for (int jb = 0; jb < JB; ++jb) {
            const int j = 16 * jb + 4 * kq;
            if (j >= r8) continue;
            const f32x4 f = acc[jb][tb] + red[0][jb * TB + tb][lane];
            if (v_f32) {
                *reinterpret_cast<f32x4 *>(dst + (int64_t)u.ks * slice_stride + row + j) = f;
                if (u.ks == 0)
                    for (int sl = n_ks; sl < n_slices; ++sl)
                        *reinterpret_cast<f32x4 *>(dst + (int64_t)sl * slice_stride + row + j) =
                            f32x4{0.f, 0.f, 0.f, 0.f};
            } else {
                st_through_f32x4(dst + (int64_t)u.ks * slice_stride + row + j, f);
            }
        }
    }
    if (v_f32) return;
    stores_done();
    unsigned old = 0;
    if (lane == 0) old = atomicAdd(sy.counters + u.sync_idx, 1u);
    old = __builtin_amdgcn_readfirstlane(old);
    __atomic_signal_fence(__ATOMIC_SEQ_CST);  // the loads of the slices stay behind the arrival
    if (old + 1u == (unsigned)n_ks) {
        if (lane == 0) atomicExch(sy.counters + u.sync_idx, 0u);  // back to zero for the next launch
        const int tasks = ntok * (u.r8 >> 3);
        for (int task = lane; task < tasks; task += 64) {
            f32x4 f0, f1;
            sum_slices(parts + u.v_off + 8 * task, n_ks, slice_stride, f0, f1);
            uint4 ph, pl;
            split_bf16(f0, f1, ph, pl);
            st_through_u16x8(v_hi + u.v_off + 8 * task, ph);
            st_through_u16x8(v_lo + u.v_off + 8 * task, pl);
        }
    }
}

// Token-heavy units above rank 64: 16 * TB tokens, all rank rows, all of k or a slice of it.  Here the
// four wavefronts split the rank rows (JBW blocks of 16 each) instead of k: every 16-byte piece of
// A^T is then loaded once per work group, straight into the registers of the one wavefront that owns
// its rows, and x, which all four need, is staged once per work group in LDS (two buffers of 128 of k,
// one barrier per pass).  With k split over the wavefronts as above, a unit of 32 tokens loads all of
// A^T for 32 tokens' worth of x: at rank 128 four times the bytes of x, which made the compute units'
// vector caches, not memory, the bound (uniform rank 128 on cfg2's routing: 78 us against 35 us at
// rank 8; 62 us with this body).  No sums cross wavefronts: each stores the rows of v it owns.  (Up to
// rank 64 the k-split body of 32 tokens stayed as fast or faster: 50 us at uniform rank 64 either way.
// Ranks 129..192 take three row blocks per wavefront and 64 tokens, ranks 193..256 four and 32 tokens, the
// accumulators of 64 not fitting the registers: against units of 16 tokens with k split, the shrink
// launch at uniform rank 160 / 192 / 256 went from 105 / 121 / 156 us to 78 / 86 / 112.)
template <int JBW, int TB, int PD, int WP>
static __device__ __forceinline__ void shrink_prefill_rowsplit(const Unit &u, const int32_t *__restrict__ perm,
                                                               const uint16_t *__restrict__ arena,
                                                               const uint16_t *__restrict__ x, int64_t ldx, int in,
                                                               uint16_t *__restrict__ v_hi,
                                                               uint16_t *__restrict__ v_lo, float *__restrict__ v_f32,
                                                               int n_slices, int64_t slice_stride, char *lds,
                                                               float *__restrict__ parts, const Sync &sy)
{
    constexpr int TOK = 16 * TB;
    constexpr int SP = kPfPassK / 32;  // k steps of a pass
    static_assert(PD % 2 == 0 && PD % WP == 0, "the rings are indexed by the pass's place in a round of PD");
    static_assert(2 * TOK * kPfRow * 2 <= kPrefillLds, "two x buffers fit the LDS");
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    uint16_t(*buf)[kPfRow] = reinterpret_cast<uint16_t(*)[kPfRow]>(lds);  // [2 * TOK] rows
    const int n = lane & 15;
    const int kq = lane >> 4;
    const int r8 = u.r8;
    const int ntok = u.ntok;

    // staging: thread (xr, xc) copies 16-byte chunk xc of tokens xr, xr + 16, ...
    const int xr = threadIdx.x >> 4, xc = threadIdx.x & 15;
    const uint16_t *xrow[TB];
#pragma unroll
    for (int i = 0; i < TB; ++i) xrow[i] = x + (int64_t)perm[u.perm_off + min(xr + 16 * i, ntok - 1)] * ldx;

    // A wavefront whose row blocks lie beyond the padded rank (ranks that are not multiples of 64) works on
    // the last block that exists instead: its sums are never stored, and the loop needs no branch for it.
    const uint16_t *wbase = arena + u.w_off;
    const int nblk = (r8 + 15) >> 4;
    int woff[JBW], wh[JBW];
#pragma unroll
    for (int j = 0; j < JBW; ++j) {
        const int jb = min(wave * JBW + j, nblk - 1);
        const int h = min(16, r8 - 16 * jb);
        wh[j] = h;
        // lanes n >= 8 of an 8-row block read the piece of row n - 8: they only reach accumulator rows
        // beyond the padded rank, which are never stored
        woff[j] = 16 * jb * in + (kq * h + (n & (h - 1))) * 8;
    }

    f32x4 acc[JBW][TB];
#pragma unroll
    for (int j = 0; j < JBW; ++j)
#pragma unroll
        for (int tb = 0; tb < TB; ++tb) acc[j][tb] = f32x4{0.f, 0.f, 0.f, 0.f};

    const int n_ks = u.sync_n > 1 ? u.sync_n : 1;
    const int ks_len = n_ks > 1 ? ((in / n_ks + 127) / 128) * 128 : in;
    const int kbeg = min(in, u.ks * ks_len);
    const int kend = min(in, kbeg + ks_len);
    const int npass = (kend - kbeg + kPfPassK - 1) / kPfPassK;
    const int nfull = (kend - kbeg) / kPfPassK;  // passes that hold 128 of k (in is a multiple of 64: the last may hold 64)

    // Loads without conditions (rows of tokens beyond ntok are the last token's, see xrow; a chunk beyond
    // the row is fetched from the row's last chunk and a k step beyond kend from the last step, neither
    // enters an MFMA): with a branch around a load the compiler no longer counts the loads in flight and
    // waits for all of them, the ones requested for later passes included, at every wait.
    auto x_pass = [&](int k0, uint4(&xs)[TB]) __attribute__((always_inline)) {
        const int kx = min(k0 + 8 * xc, in - 8);
#pragma unroll
        for (int i = 0; i < TB; ++i) xs[i] = ld16_stream(xrow[i] + kx);
    };
    auto w_step = [&](int k, int j) __attribute__((always_inline)) {
        return ld16(wbase + woff[j] + (int64_t)min(k, in - 32) * wh[j]);
    };
    auto stage = [&](int base, const uint4(&xs)[TB]) __attribute__((always_inline)) {
#pragma unroll
        for (int t = 0; t < TB; ++t) *reinterpret_cast<uint4 *>(&buf[base + xr + 16 * t][8 * xc]) = xs[t];
    };
    // one 32-wide k step of the pass staged at `base`: rows of tokens beyond ntok hold the last token's x
    // and only reach accumulator columns that are never stored
    auto k_step = [&](int base, int d, const uint4(&ws)[JBW]) __attribute__((always_inline)) {
        bf16x8 xo[TB];
#pragma unroll
        for (int tb = 0; tb < TB; ++tb)
            xo[tb] = as_bf16x8(*reinterpret_cast<const uint4 *>(&buf[base + 16 * tb + n][32 * d + 8 * kq]));
#pragma unroll
        for (int j = 0; j < JBW; ++j) {
            const bf16x8 ww = as_bf16x8(ws[j]);
#pragma unroll
            for (int tb = 0; tb < TB; ++tb)
                acc[j][tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ww, xo[tb], acc[j][tb], 0, 0, 0);
        }
    };

    // PD passes of x and WP passes of A^T are in flight per wavefront (registers).  The steady state has
    // no branch: pass i stages its x, asks for the x of pass i + PD, and after each k step for the rows of
    // A^T of the same step of pass i + WP.  One barrier per pass: the buffer a pass writes was last read
    // two passes ago, and every wavefront has passed the previous pass's barrier since those reads.
    uint4 xs[PD][TB], w[WP][SP][JBW];
#pragma unroll
    for (int q = 0; q < PD; ++q) {
        x_pass(kbeg + min(q, max(npass - 1, 0)) * kPfPassK, xs[q]);
        if (q < WP) {
#pragma unroll
            for (int d = 0; d < SP; ++d)
#pragma unroll
                for (int j = 0; j < JBW; ++j) w[q][d][j] = w_step(kbeg + q * kPfPassK + 32 * d, j);
        }
    }
#ifdef LORA_WG_CLOCKS
    unsigned long long c_wait = 0;  // from the top of a pass to the barrier's exit, summed over the passes
#endif
    int i0 = 0;
    for (; i0 + 2 * PD <= nfull; i0 += PD) {
#pragma unroll
        for (int q = 0; q < PD; ++q) {
            const int k0 = kbeg + (i0 + q) * kPfPassK;
            const int base = (q & 1) * TOK;
#ifdef LORA_WG_CLOCKS
            const unsigned long long c_top = wall_clock64();
#endif
            stage(base, xs[q]);
            x_pass(k0 + PD * kPfPassK, xs[q]);
            __syncthreads();
#ifdef LORA_WG_CLOCKS
            c_wait += wall_clock64() - c_top;
#endif
#pragma unroll
            for (int d = 0; d < SP; ++d) {
                k_step(base, d, w[q % WP][d]);
#pragma unroll
                for (int j = 0; j < JBW; ++j) w[q % WP][d][j] = w_step(k0 + WP * kPfPassK + 32 * d, j);
            }
        }
    }
    // the last passes (fewer than 2 PD, the last maybe 64 of k): the same, with every request and every k
    // step under its condition
#pragma unroll
    for (int q = 0; q < 2 * PD; ++q) {
        const int i = i0 + q;
        if (i < npass) {
            const int k0 = kbeg + i * kPfPassK;
            const int base = (q & 1) * TOK;
            stage(base, xs[q % PD]);
            if (i + PD < npass) x_pass(k0 + PD * kPfPassK, xs[q % PD]);
            __syncthreads();
#pragma unroll
            for (int d = 0; d < SP; ++d) {
                if (k0 + 32 * d < kend) k_step(base, d, w[q % WP][d]);
                if (i + WP < npass) {
#pragma unroll
                    for (int j = 0; j < JBW; ++j) w[q % WP][d][j] = w_step(k0 + WP * kPfPassK + 32 * d, j);
                }
            }
        }
    }
#ifdef LORA_WG_CLOCKS
    if (g_clock_buf && threadIdx.x == 0 && blockIdx.x < g_clock_slots) g_clock_buf[(size_t)blockIdx.x * 8 + 1] = c_wait;
    LORA_CLOCK(2);
#endif
    // lane (n, kq) holds, for token block tb and its row block j, v[token 16 tb + n][16 jb + 4 kq + e]
    if (n_ks == 1) {
#pragma unroll
        for (int tb = 0; tb < TB; ++tb) {
            if (16 * tb + n >= ntok) continue;
            const int64_t row = u.v_off + (int64_t)(16 * tb + n) * r8;
#pragma unroll
            for (int j = 0; j < JBW; ++j) {
                const int jr = 16 * (wave * JBW + j) + 4 * kq;
                if (jr < r8) store_v4(acc[j][tb], row + jr, v_hi, v_lo, v_f32, n_slices, slice_stride);
            }
        }
        return;
    }
    // A k-slice of the unit's tokens, as in the body above: the sums go to slice u.ks of the fp32
    // partial sums; the unit that completes the tile adds the slices in slice order.
    float *dst = v_f32 ? v_f32 : parts;
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) {
        if (16 * tb + n >= ntok) continue;
        const int64_t row = u.v_off + (int64_t)(16 * tb + n) * r8;
#pragma unroll
        for (int j = 0; j < JBW; ++j) {
            const int jr = 16 * (wave * JBW + j) + 4 * kq;
            if (jr >= r8) continue;
            if (v_f32) {
                *reinterpret_cast<f32x4 *>(dst + (int64_t)u.ks * slice_stride + row + jr) = acc[j][tb];
                if (u.ks == 0)
                    for (int sl = n_ks; sl < n_slices; ++sl)
                        *reinterpret_cast<f32x4 *>(dst + (int64_t)sl * slice_stride + row + jr) =
                            f32x4{0.f, 0.f, 0.f, 0.f};
            } else {
                st_through_f32x4(dst + (int64_t)u.ks * slice_stride + row + jr, acc[j][tb]);
            }
        }
    }
    if (v_f32) return;
    stores_done();
    __syncthreads();  // every wavefront's partial sums are out (and nobody reads the x buffers any more)
    unsigned *arrived = reinterpret_cast<unsigned *>(lds);
    if (threadIdx.x == 0) *arrived = atomicAdd(sy.counters + u.sync_idx, 1u);
    __syncthreads();
    const unsigned old = *arrived;
    __atomic_signal_fence(__ATOMIC_SEQ_CST);  // the loads of the slices stay behind the arrival
    if (old + 1u == (unsigned)n_ks) {
        if (threadIdx.x == 0) atomicExch(sy.counters + u.sync_idx, 0u);  // back to zero for the next launch
        const int tasks = ntok * (r8 >> 3);
        for (int task = threadIdx.x; task < tasks; task += kThreads) {
            f32x4 f0, f1;
            sum_slices(parts + u.v_off + 8 * task, n_ks, slice_stride, f0, f1);
            uint4 ph, pl;
            split_bf16(f0, f1, ph, pl);
            st_through_u16x8(v_hi + u.v_off + 8 * task, ph);
            st_through_u16x8(v_lo + u.v_off + 8 * task, pl);
        }
    }
}

// One wavefront copies 1 KB from memory into LDS without passing through registers: lane l's 16 bytes
// at gptr (per lane) land at lds_piece + 16*l (lds_piece wave-uniform).  Written as an instruction the
// compiler does not look into: for its own form of this load it waits until the copy has landed
// before the wavefront may issue anything else that touches LDS or the registers involved, which
// leaves nothing of the overlap the copy exists for.  The caller waits (vmcnt(0)) and synchronises
// the work group before anyone reads the destination.
static __device__ __forceinline__ void dma16_to_lds(const uint4 *gptr, const uint4 *lds_piece)
{
    const uint32_t lds_addr = __builtin_amdgcn_readfirstlane(
        (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) void *)lds_piece);
    // M0 carries the LDS address of the piece; its old value is put back, so the register the
    // compiler reserves for itself is unchanged after the statement
    uint32_t saved_m0;
    asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off\n\t"
                 "s_mov_b32 m0, %0"
                 : "=&s"(saved_m0)
                 : "v"(gptr), "s"(lds_addr)
                 : "memory");
}

// Picks the body by the unit's rank rows.  ANY = false: the launch holds no unit above rank 64 and the
// bodies fit 128 registers (four work groups per compute unit).  ANY = true: any rank (two work groups
// per compute unit); ranks above 64 take the row-split body, with 64 tokens up to rank 192 and 32 above.
template <bool ANY>
static __device__ __forceinline__ void prefill_dispatch(const Unit &u, const int32_t *__restrict__ perm,
                                                        const uint16_t *__restrict__ arena,
                                                        const uint16_t *__restrict__ x, int64_t ldx, int in,
                                                        uint16_t *__restrict__ v_hi, uint16_t *__restrict__ v_lo,
                                                        float *__restrict__ v_f32, int n_slices,
                                                        int64_t slice_stride, char *lds,
                                                        float *__restrict__ parts, const Sync &sy)
{
    const int r8 = u.r8;
    // (three in flight for ranks up to 32: cfg2 4096 -> 4096 shrink 48.3 against 43.9 us)
    constexpr int XD = ANY ? 2 : 1;  // passes of x in flight per wavefront: two where two work groups share a compute unit
    if (r8 <= 16)
        shrink_prefill_ksplit<1, 2, 4, XD>(u, perm, arena, x, ldx, in, v_hi, v_lo, v_f32, n_slices, slice_stride, lds, parts, sy);
    else if (r8 <= 32)
        shrink_prefill_ksplit<2, 2, 4, XD>(u, perm, arena, x, ldx, in, v_hi, v_lo, v_f32, n_slices, slice_stride, lds, parts, sy);
    else if (!ANY)  // the launcher takes this form only for batches whose token-heavy units are all up to rank 64
        shrink_prefill_ksplit<4, 2, 1>(u, perm, arena, x, ldx, in, v_hi, v_lo, v_f32, n_slices, slice_stride, lds, parts, sy);
    else if (r8 <= 64)
        shrink_prefill_ksplit<4, 2, 4, XD>(u, perm, arena, x, ldx, in, v_hi, v_lo, v_f32, n_slices, slice_stride, lds, parts, sy);
    else if constexpr (ANY) {
        if (r8 <= 128)
            shrink_prefill_rowsplit<2, 4, 2, 1>(u, perm, arena, x, ldx, in, v_hi, v_lo, v_f32, n_slices, slice_stride, lds, parts, sy);
        else if (r8 <= 192)
            shrink_prefill_rowsplit<3, 4, 2, 1>(u, perm, arena, x, ldx, in, v_hi, v_lo, v_f32, n_slices, slice_stride, lds, parts, sy);
        else  // 32 tokens: the 16 accumulator tiles of 64 tokens x 64 rank rows per wavefront do not fit the registers
            shrink_prefill_rowsplit<4, 2, 2, 1>(u, perm, arena, x, ldx, in, v_hi, v_lo, v_f32, n_slices, slice_stride, lds, parts, sy);
    }
}

__global__ __launch_bounds__(kThreads, 4) void k_shrink_prefill(const Unit *__restrict__ units,
                                                                const int32_t *__restrict__ perm,
                                                                const uint16_t *__restrict__ arena,
                                                                const uint16_t *__restrict__ x, int64_t ldx, int in,
                                                                uint16_t *__restrict__ v_hi,
                                                                uint16_t *__restrict__ v_lo,
                                                                float *__restrict__ v_f32, int n_slices,
                                                                int64_t slice_stride, float *__restrict__ parts, Sync sy)
{
    __shared__ __attribute__((aligned(16))) char lds[kPrefillLds];
    if (units[blockIdx.x].ntok <= 0) return;  // a place the planner filled so that every XCD's list has the same length
    LORA_CLOCK(0);
    prefill_dispatch<false>(units[blockIdx.x], perm, arena, x, ldx, in, v_hi, v_lo, v_f32, n_slices, slice_stride,
                            lds, parts, sy);
    LORA_CLOCK(4);
}

// A batch that has units above rank 64 runs all its token-heavy units here, in one launch: two
// launches one after the other (high ranks here, the rest above) measured slower, the first one
// leaving most of the chip idle.
__global__ __launch_bounds__(kThreads, 2) void k_shrink_prefill_any(const Unit *__restrict__ units,
                                                                    const int32_t *__restrict__ perm,
                                                                    const uint16_t *__restrict__ arena,
                                                                    const uint16_t *__restrict__ x, int64_t ldx,
                                                                    int in, uint16_t *__restrict__ v_hi,
                                                                    uint16_t *__restrict__ v_lo,
                                                                    float *__restrict__ v_f32, int n_slices,
                                                                    int64_t slice_stride, float *__restrict__ parts, Sync sy)
{
    __shared__ __attribute__((aligned(16))) char lds[kPrefillLds];
    if (units[blockIdx.x].ntok <= 0) return;  // a place the planner filled so that every XCD's list has the same length
    LORA_CLOCK(0);
    prefill_dispatch<true>(units[blockIdx.x], perm, arena, x, ldx, in, v_hi, v_lo, v_f32, n_slices, slice_stride,
                           lds, parts, sy);
    LORA_CLOCK(4);
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

// KSTEPS: 32-wide steps that cover the padded rank (1, 2, 4 or 8).  A unit may hold several blocks
// of 16 tokens; the weights of a column pass stay in registers while the token blocks go by.
template <int KSTEPS, bool BIG, bool VF32>
static __device__ __forceinline__ void expand_body(const Unit &u, const int32_t *__restrict__ perm,
                                                   const uint16_t *__restrict__ arena,
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
    const int ntok_all = u.ntok;
    const int ncols = u.pn;
    const uint4 zero = {0u, 0u, 0u, 0u};
    const int my_strip = wave / P;
    const int my_part = wave % P;
    const int32_t *toks = BIG ? perm + u.perm_off : u.tok;

    // epilogue role of this thread: token e_tok of the block, 8 columns starting at 8*e_cg of every strip
    const int e_tok = tid >> 4;
    const int e_cg = tid & 15;
    const float scale = u.scale;
    // The row of y this thread updates in the first block of tokens, fetched before anything else: a
    // wavefront's loads return in request order, so requested behind the weights it would come back
    // with the last of them, and the loads of y (which need it) would only start then, a second trip
    // to memory on the unit's critical path.
    const int64_t first_row = toks[e_tok < min(kTokTile, ntok_all) ? e_tok : 0];
    __builtin_amdgcn_sched_barrier(0);

    int jc[ITEMS];
    bool j_ok[ITEMS];
#pragma unroll
    for (int it = 0; it < ITEMS; ++it) {
        const int j = 32 * (my_part + P * it) + 8 * kq;
        j_ok[it] = j < r8;
        jc[it] = j_ok[it] ? j : 0;
    }
    bool first = true;

    for (int c0 = 0; c0 < ncols; c0 += S * kStrip) {
        const int cs = c0 + my_strip * kStrip;  // this wavefront's strip
        const bool strip_ok = cs < ncols;
        // this lane's piece of sub-block 0, rank piece 0 of the wavefront's strip; sub-block b is
        // 16*r8 elements further, rank piece kp 128 elements further
        const uint16_t *brow = arena + u.w_off + (int64_t)(strip_ok ? cs : 0) * r8 + n * 8;
        // weights: row (column of y) cs + 8*n + b, 16 bytes at jc.  One k step per wavefront: they stay
        // in registers for all token blocks; two (rank > 128): each block re-reads them (L1 / L2 hits).
        uint4 w[8];
        if (ITEMS == 1) {
#pragma unroll
            for (int b = 0; b < 8; ++b) w[b] = ld16_stream(brow + b * 16 * r8 + jc[0] * 16);
            // nothing that needs the row index (a wait for its load) moves up in front of these requests
            __builtin_amdgcn_sched_barrier(0);
        }

        // one block of 16 tokens: this thread's share of y and this wavefront's v operand
        struct Blk {
            uint4 yv[S];
            uint4 vh[ITEMS], vl[ITEMS];
            uint16_t *e_y;
            int ntok;
        };
        auto load_blk = [&](int t0, Blk &bk) __attribute__((always_inline)) {
            bk.ntok = min(kTokTile, ntok_all - t0);
            const bool e_ok = e_tok < bk.ntok;
            const int64_t row = t0 == 0 ? first_row : (int64_t)toks[e_ok ? t0 + e_tok : 0];
            bk.e_y = y + row * ldy + u.p0 + 8 * e_cg;
#pragma unroll
            for (int s = 0; s < S; ++s) {
                // no per-lane condition around the 16-byte load (it would be split into four masked
                // 4-byte loads): threads without a token read the unit's first token's row
                bk.yv[s] = zero;
                if (c0 + s * kStrip < ncols) bk.yv[s] = ld16_stream(bk.e_y + c0 + s * kStrip);
            }
#pragma unroll
            for (int it = 0; it < ITEMS; ++it) {
                const bool ok = (n < bk.ntok) && j_ok[it];
                const int64_t off = u.v_off + (int64_t)(ok ? t0 + n : 0) * r8 + jc[it];
                uint4 ph, pl;
                if (!VF32) {
                    if (!BIG && sy.wait) {  // written earlier in this very launch: read through to memory
                        ph = ld_through_u16x8(sy.v_hi + off);
                        pl = ld_through_u16x8(sy.v_lo + off);
                    } else {
                        ph = ld16(sy.v_hi + off);
                        pl = ld16(sy.v_lo + off);
                    }
                } else {
                    bf16x8 h, l;
                    load_v_operand(v_in + off, ok, n_slices, slice_stride, h, l);
                    ph = __builtin_bit_cast(uint4, h);
                    pl = __builtin_bit_cast(uint4, l);
                }
                bk.vh[it] = ok ? ph : zero;
                bk.vl[it] = ok ? pl : zero;
            }
        };

        if (!BIG && !VF32 && first && sy.counters && sy.wait) wait_for(sy, u.sync_idx);  // weights are in flight
        // all of the unit's y and v go out at once (up to 4 blocks of 16 tokens), so that the HBM
        // latency of y is paid once per column pass, not once per block
        constexpr int NB = BIG ? 4 : 1;
        Blk blk[NB];
#pragma unroll
        for (int ib = 0; ib < NB; ++ib)
            if (ib * kTokTile < ntok_all) load_blk(ib * kTokTile, blk[ib]);
#pragma unroll
        for (int ib = 0; ib < NB; ++ib) {
            if (ib * kTokTile >= ntok_all) break;
            Blk &cur = blk[ib];
            if (!first) __syncthreads();  // the previous block's partial tiles have been consumed
            first = false;
            const int ntok = cur.ntok;
            const bool e_ok = e_tok < ntok;

            f32x4 acc[8];
#pragma unroll
            for (int b = 0; b < 8; ++b) acc[b] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int it = 0; it < ITEMS; ++it) {
                if (ITEMS > 1) {
#pragma unroll
                    for (int b = 0; b < 8; ++b) w[b] = ld16_stream(brow + b * 16 * r8 + jc[it] * 16);
                }
#pragma unroll
                for (int b = 0; b < 8; ++b) {
                    const bf16x8 ww = as_bf16x8(j_ok[it] ? w[b] : zero);
                    acc[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(cur.vh[it]), ww, acc[b], 0, 0, 0);
                    acc[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(cur.vl[it]), ww, acc[b], 0, 0, 0);
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
                        const uint4 yy = cur.yv[s];
                        uint4 o;
                        o.x = pack_bf16_rne(bf16_bits_to_f32(yy.x & 0xFFFFu) + scale * d0[0],
                                            __uint_as_float(yy.x & 0xFFFF0000u) + scale * d0[1]);
                        o.y = pack_bf16_rne(bf16_bits_to_f32(yy.y & 0xFFFFu) + scale * d0[2],
                                            __uint_as_float(yy.y & 0xFFFF0000u) + scale * d0[3]);
                        o.z = pack_bf16_rne(bf16_bits_to_f32(yy.z & 0xFFFFu) + scale * d1[0],
                                            __uint_as_float(yy.z & 0xFFFF0000u) + scale * d1[1]);
                        o.w = pack_bf16_rne(bf16_bits_to_f32(yy.w & 0xFFFFu) + scale * d1[2],
                                            __uint_as_float(yy.w & 0xFFFF0000u) + scale * d1[3]);
                        st16_stream(cur.e_y + c0 + s * kStrip, o);
                    }
                }
            }
        }
    }
}

// ------------------------------------------------------------------------------------------------
// expand of token-heavy groups: one unit = (group, up to 64 tokens, a run of 128-column strips).
// Each wavefront owns 16 of the tokens for the whole unit and all of the rank, so nothing is summed
// across wavefronts and there is no barrier per token block: its v operands (bf16 hi + lo, every
// k step) are loaded once and stay in registers; a strip's B^T tile (128 columns x rank, one
// contiguous piece of the pool) is copied into LDS once per work group and read from there by the
// four wavefronts; the MFMA result (token x column, lane n holding 8 consecutive columns of 4
// tokens) goes straight to the y update, 16 bytes per lane, four 256-byte row pieces per store.
// While a strip computes, the next strip's B^T tile and this lane's y pieces are already on their
// way (the tile waits in registers, then goes into the other half of the LDS buffer).
// ------------------------------------------------------------------------------------------------
constexpr int kBigLds = 64 * 1024;

template <int KSTEPS, bool VF32>
static __device__ __forceinline__ void expand_big_body(const Unit &u, const int32_t *__restrict__ perm,
                                                       const uint16_t *__restrict__ arena,
                                                       const float *__restrict__ v_in, int n_slices,
                                                       int64_t slice_stride, uint16_t *__restrict__ y,
                                                       int64_t ldy, char *lds, const Sync &sy)
{
    // the tile of one strip is 128 * r8 * 2 bytes: <= 32 KiB up to rank 128, two buffers of 32 KiB; above,
    // one buffer of 64 KiB, filled between two strips
    static_assert(KSTEPS <= 8, "token-heavy expand units exist up to rank 256");
    constexpr bool DB = KSTEPS <= 4;
    constexpr int WREG = 2 * KSTEPS;  // 16-byte pieces of a tile per thread (256 threads): 128*32*KSTEPS*2 / 4096
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int n = lane & 15;
    const int kq = lane >> 4;
    const int r8 = u.r8;
    const int ntok_all = u.ntok;
    const int ncols = u.pn;
    const uint4 zero = {0u, 0u, 0u, 0u};
    const int32_t *toks = perm + u.perm_off;
    const float scale = u.scale;
    const int tile_pieces = 16 * r8;  // 16-byte pieces in one strip's tile (128 * r8 * 2 / 16)

    // this wavefront's 16 tokens: v operands for every k step
    const int nt = min(kTokTile, ntok_all - kTokTile * wave);  // may be <= 0: the wavefront only helps copying
    uint4 vh[KSTEPS], vl[KSTEPS];
    bool j_ok[KSTEPS];
#pragma unroll
    for (int st = 0; st < KSTEPS; ++st) {
        const int j = 32 * st + 8 * kq;
        j_ok[st] = j < r8;
        const bool ok = (n < nt) && j_ok[st];
        const int64_t off = u.v_off + (int64_t)(ok ? kTokTile * wave + n : 0) * r8 + (j_ok[st] ? j : 0);
        uint4 ph, pl;
        if (!VF32) {
            ph = ld16(sy.v_hi + off);
            pl = ld16(sy.v_lo + off);
        } else {
            bf16x8 h, l;
            load_v_operand(v_in + off, ok, n_slices, slice_stride, h, l);
            ph = __builtin_bit_cast(uint4, h);
            pl = __builtin_bit_cast(uint4, l);
        }
        vh[st] = ok ? ph : zero;
        vl[st] = ok ? pl : zero;
    }
    // the MFMA leaves tokens 4*kq + e (e = 0..3), columns 8*n .. 8*n+7 of the strip in this lane
    uint16_t *yrow[4];
    bool y_ok[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        y_ok[e] = 4 * kq + e < nt;
        yrow[e] = y + (int64_t)toks[y_ok[e] ? kTokTile * wave + 4 * kq + e : 0] * ldy + u.p0 + 8 * n;
    }

    const uint4 *gtile = reinterpret_cast<const uint4 *>(arena + u.w_off);  // strip s starts tile_pieces * s further
    uint4 *ltile = reinterpret_cast<uint4 *>(lds);
    const int nstrips = ncols / kStrip;

    // Copy of strip S_'s tile from the pool into LDS buffer BUF_ with loads that write LDS directly
    // (no registers in between, so the copy runs while the MFMAs of the current strip do): every
    // wavefront moves 1 KB pieces, lane l's 16 bytes landing at the piece's LDS base + 16*l.  The
    // tile is 16*r8 pieces of 16 bytes, a multiple of 64, so a wavefront's piece is whole or absent.
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
#define LORA_DMA_TILE(BUF_, S_)                                                                         \
    _Pragma("unroll") for (int q = 0; q < WREG; ++q) {                                                  \
        const int piece0 = 64 * wave_u + kThreads * q;                                                  \
        if (piece0 < tile_pieces)                                                                       \
            dma16_to_lds(gtile + (int64_t)(S_) * tile_pieces + piece0 + lane, ltile + (BUF_) * 2048 + piece0); \
    }
    // the copies (and everything else this wavefront has in flight) have landed
#define LORA_DMA_WAIT()                       \
    __atomic_signal_fence(__ATOMIC_SEQ_CST);  \
    __builtin_amdgcn_s_waitcnt(kWaitcntVmcnt0); \
    __atomic_signal_fence(__ATOMIC_SEQ_CST);
    uint4 ya[4], yb[4];
    auto fetch_y = [&](int s, uint4 (&yv)[4]) __attribute__((always_inline)) {
#pragma unroll
        // unconditional: rows of absent tokens point at the unit's first token (a per-lane condition
        // around a 16-byte load makes the compiler split it into four masked 4-byte loads)
        for (int e = 0; e < 4; ++e) yv[e] = ld16_stream(yrow[e] + s * kStrip);
    };
    auto compute = [&](int s, int buf, const uint4 (&yv)[4]) __attribute__((always_inline)) {
        if (nt <= 0) return;
        const uint4 *t = ltile + buf * 2048;
        f32x4 acc[8];
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            acc[b] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int st = 0; st < KSTEPS; ++st) {
                if (32 * st < r8) {  // uniform
                    // piece (sub-block b, rank piece 4*st + kq, column slot n).  Lanes whose rank piece
                    // lies beyond the padded rank read piece 0 instead (their v operand is zero): an
                    // unconditional 16-byte read stays one instruction, a conditional one becomes four
                    const uint4 wv = t[(b * (r8 >> 3) + (j_ok[st] ? 4 * st + kq : 0)) * 16 + n];
                    acc[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(vh[st]), as_bf16x8(wv), acc[b], 0, 0, 0);
                    acc[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(vl[st]), as_bf16x8(wv), acc[b], 0, 0, 0);
                }
            }
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (y_ok[e]) {
                const uint4 yy = yv[e];
                uint4 o;
                o.x = pack_bf16_rne(bf16_bits_to_f32(yy.x & 0xFFFFu) + scale * acc[0][e],
                                    __uint_as_float(yy.x & 0xFFFF0000u) + scale * acc[1][e]);
                o.y = pack_bf16_rne(bf16_bits_to_f32(yy.y & 0xFFFFu) + scale * acc[2][e],
                                    __uint_as_float(yy.y & 0xFFFF0000u) + scale * acc[3][e]);
                o.z = pack_bf16_rne(bf16_bits_to_f32(yy.z & 0xFFFFu) + scale * acc[4][e],
                                    __uint_as_float(yy.z & 0xFFFF0000u) + scale * acc[5][e]);
                o.w = pack_bf16_rne(bf16_bits_to_f32(yy.w & 0xFFFFu) + scale * acc[6][e],
                                    __uint_as_float(yy.w & 0xFFFF0000u) + scale * acc[7][e]);
                st16_stream(yrow[e] + s * kStrip, o);
            }
        }
    };

    LORA_DMA_TILE(0, 0)
    fetch_y(0, ya);
    LORA_DMA_WAIT()
    __syncthreads();
    for (int s = 0; s < nstrips; s += 2) {
        // even strips from buffer 0, odd strips from buffer 1 (a single buffer above rank 128)
        if (s + 1 < nstrips) {
            if (DB) { LORA_DMA_TILE(1, s + 1) }
            fetch_y(s + 1, yb);
        }
        compute(s, 0, ya);
        if (s + 1 >= nstrips) break;
        if (!DB) {
            __syncthreads();  // single buffer: everyone has finished reading strip s
            LORA_DMA_TILE(0, s + 1)
        }
        LORA_DMA_WAIT()
        __syncthreads();
        if (s + 2 < nstrips) {
            if (DB) { LORA_DMA_TILE(0, s + 2) }
            fetch_y(s + 2, ya);
        }
        compute(s + 1, DB ? 1 : 0, yb);
        if (s + 2 >= nstrips) break;
        if (!DB) {
            __syncthreads();
            LORA_DMA_TILE(0, s + 2)
        }
        LORA_DMA_WAIT()
        __syncthreads();
    }
#undef LORA_DMA_TILE
#undef LORA_DMA_WAIT
}

template <bool BIG, bool VF32>
static __device__ __forceinline__ void expand_dispatch(const Unit &u, const int32_t *__restrict__ perm,
                                                       const uint16_t *__restrict__ arena,
                                                       const float *__restrict__ v_in, int n_slices,
                                                       int64_t slice_stride, uint16_t *__restrict__ y,
                                                       int64_t ldy, char *lds, const Sync &sy)
{
    const int r8 = u.r8;
    if (BIG) {
        if (r8 <= 32)
            expand_big_body<1, VF32>(u, perm, arena, v_in, n_slices, slice_stride, y, ldy, lds, sy);
        else if (r8 <= 64)
            expand_big_body<2, VF32>(u, perm, arena, v_in, n_slices, slice_stride, y, ldy, lds, sy);
        else if (r8 <= 128)
            expand_big_body<4, VF32>(u, perm, arena, v_in, n_slices, slice_stride, y, ldy, lds, sy);
        else
            expand_big_body<8, VF32>(u, perm, arena, v_in, n_slices, slice_stride, y, ldy, lds, sy);
    } else {
        if (r8 <= 32)
            expand_body<1, false, VF32>(u, perm, arena, v_in, n_slices, slice_stride, y, ldy, lds, sy);
        else if (r8 <= 64)
            expand_body<2, false, VF32>(u, perm, arena, v_in, n_slices, slice_stride, y, ldy, lds, sy);
        else if (r8 <= 128)
            expand_body<4, false, VF32>(u, perm, arena, v_in, n_slices, slice_stride, y, ldy, lds, sy);
        else
            expand_body<8, false, VF32>(u, perm, arena, v_in, n_slices, slice_stride, y, ldy, lds, sy);
    }
}


// ------------------------------------------------------------------------------------------------
// Decode apply in one launch.  A decode co-batch is a few tens of megabytes of adapter weights read
// once: at that size a launch lasts about as long as its first and its last byte take to arrive, and
// two launches pay that twice.  Here one grid of at most one work group (16 wavefronts) per compute
// unit does both halves:
//   * work group b runs shrink unit b exactly as k_shrink_wide does (same tiles, same order of
//     additions, so v and y are bitwise those of the two launches), then each of its four groups of
//     four wavefronts runs expand unit 4b + q as k_expand does.  Empty places in either list (ntok
//     == 0) are skipped.  The expand units' B^T operands and rows of y are requested as soon as the
//     work group's part of v has been stored, so the chip's loads of B^T follow those of A^T without
//     the tail, the pause and the ramp of a launch boundary;
//   * v is handed over inside an XCD.  Each of the chip's XCDs has an L2 of its own, and a store that
//     must reach memory queues behind everything the chip has requested (several microseconds once
//     the loads of B^T are out).  The work groups of a launch go to the XCDs in turn (work group b to
//     the XCD of b mod 8), and the host puts every shrink unit and every expand unit of one (group,
//     token tile) at places of one residue mod 8: v is then written with plain stores into that XCD's
//     L2, the tile's ready counter is bumped by an atomic that the L2 executes, the expand units poll it
//     with a returning atomic (executed by the L2 as well; a plain load could be served by the compute
//     unit's L1) and read v with agent-scope loads, which pass the compute unit's L1 and are served
//     by the L2.  (Not plain loads behind an L1 invalidate: at work-group scope the invalidate does
//     nothing here, and a 128-byte line of v can hold rows of two tiles, so that a unit of the same work
//     group may have fetched the line before this tile's rows were stored; the agent-scope
//     invalidate, which does drop the lines, made the launch 2.6 times as long.)
//     The counters only grow: the target is epoch * sync_n, epoch = such launches the table has seen.
//     Every work group checks that the work groups on its XCD all have its residue (see the start of
//     the kernel); if not it sets bit 1 of the time-out flag: the launch's result is then not valid
//     and lora_segments_check says so.
//   * every work group stores its part of v before its first wait, and the grid fits the chip, so
//     every wait ends; it is bounded all the same (spin_limit polls, then bit 0 of the flag).
// ------------------------------------------------------------------------------------------------
constexpr int kDecodeMaxGrid = 256;  // work groups of the launch at most (one per compute unit)
static_assert(4 * kExpandLds <= kWideWaves * kWideSlab, "the four expand units' partial tiles fit where the x regions were");

// returning atomic OR with 0: the counter's value as the L2 holds it
static __device__ __forceinline__ unsigned l2_counter_value(unsigned *p)
{
    unsigned v;
    const unsigned zero = 0u;
    asm volatile("global_atomic_or %0, %1, %2, off sc0\n\ts_waitcnt vmcnt(0)" : "=v"(v) : "v"(p), "v"(zero) : "memory");
    return v;
}

// atomic add executed by the L2, nothing returned
static __device__ __forceinline__ void l2_counter_add(unsigned *p, unsigned n)
{
    asm volatile("global_atomic_add %0, %1, off" : : "v"(p), "v"(n) : "memory");
}

__global__ __launch_bounds__(kWideThreads) void k_decode_fused(
    const Unit *__restrict__ s_units, int n_s, const Unit *__restrict__ e_units, int n_e,
    const uint16_t *__restrict__ arena, const uint16_t *__restrict__ x, int64_t ldx, int in, int k_slice_len,
    int n_slices, uint16_t *__restrict__ y, int64_t ldy, unsigned xcc_map, Sync sy)
{
    __shared__ __attribute__((aligned(16))) char lds[kWideLds + 64];  // + one flag per group of four wavefronts, 8 words of the XCD check
    const int bid = blockIdx.x;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int slice = wave >> 2;  // shrink: the k-slice this wavefront works on; expand: its group of four
    const int wq = wave & 3;      // its place among the four
    const int i = lane & 15;
    const int kq = lane >> 4;
    const uint4 zero = {0u, 0u, 0u, 0u};
    uint16_t(*slab)[kWideRow] = reinterpret_cast<uint16_t(*)[kWideRow]>(lds + wave * kWideSlab);
    f32x4(*red)[64] = reinterpret_cast<f32x4(*)[64]>(lds + kWideWaves * kWideSlab);
    volatile unsigned *qflag = reinterpret_cast<volatile unsigned *>(lds + kWideLds) + slice;
    if (tid < 4) reinterpret_cast<volatile unsigned *>(lds + kWideLds)[tid] = 0u;
    // the shrink unit's record, one request (load_unit_words)
    const uint32_t s_rec = load_unit_words(s_units + (bid < n_s ? bid : 0));
    // Which XCD do the work groups of each residue run on?  The hardware deals the work groups of a
    // launch to the XCDs in turn, but not every launch starts at the same XCD: all that the hand-over
    // needs is that work groups of one residue mod 8 share an XCD, i.e. that every work group on an XCD
    // finds the same difference d between its place and the XCD's position in the dealing order
    // (xcc_map: 4 bits per XCD number, its position as a probe launch found it).  Each work group
    // leaves (epoch, XCD, d) in a word of its own (a plain store: nothing waits for it); the words
    // alternate between two sets from launch to launch, and the last work group of the following launch
    // (the one with the lightest shrink unit, where a trip to memory in front of the operand loads
    // costs the launch nothing) reads what the finished launch left: two values of d on one XCD mean
    // that its result cannot be trusted (bit 1 of the time-out flag).  The host reads the last launch's
    // set itself.
    // hardware register XCC_ID, bits 3:0
    const unsigned xcc = __builtin_amdgcn_s_getreg(20 | (3 << 11)) & 15u;
    const unsigned my_d = ((unsigned)bid - ((xcc < 8u ? xcc_map >> (4 * xcc) : 0u) & 15u)) & 7u;
    unsigned *const xcd_words = sy.timeout_flag + 4;  // [2][kDecodeMaxGrid]
    if (bid == (int)gridDim.x - 1 && sy.epoch > 1u) {
        volatile unsigned *seen = reinterpret_cast<volatile unsigned *>(lds + kWideLds) + 4;  // 8 words
        if (tid < 8) seen[tid] = 0u;
        __syncthreads();
        if (tid < (int)gridDim.x) {
            const unsigned left = xcd_words[kDecodeMaxGrid * ((sy.epoch + 1u) & 1u) + tid];
            if ((left >> 8) == ((sy.epoch - 1u) & 0xFFFFFFu)) {
                if ((left & 0x80u) == 0u)
                    atomicOr(const_cast<unsigned *>(seen) + ((left >> 4) & 7u), 1u << (left & 7u));
                else
                    atomicOr(sy.timeout_flag, 2u);  // an XCD number beyond 7
            }
        }
        __syncthreads();
        if (tid < 8) {
            const unsigned d_seen = seen[tid];
            if (d_seen & (d_seen - 1u)) {
                atomicOr(sy.timeout_flag, 2u);
                sy.timeout_flag[2] = (tid << 8) | d_seen;  // the XCD and the differences seen there
            }
        }
    }
    if (tid == 0) xcd_words[kDecodeMaxGrid * (sy.epoch & 1u) + bid] = (sy.epoch << 8) | (xcc << 4) | my_d;
    LORA_CLOCK(0);
#ifdef LORA_WG_CLOCKS
    if (g_clock_buf && tid == 0 && blockIdx.x < g_clock_slots)
        g_clock_buf[(size_t)blockIdx.x * 8 + 5] = 1000 + (__builtin_amdgcn_s_getreg(20 | (3 << 11)) & 15u);
#endif

    // ---- the shrink unit ----
    auto s_word = [&](int w) __attribute__((always_inline)) { return unit_word(s_rec, w); };
    const int ntok = (int)s_word(5), pn = (int)s_word(7);
    const bool s_has = bid < n_s && ntok > 0;
    if (s_has) {
        const uint64_t u_w_off = s_word(0) | ((uint64_t)s_word(1) << 32);
        const int64_t u_v_off = (int64_t)(s_word(2) | ((uint64_t)s_word(3) << 32));
        const int u_r8 = (int)s_word(4), u_p0 = (int)s_word(6), u_sync_idx = (int)s_word(12);
        const bool w_ok = i < pn;
        const int blk_rows = min(kRowTile, u_r8 - (u_p0 & ~(kRowTile - 1)));
        const int row0 = u_p0 & (kRowTile - 1);
        const uint16_t *wrow = arena + u_w_off + (kq * blk_rows + row0 + (w_ok ? i : 0)) * 8;
        const int half = lane >> 5;
        const int s_chunk = lane & 31;
        const uint16_t *xrow[kTokTile / 2];
#pragma unroll
        for (int t = 0; t < kTokTile / 2; ++t) {
            const int tok_even = (int)s_word(16 + 2 * t), tok_odd = (int)s_word(17 + 2 * t);
            xrow[t] = x + (int64_t)(half ? tok_odd : tok_even) * ldx;
        }
        const int kslice_beg = slice * k_slice_len;
        int kslice_end = kslice_beg + k_slice_len;
        if (kslice_end > in) kslice_end = in;
        if (slice >= n_slices) kslice_end = kslice_beg;
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
        for (int kp = kslice_beg; kp < kslice_end; kp += 4 * kWideK) {
            const int kbeg = kp + wq * kWideK;  // wavefront-uniform
            if (kbeg >= kslice_end) break;
            uint4 a[kShrinkSteps];
#pragma unroll
            for (int q = 0; q < kShrinkSteps; ++q) {
                const int k = kbeg + 32 * q;
                a[q] = (k < kslice_end) ? ld16_stream(wrow + (int64_t)k * blk_rows) : zero;
            }
            int kx = kbeg + 8 * s_chunk;
            if (kx > in - 8) kx = in - 8;
            uint4 xs[kTokTile / 2];
#pragma unroll
            for (int t = 0; t < kTokTile / 2; ++t)
                if (2 * t < ntok) xs[t] = ld16(xrow[t] + kx);
#pragma unroll
            for (int t = 0; t < kTokTile / 2; ++t)
                if (2 * t < ntok) *reinterpret_cast<uint4 *>(&slab[2 * t + half][8 * s_chunk]) = xs[t];
            __atomic_signal_fence(__ATOMIC_SEQ_CST);
            __builtin_amdgcn_wave_barrier();
            __atomic_signal_fence(__ATOMIC_SEQ_CST);
#pragma unroll
            for (int q = 0; q < kShrinkSteps; ++q) {
                const int k = kbeg + 32 * q;
                if (k < kslice_end) {
                    const uint4 aa = w_ok ? a[q] : zero;
                    const uint4 bb = *reinterpret_cast<const uint4 *>(&slab[i][32 * q + 8 * kq]);
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(aa), as_bf16x8(bb), acc, 0, 0, 0);
                }
            }
            __atomic_signal_fence(__ATOMIC_SEQ_CST);
            __builtin_amdgcn_wave_barrier();
            __atomic_signal_fence(__ATOMIC_SEQ_CST);
        }
        LORA_CLOCK(1);
        // the sixteen tiles added in the order of the k-slice plan (inside a slice by wavefront, then the
        // slices), by wavefront 0 alone: one barrier instead of two
        red[wave][lane] = acc;
        __syncthreads();
        if (wave == 0) {
            f32x4 t = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int sl = 0; sl < kMaxSlices; ++sl) {
                if (sl < n_slices) {
                    f32x4 ts = red[4 * sl][lane];
                    ts += red[4 * sl + 1][lane];
                    ts += red[4 * sl + 2][lane];
                    ts += red[4 * sl + 3][lane];
                    t = sl ? t + ts : ts;
                }
            }
            if (i < ntok && 4 * kq < pn) {
                const int64_t off = u_v_off + (int64_t)i * u_r8 + 4 * kq;
                uint2 h, l;
                h.x = pack_bf16_rne(t[0], t[1]);
                h.y = pack_bf16_rne(t[2], t[3]);
                l.x = pack_bf16_rne(t[0] - bf16_bits_to_f32(h.x & 0xFFFFu), t[1] - __uint_as_float(h.x & 0xFFFF0000u));
                l.y = pack_bf16_rne(t[2] - bf16_bits_to_f32(h.y & 0xFFFFu), t[3] - __uint_as_float(h.y & 0xFFFF0000u));
                *reinterpret_cast<uint2 *>(sy.v_hi + off) = h;
                *reinterpret_cast<uint2 *>(sy.v_lo + off) = l;
            }
        }
        // Nobody requests expand operands before the stores of v have been issued: a compute unit passes
        // its memory operations on in the order they were issued, and behind 120 KB of requests for B^T
        // the stores would reach the L2 microseconds later.
        __syncthreads();
        LORA_CLOCK(7);
        if (wave == 0) {
            stores_done();  // the stores have reached the L2
            if (lane == 0) l2_counter_add(sy.ready + u_sync_idx, 1u);
            LORA_CLOCK(2);
        }
    } else {
        __syncthreads();  // the flags in LDS are set
    }

    // ---- the expand unit of this group of four wavefronts ----
    const int e_idx = 4 * bid + slice;
    const Unit *eu = e_units + (e_idx < n_e ? e_idx : 0);
    const int e_ntok = e_idx < n_e ? eu->ntok : 0;
    const bool e_has = e_ntok > 0;
    const int qtid = tid & 255;
    const int e_tok = qtid >> 4;  // epilogue role: token e_tok of the unit, 8 columns from 8*e_cg of every strip
    const int e_cg = qtid & 15;
    float(*part)[kTokTile][kPartRow] = reinterpret_cast<float(*)[kTokTile][kPartRow]>(lds + slice * kExpandLds);
    const int e_r8 = eu->r8, e_ncols = eu->pn;
    const int P = e_r8 <= 32 ? 1 : (e_r8 <= 64 ? 2 : 4);  // wavefronts that share a strip, each a part of the rank
    const int S = 4 / P;                                   // strips per pass
    const int my_strip = wq / P, my_part = wq % P;
    const int j0 = 32 * my_part + 8 * kq, j1 = 32 * (my_part + 4) + 8 * kq;
    const bool j_ok0 = j0 < e_r8, j_ok1 = j1 < e_r8;
    const int jc0 = j_ok0 ? j0 : 0, jc1 = j_ok1 ? j1 : 0;
    const bool strip_ok = my_strip * kStrip < e_ncols;
    uint4 w[8], yv[4];
    uint16_t *e_y = y;
    const uint16_t *brow = arena;
    if (e_has) {
        // requests that do not need v: the B^T operands of the first k step and the rows of y
        const int64_t row = eu->tok[e_tok < e_ntok ? e_tok : 0];
        brow = arena + eu->w_off + (int64_t)(strip_ok ? my_strip * kStrip : 0) * e_r8 + i * 8;
#pragma unroll
        for (int b = 0; b < 8; ++b) w[b] = ld16_stream(brow + b * 16 * e_r8 + jc0 * 16);
        e_y = y + row * ldy + eu->p0 + 8 * e_cg;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            yv[s] = zero;
            if (s < S && s * kStrip < e_ncols) yv[s] = ld16_stream(e_y + s * kStrip);
        }
        // Wait for the tile's v.  The first wavefront of the four polls the tile's counter in the L2 and
        // tells the other three through LDS.
        if (wq == 0) {
            const unsigned target = sy.epoch * (unsigned)eu->sync_n;
            unsigned spins = 0;
            // one lane polls (an atomic is executed once per lane, even on one address)
            for (;;) {
                unsigned seen = 0u;
                if (lane == 0) seen = l2_counter_value(sy.ready + eu->sync_idx);
                seen = __builtin_amdgcn_readfirstlane(seen);
                if ((int)(seen - target) >= 0) break;
                if (++spins > sy.spin_limit) {
                    if (lane == 0) atomicOr(sy.timeout_flag, 1u);
                    break;
                }
                __builtin_amdgcn_s_sleep(4);
            }
            if (lane == 0) *qflag = 1u;
        } else {
            unsigned spins = 0;
            while (*qflag == 0u) {
                if (++spins > sy.spin_limit) break;  // the polling wavefront reports the time-out
                __builtin_amdgcn_s_sleep(2);
            }
        }
        __atomic_signal_fence(__ATOMIC_SEQ_CST);
        LORA_CLOCK(3);
        const bool ok0 = (i < e_ntok) && j_ok0;
        const int64_t off0 = eu->v_off + (int64_t)(ok0 ? i : 0) * e_r8 + jc0;
        // Agent-scope loads, which do not stop at this compute unit's vector cache: a 128-byte line of v
        // can hold rows of two token tiles, and another unit of this work group may have fetched the line
        // for its own tile before this tile's rows were stored (seen as rows without their delta, on a
        // first, cold launch at 14,336 input features, where the shrink units end far apart).
        uint4 vh0 = ld_through_u16x8(sy.v_hi + off0), vl0 = ld_through_u16x8(sy.v_lo + off0);
        uint4 vh1 = zero, vl1 = zero;
        const bool ok1 = (i < e_ntok) && j_ok1;
        if (e_r8 > 128) {
            const int64_t off1 = eu->v_off + (int64_t)(ok1 ? i : 0) * e_r8 + jc1;
            vh1 = ld_through_u16x8(sy.v_hi + off1);
            vl1 = ld_through_u16x8(sy.v_lo + off1);
        }
        if (!ok0) vh0 = vl0 = zero;
        if (!ok1) vh1 = vl1 = zero;
        f32x4 acc[8];
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            const bf16x8 ww = as_bf16x8(j_ok0 ? w[b] : zero);
            acc[b] = f32x4{0.f, 0.f, 0.f, 0.f};
            acc[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(vh0), ww, acc[b], 0, 0, 0);
            acc[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(vl0), ww, acc[b], 0, 0, 0);
        }
        if (e_r8 > 128) {
            // the second k step of ranks above 128 re-uses the operand registers
#pragma unroll
            for (int b = 0; b < 8; ++b) w[b] = ld16_stream(brow + b * 16 * e_r8 + jc1 * 16);
#pragma unroll
            for (int b = 0; b < 8; ++b) {
                const bf16x8 ww = as_bf16x8(j_ok1 ? w[b] : zero);
                acc[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(vh1), ww, acc[b], 0, 0, 0);
                acc[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(vl1), ww, acc[b], 0, 0, 0);
            }
        }
        if (strip_ok) {
            // lane (n, kq) holds tokens 4*kq + e, columns 8*n + b
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int tok = 4 * kq + e;
                if (tok < e_ntok) {
                    const f32x4 lo = {acc[0][e], acc[1][e], acc[2][e], acc[3][e]};
                    const f32x4 hi = {acc[4][e], acc[5][e], acc[6][e], acc[7][e]};
                    *reinterpret_cast<f32x4 *>(&part[wq][tok][8 * i]) = lo;
                    *reinterpret_cast<f32x4 *>(&part[wq][tok][8 * i + 4]) = hi;
                }
            }
        }
    }
    __syncthreads();
    if (e_has && e_tok < e_ntok) {
        const float scale = eu->scale;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            if (s < S && s * kStrip < e_ncols) {
                f32x4 d0 = *reinterpret_cast<const f32x4 *>(&part[s * P][e_tok][8 * e_cg]);
                f32x4 d1 = *reinterpret_cast<const f32x4 *>(&part[s * P][e_tok][8 * e_cg + 4]);
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
                st16_stream(e_y + s * kStrip, o);
            }
        }
    }
    LORA_CLOCK(4);
}

// One work group per place of a launch writes the XCD it runs on (hardware register XCC_ID, bits 3:0).
__global__ void k_probe_xcc(unsigned *out)
{
    if (threadIdx.x == 0) out[blockIdx.x] = __builtin_amdgcn_s_getreg(20 | (3 << 11)) & 15u;
}

constexpr int kFusedLds = kShrinkLds > kExpandLds ? kShrinkLds : kExpandLds;

__global__ __launch_bounds__(kThreads) void k_shrink(const Unit *__restrict__ units,
                                                     const uint16_t *__restrict__ arena,
                                                     const uint16_t *__restrict__ x, int64_t ldx, int in,
                                                     int k_slice_len, float *__restrict__ v_out, int n_slices,
                                                     int64_t slice_stride, Sync sy)
{
    __shared__ __attribute__((aligned(16))) char lds[kShrinkLds];
    LORA_CLOCK(0);
    shrink_body(units[blockIdx.x], arena, x, ldx, in, k_slice_len, v_out, n_slices, slice_stride, lds, sy);
    LORA_CLOCK(4);
}

// BIG: units of up to 64 tokens (token-heavy groups), token indices from perm, the next token block's
// loads in flight while the current one computes.  VF32: v is fp32 from the caller (stand-alone expand).
template <bool BIG, bool VF32>
__global__ __launch_bounds__(kThreads, BIG ? 2 : 4) void k_expand(const Unit *__restrict__ units,
                                                                  const int32_t *__restrict__ perm,
                                                                  const uint16_t *__restrict__ arena,
                                                                  const float *__restrict__ v_in, int n_slices,
                                                                  int64_t slice_stride, uint16_t *__restrict__ y,
                                                                  int64_t ldy, Sync sy)
{
    __shared__ __attribute__((aligned(16))) char lds[BIG ? kBigLds : kExpandLds];
    LORA_CLOCK_E(0);
    expand_dispatch<BIG, VF32>(units[blockIdx.x], perm, arena, v_in, n_slices, slice_stride, y, ldy, lds, sy);
    LORA_CLOCK_E(4);
}

// Both halves in one launch: blocks [0, n_shrink) are shrink units, the rest expand units that wait
// for their tokens' v through the counters.
__global__ __launch_bounds__(kThreads, 4) void k_apply_fused(const Unit *__restrict__ shrink_units, int n_shrink,
                                                          const Unit *__restrict__ expand_units,
                                                          const int32_t *__restrict__ perm,
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
        expand_dispatch<false, false>(expand_units[b - n_shrink], perm, arena, parts, n_slices, slice_stride, y, ldy,
                                      lds, sy);
}

// A mixed batch in two launches on one queue: the token-heavy groups' units first in the grid (they
// last longest), the decode-sized groups' k-slice units behind them, which fill the places the long
// units leave.  Every unit does what it does in a launch of its own kind: the token-heavy shrink
// units write v complete as bf16 hi + lo, the k-slice units leave partial sums and the one that
// completes a token tile writes its hi + lo; both kinds of expand unit read v from there.
constexpr int kMixedShrinkLds = kPrefillLds > kShrinkLds ? kPrefillLds : kShrinkLds;
constexpr int kMixedExpandLds = kBigLds > kExpandLds ? kBigLds : kExpandLds;

template <bool ANY>
__global__ __launch_bounds__(kThreads, ANY ? 2 : 4) void k_shrink_mixed(
    const Unit *__restrict__ heavy_units, int n_heavy, const Unit *__restrict__ units,
    const int32_t *__restrict__ perm, const uint16_t *__restrict__ arena, const uint16_t *__restrict__ x, int64_t ldx,
    int in, int k_slice_len, float *__restrict__ parts, int n_slices, int64_t slice_stride, Sync sy)
{
    __shared__ __attribute__((aligned(16))) char lds[kMixedShrinkLds];
    const int b = blockIdx.x;
    if (b < n_heavy && heavy_units[b].ntok <= 0) return;  // a place that only pads an XCD's list of token-heavy units
    LORA_CLOCK(0);
    if (b < n_heavy)
        prefill_dispatch<ANY>(heavy_units[b], perm, arena, x, ldx, in, sy.v_hi, sy.v_lo, nullptr, n_slices,
                              slice_stride, lds, parts, sy);
    else
        shrink_body(units[b - n_heavy], arena, x, ldx, in, k_slice_len, parts, n_slices, slice_stride, lds, sy);
    LORA_CLOCK(4);
}

__global__ __launch_bounds__(kThreads, 2) void k_expand_mixed(const Unit *__restrict__ big_units, int n_big,
                                                              const Unit *__restrict__ units,
                                                              const int32_t *__restrict__ perm,
                                                              const uint16_t *__restrict__ arena,
                                                              const float *__restrict__ parts, int n_slices,
                                                              int64_t slice_stride, uint16_t *__restrict__ y,
                                                              int64_t ldy, Sync sy)
{
    __shared__ __attribute__((aligned(16))) char lds[kMixedExpandLds];
    const int b = blockIdx.x;
    LORA_CLOCK_E(0);
    if (b < n_big)
        expand_dispatch<true, false>(big_units[b], perm, arena, parts, n_slices, slice_stride, y, ldy, lds, sy);
    else
        expand_dispatch<false, false>(units[b - n_big], perm, arena, parts, n_slices, slice_stride, y, ldy, lds, sy);
    LORA_CLOCK_E(4);
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

// ------------------------------------------------------------------------------------------------
// The adapted layer as one GEMM whose epilogue adds the delta: y = bf16(x W + s_a (x A_a) B_a), y written
// once and never read (the delta on its own reads y and writes it back: two thirds of its traffic on
// token-heavy batches).  Rows are taken in the order "tokens grouped by adapter, groups padded to
// multiples of 16", so that every 16-row MFMA block has one adapter; x is gathered and y scattered
// through that order, so no copy of either is made.
//   * One work group (8 wavefronts) computes a 256 x 256 tile, wavefront w the rows 64 (w mod 4) .. + 63
//     of it and the 128-column strip w / 4: 4 x 8 MFMA tiles of 16 x 16, 128 accumulator registers.  With
//     the columns of sub-block b being 8 n + b, lane n ends up with 8 consecutive columns of 4 tokens per
//     row block, and y leaves in 16-byte pieces.  (A compute unit takes about 50 GB/s from the L2s
//     whatever it runs; a 256 x 128 tile draws 48 KB per 64 of k and sat exactly at that rate, 720 us for
//     cfg2's 22.5 k x 4096 x 4096; two strips per tile share the 32 KB of x.)
//   * Everything is copied by loads that write LDS directly, through a ring of five 32 KB slots (all of a
//     compute unit's LDS), so no request passes through registers the compiler tracks and the waits are
//     exact: every wavefront issues four copies per slot and waits until at most four are in flight.
//     W comes packed in operand order (1 KB per wavefront operand, see launch_pack_weight), so a 32-wide
//     k step of a strip is 8 KB of consecutive bytes.  x is gathered in operand order by the copy itself,
//     in full cache lines: a copy takes 128 bytes (64 of k) of 8 rows (64 bytes of 16 rows took twice as
//     long to arrive), so a slot holds, of x, one half of the tile's rows for a pair of k steps and, of
//     W, one k step; pair j is computed from slots 2 j and 2 j + 1 while the copies of the next three
//     slots are in flight, one barrier per pair.  Inside a 1 KB block of x, piece p of row r sits in
//     slot 8 r + (p XOR r), so that the 8 lanes that read one piece of 8 rows meet 8 bank groups.
//   * After the k loop every row block adds s (v_hi + v_lo) B_a for its adapter: ceil(r8 / 32) more k
//     steps whose operands come straight from memory (v rows, and B^T in the pool's operand order,
//     the very pieces the expand kernels read), accumulated apart and scaled once, as the expand does.
// ------------------------------------------------------------------------------------------------
constexpr int kLinThreads = 512;
constexpr int kLinRing = 5;
constexpr int kLinXBuf = (kLinTileM / 16) * 1024;       // bytes of x per slot: 128 rows x 128 bytes = 16 KB
constexpr int kLinWBuf = 8 * 1024 * (kLinTileN / 128);  // bytes of W per slot: one k step of 2 strips, 8 KB each
constexpr int kLinLds = kLinRing * (kLinXBuf + kLinWBuf);  // 160 KB, all of a compute unit's LDS: one work group per compute unit
static_assert(kLinTileM == 256 && kLinTileN == 256, "the wavefront roles below are written for 256 x 256");

__global__ __launch_bounds__(kLinThreads, 1) void k_linear_lora(
    const int32_t *__restrict__ rows, const LinBlock *__restrict__ blocks, int m_tiles, int mt_per_xcd, int n_tiles,
    const uint16_t *__restrict__ arena, const uint16_t *__restrict__ wp, const uint16_t *__restrict__ x, int64_t ldx,
    int in, int out, const uint16_t *__restrict__ v_hi, const uint16_t *__restrict__ v_lo, uint16_t *__restrict__ y,
    int64_t ldy)
{
    __shared__ __attribute__((aligned(16))) char lds[kLinLds];
    // Work group b runs on XCD b mod 8.  Each XCD takes a run of row tiles, and the 32 work groups it runs
    // at a time (one per compute unit) are 8 row tiles x 4 column tiles that walk k together: every
    // chunk of x and of W that one of them brings into the XCD's L2 serves four or eight of them.
    const int xcd = blockIdx.x & 7, jloc = blockIdx.x >> 3;
    const int ngroups_n = (n_tiles + 3) >> 2;
    const int grp = jloc >> 5, within = jloc & 31;
    const int mt_loc = (grp / ngroups_n) * 8 + (within >> 2);
    const int nt = (grp % ngroups_n) * 4 + (within & 3);
    const int mt = xcd * mt_per_xcd + mt_loc;
    if (mt_loc >= mt_per_xcd || mt >= m_tiles || nt >= n_tiles) return;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int rw = wave & 3;                     // rows 64 rw .. 64 rw + 63 of the tile
    const int strip = 2 * nt + (wave >> 2);      // this wavefront's 128-column strip
    const bool has_strip = strip * 128 < out;    // out is a multiple of 128: the last tile may hold one strip
    const int n = lane & 15, kq = lane >> 4;
    const int m0 = mt * kLinTileM;
    const uint4 zero = {0u, 0u, 0u, 0u};
    auto xbuf = [&](int which) __attribute__((always_inline)) { return lds + which * (kLinXBuf + kLinWBuf); };
    auto wbuf = [&](int which) __attribute__((always_inline)) { return lds + which * (kLinXBuf + kLinWBuf) + kLinXBuf; };

    // Copies of x.  A copy takes 8 rows x 128 bytes (64 of k): full cache lines; with 64 bytes of 16 rows per
    // copy the same bytes took twice as long to arrive (0.57 against 0.33 us per 32 of k and compute unit
    // in a kernel that only copies).  One ring slot ("half stage" h) therefore holds, of x, the 128 rows
    // of row half h mod 2 for the 64 of k of pair h / 2, as 16 blocks of 1 KB; this wavefront fills blocks
    // 2 wave and 2 wave + 1, its lane l the slot l of a block with piece (l mod 8) XOR (l / 8) of row l / 8,
    // so that the 8 lanes that read one piece of 8 rows meet 8 different bank groups.
    const uint16_t *xsrc[2][2];
    {
        const int r = lane >> 3, piece = (lane & 7) ^ r;
#pragma unroll
        for (int hf = 0; hf < 2; ++hf)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int row = rows[m0 + 128 * hf + 8 * (2 * wave + j) + r];
                xsrc[hf][j] = x + (int64_t)(row < 0 ? 0 : row) * ldx + 8 * piece;
            }
    }
    // copies of W: k step h of a strip is 8 KB at wp + (strip * (in / 32) + h) * 4096 elements; the four
    // wavefronts of a strip copy two of its eight 1 KB pieces each.  (The wavefronts of a strip the matrix
    // does not have copy strip 0's pieces into their unused half: every wavefront then has the same
    // number of copies in flight, which the waits below count.)
    const uint4 *wsrc = reinterpret_cast<const uint4 *>(wp + (size_t)(has_strip ? strip : 0) * (in / 32) * 4096);
    const int w_half = (wave >> 2) * (kLinWBuf / 2);
    auto issue = [&](int h, int which) __attribute__((always_inline)) {
        const int hf = h & 1;
#pragma unroll
        for (int j = 0; j < 2; ++j)
            dma16_to_lds(reinterpret_cast<const uint4 *>((hf ? xsrc[1][j] : xsrc[0][j]) + (h >> 1) * 64),
                         reinterpret_cast<const uint4 *>(xbuf(which) + (2 * wave + j) * 1024));
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const int piece = 2 * rw + q;
            dma16_to_lds(wsrc + (size_t)h * 512 + piece * 64 + lane,
                         reinterpret_cast<const uint4 *>(wbuf(which) + w_half + piece * 1024));
        }
    };

    f32x4 acc[4][8];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int b = 0; b < 8; ++b) acc[i][b] = f32x4{0.f, 0.f, 0.f, 0.f};

    // Pair j (64 of k) is computed from half stages 2 j and 2 j + 1; while it is, the copies of 2 j + 2 ..
    // 2 j + 4 are in flight (a ring of five slots, all of the LDS).  One barrier per pair.
    const int nh = in / 32;   // half stages; in is a multiple of 64, so nh is even
    static_assert(kLinRing == 5, "the schedule below is written for five slots");
#pragma unroll
    for (int h = 0; h < 3; ++h)
        if (h < nh) issue(h, h);
    // this wavefront's rows 64 rw .. 64 rw + 63 lie in row half rw / 2, blocks 8 (rw mod 2) .. + 7 of its 16
    const int x_half = rw >> 1;
    const int x_blk0 = 8 * (rw & 1);
    for (int j = 0; 2 * j < nh; ++j) {
        // half stages 2 j and 2 j + 1 have landed when at most the copies of 2 j + 2 are in flight (4 per half
        // stage and wavefront)
        __atomic_signal_fence(__ATOMIC_SEQ_CST);
        if (2 * j + 2 < nh)
            asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
        else
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __atomic_signal_fence(__ATOMIC_SEQ_CST);
        // everyone's copies have landed, and everyone has left the slots of pair j - 1, which the copies of
        // half stages 2 j + 3 and 2 j + 4 now fill
        __syncthreads();
        if (2 * j + 3 < nh) issue(2 * j + 3, (2 * j + 3) % kLinRing);
        if (2 * j + 4 < nh) issue(2 * j + 4, (2 * j + 4) % kLinRing);
        if (has_strip) {
            const char *xcur = xbuf((2 * j + x_half) % kLinRing);
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                const char *wcur = wbuf((2 * j + ks) % kLinRing) + w_half;
                bf16x8 xo[4], wo[8];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    // row 16 i + n of this wavefront's rows: block x_blk0 + 2 i + n / 8, row n mod 8 of it, piece 4 ks + kq
                    const int r = n & 7, p = 4 * ks + kq;
                    xo[i] = as_bf16x8(*reinterpret_cast<const uint4 *>(
                        xcur + (x_blk0 + 2 * i + (n >> 3)) * 1024 + (r * 8 + (p ^ r)) * 16));
                }
#pragma unroll
                for (int b = 0; b < 8; ++b)
                    wo[b] = as_bf16x8(*reinterpret_cast<const uint4 *>(wcur + (b * 64 + lane) * 16));
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int b = 0; b < 8; ++b)
                        acc[i][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xo[i], wo[b], acc[i][b], 0, 0, 0);
            }
        }
    }
    if (!has_strip) return;

    // ---- the delta of each row block, then the store of y ----
    const int c0 = strip * 128;
    const LinBlock *bks = blocks + (m0 >> 4) + 4 * rw;
    // the delta of one row block from its own loads of B^T (row blocks whose neighbours have other adapters)
    auto delta_one = [&](int i) __attribute__((always_inline)) {
        const LinBlock &bk = bks[i];
        const int r8 = bk.r8;
        if (r8 <= 0) return;
        f32x4 dl[8];
#pragma unroll
        for (int b = 0; b < 8; ++b) dl[b] = f32x4{0.f, 0.f, 0.f, 0.f};
        const uint16_t *bt = arena + bk.b_off + (size_t)c0 * r8 + n * 8;
        for (int j = 0; j < r8; j += 32) {
            const int jj = j + 8 * kq;
            const bool j_ok = jj < r8;
            const bool ok = j_ok && n < bk.ntok;
            const int64_t off = bk.v_off + (int64_t)(ok ? n : 0) * r8 + (j_ok ? jj : 0);
            uint4 vh = ld16(v_hi + off), vl = ld16(v_lo + off);
            if (!ok) vh = vl = zero;
#pragma unroll
            for (int b = 0; b < 8; ++b) {
                // piece (sub-block b, rank piece jj / 8, column slot n) of the strip's B^T tile
                const uint4 wv = ld16(bt + (size_t)(b * (r8 >> 3) + (j_ok ? jj >> 3 : 0)) * 128);
                dl[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(vh), as_bf16x8(wv), dl[b], 0, 0, 0);
                dl[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(vl), as_bf16x8(wv), dl[b], 0, 0, 0);
            }
        }
        const float scale = bk.scale;
#pragma unroll
        for (int b = 0; b < 8; ++b) acc[i][b] += scale * dl[b];
    };
#pragma unroll
    for (int i = 0; i < 4; ++i) delta_one(i);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        // lane (n, kq) holds tokens 4 kq + e of the block, columns c0 + 8 n .. + 7
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int row = rows[m0 + 64 * rw + 16 * i + 4 * kq + e];
            if (row >= 0) {
                uint4 o;
                o.x = pack_bf16_rne(acc[i][0][e], acc[i][1][e]);
                o.y = pack_bf16_rne(acc[i][2][e], acc[i][3][e]);
                o.z = pack_bf16_rne(acc[i][4][e], acc[i][5][e]);
                o.w = pack_bf16_rne(acc[i][6][e], acc[i][7][e]);
                st16_stream(y + (int64_t)row * ldy + c0 + 8 * n, o);
            }
        }
    }
}

// W^T [out][in] row-major -> operand order (see launch_pack_weight).  One thread per destination element.
__global__ __launch_bounds__(256) void k_pack_w(const uint16_t *__restrict__ wt, int in, int out,
                                                uint16_t *__restrict__ dst)
{
    const int64_t d = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (d >= (int64_t)in * out) return;
    const int ksteps = in / 32;
    const int e = (int)(d & 7);
    const int slot = (int)((d >> 3) & 63);
    const int b = (int)((d >> 9) & 7);
    const int64_t rest = d >> 12;  // strip * ksteps + kstep
    const int kstep = (int)(rest % ksteps);
    const int strip = (int)(rest / ksteps);
    const int col = 128 * strip + 8 * (slot & 15) + b;
    const int k = 32 * kstep + 8 * (slot >> 4) + e;
    dst[d] = wt[(int64_t)col * in + k];
}

// Writes an adapter's packed form (see the top of this file).  One thread per destination element.
// A: [in][r] row-major -> dst of r8*in elements.
__global__ __launch_bounds__(256) void k_pack_a(const uint16_t *__restrict__ A, int in, int r, int r8,
                                                uint16_t *__restrict__ dst)
{
    const int64_t d = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (d >= (int64_t)r8 * in) return;
    const int jb = (int)(d / (16 * (int64_t)in));
    const int h = min(16, r8 - 16 * jb);
    const int64_t idx = d - (int64_t)jb * 16 * in;
    const int s = (int)(idx / (32 * h));
    const int rem = (int)(idx % (32 * h));
    const int kq = rem / (8 * h);
    const int n = (rem % (8 * h)) / 8;
    const int e = rem % 8;
    const int j = 16 * jb + n;
    const int k = 32 * s + 8 * kq + e;
    dst[d] = j < r ? A[(int64_t)k * r + j] : (uint16_t)0;
}

// B: [r][out] row-major -> dst of out*r8 elements.
__global__ __launch_bounds__(256) void k_pack_b(const uint16_t *__restrict__ B, int out, int r, int r8,
                                                uint16_t *__restrict__ dst)
{
    const int64_t d = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (d >= (int64_t)out * r8) return;
    const int strip = (int)(d / (128 * r8));
    const int idx = (int)(d % (128 * r8));
    const int b = idx / (16 * r8);
    const int rem = idx % (16 * r8);
    const int kp = rem / 128;
    const int n = (rem % 128) / 8;
    const int e = rem % 8;
    const int c = 128 * strip + 8 * n + b;
    const int j = 8 * kp + e;
    dst[d] = j < r ? B[(int64_t)j * out + c] : (uint16_t)0;
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

hipError_t launch_shrink_wide(const LaunchCtx &c, bool more_than_one_round, const uint16_t *x, int64_t ldx,
                              int k_slice_len, int n_slices, float *v_f32, uint16_t *v_hi, uint16_t *v_lo,
                              hipStream_t stream)
{
    if (c.n_units <= 0) return hipSuccess;
    if (n_slices < 1 || n_slices > kMaxSlices) return hipErrorInvalidValue;
    if (more_than_one_round)
        hipLaunchKernelGGL(k_shrink_wide<kWideHalfWaves>, dim3(c.n_units), dim3(64 * kWideHalfWaves), 0, stream,
                           c.units, c.arena, x, ldx, c.in_features, k_slice_len, n_slices, v_f32, v_hi, v_lo);
    else
        hipLaunchKernelGGL(k_shrink_wide<kWideWaves>, dim3(c.n_units), dim3(kWideThreads), 0, stream, c.units,
                           c.arena, x, ldx, c.in_features, k_slice_len, n_slices, v_f32, v_hi, v_lo);
    return hipGetLastError();
}

hipError_t launch_expand(const LaunchCtx &c, bool big, const float *v_in, int n_slices, int64_t slice_stride,
                         uint16_t *y, int64_t ldy, const SyncArgs *sync, hipStream_t stream)
{
    if (c.n_units <= 0) return hipSuccess;
    const Sync sy = make_sync(sync, 0);
    const dim3 g(c.n_units), b(kThreads);
    if (big && sync)
        hipLaunchKernelGGL((k_expand<true, false>), g, b, 0, stream, c.units, c.perm, c.arena, v_in, n_slices,
                           slice_stride, y, ldy, sy);
    else if (big)
        hipLaunchKernelGGL((k_expand<true, true>), g, b, 0, stream, c.units, c.perm, c.arena, v_in, n_slices,
                           slice_stride, y, ldy, sy);
    else if (sync)
        hipLaunchKernelGGL((k_expand<false, false>), g, b, 0, stream, c.units, c.perm, c.arena, v_in, n_slices,
                           slice_stride, y, ldy, sy);
    else
        hipLaunchKernelGGL((k_expand<false, true>), g, b, 0, stream, c.units, c.perm, c.arena, v_in, n_slices,
                           slice_stride, y, ldy, sy);
    return hipGetLastError();
}

hipError_t launch_apply_fused(const LaunchCtx &cs, const LaunchCtx &ce, const uint16_t *x, int64_t ldx,
                              int k_slice_len, float *parts, int n_slices, int64_t slice_stride, uint16_t *y,
                              int64_t ldy, const SyncArgs *sync, hipStream_t stream)
{
    const int total = cs.n_units + ce.n_units;
    if (total <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_apply_fused, dim3(total), dim3(kThreads), 0, stream, cs.units, cs.n_units, ce.units,
                       ce.perm, cs.arena, x, ldx, cs.in_features, k_slice_len, parts, n_slices, slice_stride, y, ldy,
                       make_sync(sync, 1));
    return hipGetLastError();
}

hipError_t launch_decode_fused(const LaunchCtx &cs, const LaunchCtx &ce, int grid, const uint16_t *x, int64_t ldx,
                               int k_slice_len, int n_slices, uint16_t *y, int64_t ldy, unsigned xcc_map,
                               const SyncArgs *sync, hipStream_t stream)
{
    if (cs.n_units <= 0 && ce.n_units <= 0) return hipSuccess;
    if (!sync || grid < 1 || grid > kDecodeMaxGrid || n_slices < 1 || n_slices > kMaxSlices || cs.n_units > grid || ce.n_units > 4 * grid ||
        cs.n_units < 1 || ce.n_units < 1)
        return hipErrorInvalidValue;
    hipLaunchKernelGGL(k_decode_fused, dim3(grid), dim3(kWideThreads), 0, stream, cs.units, cs.n_units, ce.units,
                       ce.n_units, cs.arena, x, ldx, cs.in_features, k_slice_len, n_slices, y, ldy, xcc_map,
                       make_sync(sync, 1));
    return hipGetLastError();
}

// Where the work groups of a launch run: host_out[b] = XCD of work group b of an n-work-group launch (n <=
// kProbeSlots).  Synchronous; its buffer is a device array of this file's own.
constexpr int kProbeSlots = 1024;
static __device__ unsigned xcc_probe_buf[kProbeSlots];

hipError_t probe_xcc(unsigned *host_out, int n_work_groups, hipStream_t stream)
{
    if (n_work_groups < 1 || n_work_groups > kProbeSlots) return hipErrorInvalidValue;
    void *buf = nullptr;
    hipError_t e = hipGetSymbolAddress(&buf, HIP_SYMBOL(xcc_probe_buf));
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_probe_xcc, dim3(n_work_groups), dim3(64), 0, stream, (unsigned *)buf);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if ((e = hipStreamSynchronize(stream)) != hipSuccess) return e;
    return hipMemcpy(host_out, buf, sizeof(unsigned) * (size_t)n_work_groups, hipMemcpyDeviceToHost);
}

hipError_t launch_shrink_prefill(const LaunchCtx &c, int n_hi, const uint16_t *x, int64_t ldx, uint16_t *v_hi,
                                 uint16_t *v_lo, float *v_f32, int n_slices, int64_t slice_stride, float *parts,
                                 const SyncArgs *sync, hipStream_t stream)
{
    if (c.n_units <= 0) return hipSuccess;
    if (n_hi < 0 || n_hi > c.n_units) return hipErrorInvalidValue;
    const Sync sy = make_sync(sync, 0);
    if (n_hi > 0)
        hipLaunchKernelGGL(k_shrink_prefill_any, dim3(c.n_units), dim3(kThreads), 0, stream, c.units, c.perm, c.arena,
                           x, ldx, c.in_features, v_hi, v_lo, v_f32, n_slices, slice_stride, parts, sy);
    else
        hipLaunchKernelGGL(k_shrink_prefill, dim3(c.n_units), dim3(kThreads), 0, stream, c.units, c.perm, c.arena, x,
                           ldx, c.in_features, v_hi, v_lo, v_f32, n_slices, slice_stride, parts, sy);
    return hipGetLastError();
}

hipError_t launch_shrink_mixed(const LaunchCtx &heavy, int n_hi, const LaunchCtx &c, const uint16_t *x, int64_t ldx,
                               int k_slice_len, float *parts, int n_slices, int64_t slice_stride,
                               const SyncArgs *sync, hipStream_t stream)
{
    const int total = heavy.n_units + c.n_units;
    if (total <= 0) return hipSuccess;
    if (!sync || n_hi < 0 || n_hi > heavy.n_units) return hipErrorInvalidValue;
    const Sync sy = make_sync(sync, 0);
    if (n_hi > 0)
        hipLaunchKernelGGL(k_shrink_mixed<true>, dim3(total), dim3(kThreads), 0, stream, heavy.units, heavy.n_units,
                           c.units, c.perm, c.arena, x, ldx, c.in_features, k_slice_len, parts, n_slices,
                           slice_stride, sy);
    else
        hipLaunchKernelGGL(k_shrink_mixed<false>, dim3(total), dim3(kThreads), 0, stream, heavy.units, heavy.n_units,
                           c.units, c.perm, c.arena, x, ldx, c.in_features, k_slice_len, parts, n_slices,
                           slice_stride, sy);
    return hipGetLastError();
}

hipError_t launch_expand_mixed(const LaunchCtx &big, const LaunchCtx &c, const float *parts, int n_slices,
                               int64_t slice_stride, uint16_t *y, int64_t ldy, const SyncArgs *sync,
                               hipStream_t stream)
{
    const int total = big.n_units + c.n_units;
    if (total <= 0) return hipSuccess;
    if (!sync) return hipErrorInvalidValue;
    hipLaunchKernelGGL(k_expand_mixed, dim3(total), dim3(kThreads), 0, stream, big.units, big.n_units, c.units,
                       c.perm, c.arena, parts, n_slices, slice_stride, y, ldy, make_sync(sync, 0));
    return hipGetLastError();
}

hipError_t launch_linear_lora(const int32_t *rows, const LinBlock *blocks, int m_pad, const uint16_t *arena,
                              const uint16_t *w_packed, const uint16_t *x, int64_t ldx, int in, int out,
                              const uint16_t *v_hi, const uint16_t *v_lo, uint16_t *y, int64_t ldy,
                              hipStream_t stream)
{
    if (m_pad <= 0) return hipSuccess;
    if (m_pad % kLinTileM || in % 64 || out % 128 || out <= 0 || in < 64) return hipErrorInvalidValue;
    const int m_tiles = m_pad / kLinTileM, n_tiles = (out + kLinTileN - 1) / kLinTileN;
    const int mt_per_xcd = (m_tiles + 7) / 8;
    // per XCD: groups of 32 work groups = 8 row tiles x 4 column tiles (see the kernel)
    const int64_t grid = (int64_t)8 * 32 * ((mt_per_xcd + 7) / 8) * ((n_tiles + 3) / 4);
    if (grid > 0x7FFFFFFF) return hipErrorInvalidValue;
    hipLaunchKernelGGL(k_linear_lora, dim3((unsigned)grid), dim3(kLinThreads), 0, stream, rows, blocks, m_tiles,
                       mt_per_xcd, n_tiles, arena, w_packed, x, ldx, in, out, v_hi, v_lo, y, ldy);
    return hipGetLastError();
}

hipError_t launch_pack_weight(const uint16_t *wt, int in, int out, uint16_t *dst, hipStream_t stream)
{
    const int64_t n = (int64_t)in * out;
    if (n <= 0 || in % 32 || out % 128) return hipErrorInvalidValue;
    hipLaunchKernelGGL(k_pack_w, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, wt, in, out, dst);
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

// ------------------------------------------------------------------------------------------------
// Workspace of the entry point that allocates nothing (lora_apply_static): each GPU the library runs
// on holds one copy of this array, at its own address, until the process ends.  In host code the
// array's name is only a handle for hipGetSymbolAddress; every use of its memory goes through the
// address looked up here, once per device, with that device current.
// ------------------------------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

hipError_t static_scratch(void **ptr)
{
    static std::atomic<void *> addr[kMaxDevices];
    *ptr = nullptr;
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    void *p = addr[dev].load(std::memory_order_acquire);
    if (!p) {
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        addr[dev].store(p, std::memory_order_release);  // two threads racing here store the same address
    }
    *ptr = p;
    return hipSuccess;
}

hipError_t launch_pack_adapter(const uint16_t *A, const uint16_t *B, int in, int out, int r, int r8,
                               uint16_t *dst_a, uint16_t *dst_b, hipStream_t stream)
{
    const int64_t na = (int64_t)r8 * in, nb = (int64_t)out * r8;
    hipLaunchKernelGGL(k_pack_a, dim3((unsigned)((na + 255) / 256)), dim3(256), 0, stream, A, in, r, r8, dst_a);
    hipLaunchKernelGGL(k_pack_b, dim3((unsigned)((nb + 255) / 256)), dim3(256), 0, stream, B, out, r, r8, dst_b);
    return hipGetLastError();
}

}  // namespace lora

#ifdef LORA_WG_CLOCKS
// Measurement build only: device buffer of 8 clock values per work group for the next launches (NULL = off).
extern "C" int lora_debug_clock_buffer(unsigned long long *dev_buf, unsigned n_work_groups)
{
    hipError_t e = hipMemcpyToSymbol(HIP_SYMBOL(lora::g_clock_buf), &dev_buf, sizeof dev_buf);
    if (e == hipSuccess) e = hipMemcpyToSymbol(HIP_SYMBOL(lora::g_clock_slots), &n_work_groups, sizeof n_work_groups);
    return (int)e;
}
#endif
