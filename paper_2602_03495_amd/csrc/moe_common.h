// Shared device helpers of the gfx950 MoE-layer kernels: bf16 packing, MFMA fragment types,
// 64-lane wavefront reductions.  Internal to the library; the public boundary is include/moe_layer.h.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "moe_layer.h"

#define MOE_WAVE 64

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;   // one MFMA A/B fragment (8 bf16 along K)
typedef __attribute__((ext_vector_type(4))) float f32x4;     // 16x16 accumulator fragment
typedef __attribute__((ext_vector_type(16))) float f32x16;   // 32x32 accumulator fragment

// Lane layouts of the two CDNA4 bf16 MFMA shapes used here (l = lane id):
//   16x16x32: A[i][k] from lane l: i = l%16, k = 8*(l/16)+0..7; B[k][j]: j = l%16, same k;
//             D[i][j]: lane l holds i = 4*(l/16)+r (r=0..3), j = l%16.
//   32x32x16: A[i][k]: i = l%32, k = 8*(l/32)+0..7; B[k][j]: j = l%32, same k;
//             D[i][j]: lane l holds i = 8*b + 4*(l/32) + r (b=0..3, r=0..3, element 4*b+r), j = l%32.

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;   // 16 bytes = 8 bf16, as loaded
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

__device__ __forceinline__ bf16x8 as_frag(u32x4 u) { return __builtin_bit_cast(bf16x8, u); }
__device__ __forceinline__ bf16x8 as_frag(uint4 u) { return __builtin_bit_cast(bf16x8, u); }

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// float -> bf16, round to nearest even, by the hardware conversion of gfx950 (v_cvt_pk_bf16_f32: two values per
// instruction, NaN stays NaN)
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{lo, hi}, bf16x2));
}

__device__ __forceinline__ uint32_t f32_to_bf16(float f) { return pack_bf16x2(f, 0.f) & 0xffffu; }

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1)
        v += __shfl_xor(v, o, MOE_WAVE);
    return v;
}

// ---- 64-lane reductions on the DPP crossbar (VALU speed; __shfl_xor goes through LDS and is ~10x slower per step).
// Inclusive row scans by 1, 2, 4, 8 leave each 16-lane row's result in its last lane; the four row results are
// then read with v_readlane, so the value returned is wave-uniform.  The combination order is fixed.
#define MOE_DPP_SHR(ident, v, n) \
    __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(ident), __float_as_int(v), 0x110 + (n), 0xF, 0xF, false))

__device__ __forceinline__ float wave_max_dpp(float v)
{
    const float ninf = -__builtin_huge_valf();
    v = fmaxf(v, MOE_DPP_SHR(ninf, v, 1));
    v = fmaxf(v, MOE_DPP_SHR(ninf, v, 2));
    v = fmaxf(v, MOE_DPP_SHR(ninf, v, 4));
    v = fmaxf(v, MOE_DPP_SHR(ninf, v, 8));
    const int b = __float_as_int(v);
    const float r0 = __int_as_float(__builtin_amdgcn_readlane(b, 15)), r1 = __int_as_float(__builtin_amdgcn_readlane(b, 31));
    const float r2 = __int_as_float(__builtin_amdgcn_readlane(b, 47)), r3 = __int_as_float(__builtin_amdgcn_readlane(b, 63));
    return fmaxf(fmaxf(r0, r1), fmaxf(r2, r3));
}

__device__ __forceinline__ float wave_sum_dpp(float v)
{
    v += MOE_DPP_SHR(0.f, v, 1);
    v += MOE_DPP_SHR(0.f, v, 2);
    v += MOE_DPP_SHR(0.f, v, 4);
    v += MOE_DPP_SHR(0.f, v, 8);
    const int b = __float_as_int(v);
    const float r0 = __int_as_float(__builtin_amdgcn_readlane(b, 15)), r1 = __int_as_float(__builtin_amdgcn_readlane(b, 31));
    const float r2 = __int_as_float(__builtin_amdgcn_readlane(b, 47)), r3 = __int_as_float(__builtin_amdgcn_readlane(b, 63));
    return (r0 + r1) + (r2 + r3);
}

// silu(g) * u with the hardware reciprocal (1 ulp) in place of an IEEE division: the result is rounded to bf16 anyway
__device__ __forceinline__ float silu_mul(float g, float u) { return g * __builtin_amdgcn_rcpf(1.0f + __expf(-g)) * u; }

// ---- work items of the experts that have rows and are masked on, without a schedule pass --------------------
// A launch of (upper bound of working experts) x per_expert blocks: every wave derives the working set itself
// as two 64-bit ballots over counts/mask, the block id is remapped so that each of the 8 XCDs (own L2) gets one
// contiguous run of the compacted item list (expert-major), and the item's expert is found by rank among the set
// bits.  Returns false for a block beyond the list.  All 64 lanes of the wave must call it.
#define MOE_NUM_XCD 8
__device__ __forceinline__ int moe_working_experts(int N, const int32_t *__restrict__ counts, const uint8_t *__restrict__ mask,
                                                   unsigned long long &act_lo, unsigned long long &act_hi)
{
    const int l = threadIdx.x & 63;
    const bool on_lo = l < N && counts[l] > 0 && (mask == nullptr || mask[l] != 0);
    const bool on_hi = l + 64 < N && counts[l + 64] > 0 && (mask == nullptr || mask[l + 64] != 0);
    act_lo = __ballot(on_lo);
    act_hi = __ballot(on_hi);
    return __popcll(act_lo) + __popcll(act_hi);
}

// the item of block pid among (working experts) x per_expert items, or false beyond the list
__device__ __forceinline__ bool moe_item_of(unsigned long long act_lo, unsigned long long act_hi, int per_expert, int pid, int &e,
                                            int &local)
{
    const int l = threadIdx.x & 63;
    const int n_lo = __popcll(act_lo);
    const int total = (n_lo + __popcll(act_hi)) * per_expert;
    if (pid >= total) return false;
    const int q = total / MOE_NUM_XCD, rem = total % MOE_NUM_XCD;
    const int xcd = pid % MOE_NUM_XCD, loc = pid / MOE_NUM_XCD;
    const int L = xcd < rem ? xcd * (q + 1) + loc : rem * (q + 1) + (xcd - rem) * q + loc;
    int a = L / per_expert;
    local = L - a * per_expert;
    unsigned long long m = act_lo;
    int base = 0;
    if (a >= n_lo) {
        a -= n_lo;
        m = act_hi;
        base = 64;
    }
    const unsigned long long below = l == 0 ? 0ull : (m << (64 - l));     // the bits of m under position l
    const bool mine = ((m >> l) & 1ull) != 0 && __popcll(below) == a;
    e = base + __ffsll((unsigned long long)__ballot(mine)) - 1;
    return true;
}

__device__ __forceinline__ bool moe_working_item(int N, const int32_t *__restrict__ counts, const uint8_t *__restrict__ mask,
                                                 int per_expert, int pid, int &e, int &local)
{
    unsigned long long act_lo, act_hi;
    moe_working_experts(N, counts, mask, act_lo, act_hi);
    return moe_item_of(act_lo, act_hi, per_expert, pid, e, local);
}

// K splits of the tiled down projection, decided on the device from the number of tile items that have work.  The
// cost of a launch is taken as (rounds of 256 compute units) x (item time, 1/nsp of an unsplit item); starting from no
// split, the next power of two up to nsp_max is taken whenever it lowers that cost by 15 % or more.  224 items stay
// whole (448 halves would need two rounds), 160 items run as 1280 eighths in 5 rounds (0.63 of a round of whole items).
__host__ __device__ __forceinline__ int moe_dev_splits(int items, int nsp_max)
{
    if (items <= 0) return 1;
    int nsp = 1, cost = ((items + 255) / 256) * 64;            // 64 = an unsplit item
    for (int finer = 2; finer <= nsp_max; finer *= 2) {
        const int c = ((items * finer + 255) / 256) * (64 / finer);
        if (c * 100 <= cost * 85) {
            cost = c;
            nsp = finer;
        }
    }
    return nsp;
}

#define MOE_CHECK_LAUNCH()                       \
    do {                                         \
        if (hipGetLastError() != hipSuccess)     \
            return MOE_ELAUNCH;                  \
    } while (0)

static inline size_t moe_align256(size_t x) { return (x + 255) & ~(size_t)255; }

// ---- workspace layout (one per shape; every entry point carves what it needs from offset 0) ----
struct moe_ws_layout {
    size_t act;        // [T*k, I] bf16 inner activations
    size_t partial;    // [nsplit, T*k, d] fp32 split-K partial sums of the down projection (skinny path, or the tiled path's K splits)
    size_t sched;      // tile schedule of the tiled path
    size_t route;      // routing scratch: folded bias [N], idx [T*k], w [T*k] (prediction), 2 x logits [max(T,16), N] (gate product and selection in separate launches)
    size_t total;
};

#define MOE_SKINNY_MAX_T 16
#define MOE_SKINNY_WAVES 4          // waves per block on the skinny path
#define MOE_SKINNY_MAX_STEPS 32     // 32-wide K steps a wave may hold in registers (K <= 1024 per wave)
#define MOE_TILE_M 128              // token rows per tile on the tiled path (the down projection may choose 112 or 96 on the device)
#define MOE_TILE_M_MIN 96
#define MOE_SKINNY_DOWN_MIN_I 2048  // decode-sized down projections with I up to this run on the tiled kernel

static inline int moe_skinny_nsplit(int K)
{
    int per_block = MOE_SKINNY_WAVES * MOE_SKINNY_MAX_STEPS * 32;
    return (K + per_block - 1) / per_block;
}

// Tiled down projection: the most K splits a launch may use (1 = never split).  Every split keeps at least 32 k32 steps, a
// multiple of 8; the fp32 partial sums [nsp, T*k, d] must fit 64 MB.  Whether a launch splits at all is decided on
// the device (moe_dev_splits): only when the experts that have rows and are masked on leave compute units without a tile.
static inline int moe_tiled_down_max_splits(const moe_shape *s)
{
    if (s->T <= MOE_SKINNY_MAX_T) return 1;
    const int steps = s->I / 32;
    int nsp = 1;
    while (nsp < 8 && steps % (2 * nsp * 8) == 0 && steps / (2 * nsp) >= 32 &&
           (size_t)(2 * nsp) * s->T * s->k * s->d * 4 <= ((size_t)64 << 20))
        nsp *= 2;
    return nsp;
}

// one tile table of the tiled path: int32 hdr[4] + one int4 per token tile, sized for the smallest tile height
static inline size_t moe_sched_table_bytes(const moe_shape *s)
{
    return moe_align256(((size_t)s->T * s->k / MOE_TILE_M_MIN + MOE_MAX_EXPERTS + 8) * 16);
}

// one [max(T, 16), N] fp32 block of gate logits (the gate product and the selection are separate launches when the
// gate matrix has many rows)
static inline size_t moe_logits_scratch_bytes(const moe_shape *s)
{
    return moe_align256((size_t)(s->T > 16 ? s->T : 16) * (size_t)s->N * 4);
}

static inline moe_ws_layout moe_ws(const moe_shape *s)
{
    moe_ws_layout L;
    size_t R = (size_t)s->T * s->k;
    size_t off = 0;
    L.act = off;
    off += moe_align256(R * (size_t)s->I * 2);
    L.partial = off;
    size_t Rs = R < (size_t)MOE_SKINNY_MAX_T * MOE_MAX_TOPK ? R : (size_t)MOE_SKINNY_MAX_T * MOE_MAX_TOPK;
    size_t part = (size_t)moe_skinny_nsplit(s->I) * Rs * s->d * 4;
    const int nsp = moe_tiled_down_max_splits(s);
    if (nsp > 1 && (size_t)nsp * R * s->d * 4 > part) part = (size_t)nsp * R * s->d * 4;
    off += moe_align256(part);
    L.sched = off;
    off += 2 * moe_sched_table_bytes(s);              // one table for the up projection, one for the down projection
    L.route = off;
    off += moe_align256(MOE_MAX_EXPERTS * 4) + 2 * moe_align256(R * 4) + 2 * moe_logits_scratch_bytes(s);
    L.total = off;
    return L;
}
