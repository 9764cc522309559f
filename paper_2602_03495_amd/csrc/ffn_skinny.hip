// Expert FFN for decode-sized batches (at most 16 rows per expert) on gfx950: a weight-streaming path.
//
// Every weight element of a touched, masked-on expert is read from HBM exactly once.  Weights are in the
// packed layout of moe_pack_weights, where one A operand of a bf16 MFMA 16x16x32 (16 weight rows x 32 k) is
// 1 KB of contiguous memory in lane order, so a wave's 16-byte-per-lane load is one fully coalesced 1 KB read
// that goes straight from global memory into the MFMA; the
// B operand holds the (<= 16) token rows of that expert and lives in registers for the whole block, so the
// inner loop is "global_load, mfma" and nothing else.  K is split over the 4 waves of a block (and, for the
// long down projection, over several blocks); partial 16x16 tiles are reduced through LDS (and through an
// fp32 scratch + a finishing kernel when K is split over blocks), in a fixed order, so results are
// reproducible.  The grid covers the experts that can be non-empty; blocks find their (working expert, row block)
// item themselves and run the compacted item list in XCD-contiguous order, so untouched and masked-off experts
// cost no memory traffic and the blocks of one expert share an L2.
#include "moe_common.h"

#define SK_WAVES MOE_SKINNY_WAVES
#define SK_THREADS (SK_WAVES * 64)

// Token-side B fragments of one wave: rows j = lane%16 of the expert, k = (s0+s)*32 + 8*(lane/16) ...
template <int MAXS>
__device__ __forceinline__ void load_x_frags(u32x4 (&xf)[MAXS], const uint16_t *row_ptr, bool valid, int s0, int ns, int g)
{
#pragma unroll
    for (int s = 0; s < MAXS; ++s) {
        xf[s] = u32x4{0u, 0u, 0u, 0u};
        if (valid && s < ns) xf[s] = *reinterpret_cast<const u32x4 *>(row_ptr + (size_t)(s0 + s) * 32 + g * 8);
    }
}

// act[p, i] = silu(W1_e[i,:] . x_p) * (W3_e[i,:] . x_p)   for the rows p of the block's expert
template <int MAXS, int RT>
__global__ __launch_bounds__(SK_THREADS) void skinny_up_kernel(
    int d, int k, int I, int N, int blocks_per_expert, const uint16_t *__restrict__ h, const int32_t *__restrict__ perm,
    const int32_t *__restrict__ offsets, const int32_t *__restrict__ counts, const uint16_t *__restrict__ w1,
    const uint16_t *__restrict__ w3, const uint8_t *__restrict__ mask, uint16_t *__restrict__ act)
{
    int e, bx;
    if (!moe_working_item(N, counts, mask, blocks_per_expert, blockIdx.x, e, bx)) return;
    const int c = counts[e];
    __shared__ float red[SK_WAVES][RT][2][256];

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int i = lane & 15, g = lane >> 4;
    const int off = offsets[e];
    const int total = d >> 5;
    const int per = (total + SK_WAVES - 1) / SK_WAVES;
    const int s0 = wave * per;
    int ns = total - s0;
    ns = ns < 0 ? 0 : (ns > per ? per : ns);

    u32x4 xf[MAXS];
    {
        const bool valid = i < c;
        const int tok = valid ? perm[off + i] / k : 0;
        load_x_frags<MAXS>(xf, h + (size_t)tok * d, valid, s0, ns, g);
    }
    const int i0 = bx * (16 * RT);
    const int last = ns > 0 ? ns - 1 : 0;   // steps past the wave's range re-read its last step against a zero fragment
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        int rb = (i0 >> 4) + rt;                            // 16-row block of W1 / W3
        if (rb * 16 >= I) rb = (I >> 4) - 1;
        const size_t fo = (size_t)e * I * d + ((size_t)rb * total + s0) * 512 + lane * 8;
        const uint16_t *p1 = w1 + fo;
        const uint16_t *p3 = w3 + fo;
        f32x4 ag = {0.f, 0.f, 0.f, 0.f}, au = {0.f, 0.f, 0.f, 0.f};
        if (ns > 0) {
            u32x4 a1[MAXS], a3[MAXS];
#pragma unroll
            for (int s = 0; s < MAXS; ++s) {
                const int so = (s < ns ? s : last) * 512;
                a1[s] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p1 + so));
                a3[s] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p3 + so));
            }
#pragma unroll
            for (int s = 0; s < MAXS; ++s) {
                ag = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_frag(a1[s]), as_frag(xf[s]), ag, 0, 0, 0);
                au = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_frag(a3[s]), as_frag(xf[s]), au, 0, 0, 0);
            }
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            red[wave][rt][0][lane * 4 + r] = ag[r];
            red[wave][rt][1][lane * 4 + r] = au[r];
        }
    }
    __syncthreads();
    // element el = 4*lane_src + r  ->  weight row 4*(lane_src/16) + r of the tile, token lane_src%16
    const int el = threadIdx.x;
    const int src = el >> 2, r = el & 3;
    const int j = src & 15, rowin = 4 * (src >> 4) + r;
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        float gsum = 0.f, usum = 0.f;
#pragma unroll
        for (int w = 0; w < SK_WAVES; ++w) {
            gsum += red[w][rt][0][el];
            usum += red[w][rt][1][el];
        }
        const int col = i0 + rt * 16 + rowin;
        if (j < c && col < I) act[(size_t)(off + j) * I + col] = (uint16_t)f32_to_bf16(silu_mul(gsum, usum));
    }
}

// y[p, f] (or a split-K partial of it) = W2_e[f,:] . act[p,:].  A block takes nchunks consecutive K chunks of
// steps_per_block k32 steps each (4 waves x at most MAXS steps in registers), one after the other, accumulating in
// registers; the grid carries nsplit such blocks per row block.
template <int MAXS, int RT, bool DIRECT>
__global__ __launch_bounds__(SK_THREADS) void skinny_down_kernel(
    int d, int I, int R, int N, int row_blocks, int nsplit, int nchunks, int steps_per_block, const uint16_t *__restrict__ act,
    const int32_t *__restrict__ offsets, const int32_t *__restrict__ counts, const uint16_t *__restrict__ w2,
    const uint8_t *__restrict__ mask, uint16_t *__restrict__ y, float *__restrict__ partial)
{
    int e, local;
    if (!moe_working_item(N, counts, mask, row_blocks * nsplit, blockIdx.x, e, local)) return;
    const int bx = local % row_blocks, by = local / row_blocks;    // row block, K split
    const int c = counts[e];
    __shared__ float red[SK_WAVES][RT][256];

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int i = lane & 15, g = lane >> 4;
    const int off = offsets[e];
    const int total = I >> 5;
    const int per = (steps_per_block + SK_WAVES - 1) / SK_WAVES;
    const bool valid = i < c;
    const uint16_t *xrow = act + (size_t)(off + (valid ? i : 0)) * I;
    const int f0 = bx * (16 * RT);

    f32x4 acc[RT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) acc[rt] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int ch = 0; ch < nchunks; ++ch) {
        const int b0 = (by * nchunks + ch) * steps_per_block;
        int bn = total - b0;
        bn = bn > steps_per_block ? steps_per_block : bn;
        const int s0 = b0 + wave * per;
        int ns = b0 + bn - s0;
        ns = ns < 0 ? 0 : (ns > per ? per : ns);
        if (ns <= 0) continue;
        u32x4 xf[MAXS];
        load_x_frags<MAXS>(xf, xrow, valid, s0, ns, g);
        const int last = ns - 1;
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            int rb = (f0 >> 4) + rt;                            // 16-row block of W2
            if (rb * 16 >= d) rb = (d >> 4) - 1;
            const uint16_t *p2 = w2 + (size_t)e * d * I + ((size_t)rb * total + s0) * 512 + lane * 8;
            u32x4 a[MAXS];
#pragma unroll
            for (int s = 0; s < MAXS; ++s)
                a[s] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p2 + (s < ns ? s : last) * 512));
#pragma unroll
            for (int s = 0; s < MAXS; ++s)
                acc[rt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_frag(a[s]), as_frag(xf[s]), acc[rt], 0, 0, 0);
        }
    }
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int r = 0; r < 4; ++r) red[wave][rt][lane * 4 + r] = acc[rt][r];
    __syncthreads();
    const int el = threadIdx.x;
    const int src = el >> 2, r = el & 3;
    const int j = src & 15, rowin = 4 * (src >> 4) + r;
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        float sum = 0.f;
#pragma unroll
        for (int w = 0; w < SK_WAVES; ++w) sum += red[w][rt][el];
        const int f = f0 + rt * 16 + rowin;
        if (j < c && f < d) {
            if (DIRECT)
                y[(size_t)(off + j) * d + f] = (uint16_t)f32_to_bf16(sum);
            else
                partial[((size_t)by * R + off + j) * d + f] = sum;
        }
    }
}

// y[p,:] = bf16( sum over the K splits, in split order )
__global__ __launch_bounds__(256) void skinny_finish_kernel(int d, int R, int nsplit, const float *__restrict__ partial,
                                                            const int32_t *__restrict__ offsets,
                                                            const int32_t *__restrict__ counts,
                                                            const uint8_t *__restrict__ mask, uint16_t *__restrict__ y)
{
    const int e = blockIdx.y, j = blockIdx.x;
    if (j >= counts[e] || (mask != nullptr && mask[e] == 0)) return;
    const size_t p = (size_t)offsets[e] + j;
    for (int f = threadIdx.x * 4; f < d; f += 1024) {
        float4 a = *reinterpret_cast<const float4 *>(partial + p * d + f);
        for (int ks = 1; ks < nsplit; ++ks) {
            float4 b = *reinterpret_cast<const float4 *>(partial + ((size_t)ks * R + p) * d + f);
            a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w;
        }
        uint2 o;
        o.x = pack_bf16x2(a.x, a.y);
        o.y = pack_bf16x2(a.z, a.w);
        *reinterpret_cast<uint2 *>(y + p * d + f) = o;
    }
}

// ---------------------------------------------------------------------------------------------------
static int pick_rt(int tiles_per_expert, int est_active)
{
    // the most 16-row tiles per block (fewer re-loads of the token fragments) that still leaves
    // at least two blocks per compute unit
    for (int rt = 4; rt > 1; rt >>= 1)
        if ((long)(tiles_per_expert / rt) * est_active >= 512) return rt;
    return 1;
}

template <int MAXS>
static void launch_up(int rt, dim3 grid, hipStream_t st, int d, int k, int I, int N, int bpe, const uint16_t *h,
                      const int32_t *perm, const int32_t *offsets, const int32_t *counts, const uint16_t *w1,
                      const uint16_t *w3, const uint8_t *mask, uint16_t *act)
{
    if (rt == 4)
        hipLaunchKernelGGL((skinny_up_kernel<MAXS, 4>), grid, dim3(SK_THREADS), 0, st, d, k, I, N, bpe, h, perm, offsets, counts, w1, w3, mask, act);
    else if (rt == 2)
        hipLaunchKernelGGL((skinny_up_kernel<MAXS, 2>), grid, dim3(SK_THREADS), 0, st, d, k, I, N, bpe, h, perm, offsets, counts, w1, w3, mask, act);
    else
        hipLaunchKernelGGL((skinny_up_kernel<MAXS, 1>), grid, dim3(SK_THREADS), 0, st, d, k, I, N, bpe, h, perm, offsets, counts, w1, w3, mask, act);
}

template <int MAXS, bool DIRECT>
static void launch_down(int rt, dim3 grid, hipStream_t st, int d, int I, int R, int N, int rb, int nsplit, int nchunks, int spb,
                        const uint16_t *act, const int32_t *offsets, const int32_t *counts, const uint16_t *w2,
                        const uint8_t *mask, uint16_t *y, float *partial)
{
    if (rt == 4)
        hipLaunchKernelGGL((skinny_down_kernel<MAXS, 4, DIRECT>), grid, dim3(SK_THREADS), 0, st, d, I, R, N, rb, nsplit, nchunks, spb, act, offsets, counts, w2, mask, y, partial);
    else if (rt == 2)
        hipLaunchKernelGGL((skinny_down_kernel<MAXS, 2, DIRECT>), grid, dim3(SK_THREADS), 0, st, d, I, R, N, rb, nsplit, nchunks, spb, act, offsets, counts, w2, mask, y, partial);
    else
        hipLaunchKernelGGL((skinny_down_kernel<MAXS, 1, DIRECT>), grid, dim3(SK_THREADS), 0, st, d, I, R, N, rb, nsplit, nchunks, spb, act, offsets, counts, w2, mask, y, partial);
}

int moe_ffn_tiled_impl(const moe_shape *, const void *, const int32_t *, const int32_t *, const int32_t *, const void *,
                       const void *, const void *, const uint8_t *, void *, void *, int, hipStream_t);

int moe_ffn_skinny_impl(const moe_shape *s, const void *h, const int32_t *perm, const int32_t *offsets,
                        const int32_t *counts, const void *w1, const void *w3, const void *w2,
                        const uint8_t *expert_mask, void *y, void *workspace, int stages, hipStream_t st)
{
    const int d = s->d, I = s->I, N = s->N, k = s->k, R = s->T * s->k;
    if (s->T > MOE_SKINNY_MAX_T) return MOE_EUNSUPPORTED;
    if (d > SK_WAVES * MOE_SKINNY_MAX_STEPS * 32) return MOE_EUNSUPPORTED;
    moe_ws_layout L = moe_ws(s);
    uint16_t *act = (uint16_t *)((char *)workspace + L.act);
    float *partial = (float *)((char *)workspace + L.partial);
    const int est_active = N < R ? N : R;

    // ---- gate/up projections + SwiGLU ------------------------------------------------------------
    if (stages & MOE_FFN_STAGE_UP) {
        const int per = ((d >> 5) + SK_WAVES - 1) / SK_WAVES;
        const int tiles = (I + 15) / 16;
        const int rt = pick_rt(tiles, est_active);
        const int bpe = (tiles + rt - 1) / rt;               // blocks per working expert
        dim3 grid((unsigned)(bpe * est_active));
        const uint16_t *hp = (const uint16_t *)h, *p1 = (const uint16_t *)w1, *p3 = (const uint16_t *)w3;
#define UP(n) case n: launch_up<4 * n>(rt, grid, st, d, k, I, N, bpe, hp, perm, offsets, counts, p1, p3, expert_mask, act); break;
        switch ((per + 3) / 4) { UP(1) UP(2) UP(3) UP(4) UP(5) UP(6) UP(7) UP(8) default: return MOE_EUNSUPPORTED; }
#undef UP
        MOE_CHECK_LAUNCH();
    }
    // ---- down projection ---------------------------------------------------------------------------
    // With a short inner size a wave's share of K is a handful of steps and the cross-wave reduction dominates:
    // the tiled kernel, where every wave owns whole weight rows, is the faster one there.
    if ((stages & MOE_FFN_STAGE_DOWN) && I <= MOE_SKINNY_DOWN_MIN_I)
        return moe_ffn_tiled_impl(s, h, perm, offsets, counts, w1, w3, w2, expert_mask, y, workspace, MOE_FFN_STAGE_DOWN, st);
    if (stages & MOE_FFN_STAGE_DOWN) {
        const int total = I >> 5;
        const int nchunk_all = moe_skinny_nsplit(I);         // K chunks of at most 4096
        const int spb = (total + nchunk_all - 1) / nchunk_all;
        const int per = (spb + SK_WAVES - 1) / SK_WAVES;
        const int tiles = (d + 15) / 16;
        // All K chunks inside one block of one 16-row tile (no partial sums, no finishing pass) for batches of at most
        // 8 routed rows: 1 token 135 -> 129 us per step, 4 tokens 38 -> 34 / 54 -> 48 / 78 -> 74 us for the down
        // projection with 1 / 2 / 3 experts at work.  With more rows a block's token fragments, re-read per chunk and per
        // block, outweigh the saved pass (16 tokens, 7 experts at work: 148 -> 160 us): one chunk per block there.
        const bool in_block = (long)tiles * est_active >= 512 && R <= 8;
        const int nsplit = in_block ? 1 : nchunk_all, nchunks = in_block ? nchunk_all : 1;
        const int rt = in_block ? 1 : pick_rt(tiles * nsplit, est_active);
        const int rbk = (tiles + rt - 1) / rt;               // row blocks per working expert
        dim3 grid((unsigned)(rbk * nsplit * est_active));
        const uint16_t *p2 = (const uint16_t *)w2;
        uint16_t *yp = (uint16_t *)y;
#define DN(n, direct) case n: launch_down<4 * n, direct>(rt, grid, st, d, I, R, N, rbk, nsplit, nchunks, spb, act, offsets, counts, p2, expert_mask, yp, partial); break;
        if (nsplit == 1) {
            switch ((per + 3) / 4) { DN(1, true) DN(2, true) DN(3, true) DN(4, true) DN(5, true) DN(6, true) DN(7, true) DN(8, true) default: return MOE_EUNSUPPORTED; }
            MOE_CHECK_LAUNCH();
        } else {
            switch ((per + 3) / 4) { DN(1, false) DN(2, false) DN(3, false) DN(4, false) DN(5, false) DN(6, false) DN(7, false) DN(8, false) default: return MOE_EUNSUPPORTED; }
            MOE_CHECK_LAUNCH();
            hipLaunchKernelGGL(skinny_finish_kernel, dim3(MOE_SKINNY_MAX_T, N), dim3(256), 0, st, d, R, nsplit, partial,
                               offsets, counts, expert_mask, yp);
            MOE_CHECK_LAUNCH();
        }
#undef DN
    }
    return MOE_OK;
}
