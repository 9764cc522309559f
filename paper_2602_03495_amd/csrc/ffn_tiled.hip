// Grouped SwiGLU expert FFN for prefill-sized batches on gfx950: LDS-tiled bf16 MFMA 32x32x16 GEMMs.
//
// Two grouped "NT" GEMMs (both operands K-contiguous), each over the rows of the masked-on, non-empty experts:
//   up:    act[p, i] = silu(x_p . W1_e[i,:]) * (x_p . W3_e[i,:])      x_p = h[perm[p]/k, :] gathered in the tile load
//   down:  y[p, f]   = act[p,:] . W2_e[f,:]
// A work item is (expert, 128-row token tile, 256-row weight tile); for "up" the weight tile is 128 rows of
// W1 and the same 128 rows of W3, so that a thread ends up holding a gate value and its up value and the
// SwiGLU is applied in registers.  The item list is built on the device from counts/offsets/mask by
// tile_schedule_kernel (no host round trip); empty and masked-off experts get no items.  The MFMA takes the
// weight rows as its A operand and the token rows as B, so each lane owns 4 consecutive output columns of one
// token and stores them as one 8-byte word.
//
// Launch order: block ids are dealt round-robin to the 8 XCDs, so ids are remapped to give each XCD (its own
// L2) a contiguous run of items, ordered expert-major, then weight tile, then token tile: the token tiles
// that share a weight tile run next to each other on one XCD and the weight tile is fetched from HBM once.
#include "moe_common.h"

#define TM MOE_TILE_M     // token rows per tile
#define TW 256            // weight rows per tile
#define TK 64             // k per LDS stage
#define LDS_LD 72         // LDS row pitch in bf16 (64 + 8 pad: 144 B keeps 16-lane b128 reads conflict-free)
#define NUM_XCD 8

// sched layout: int32 hdr[4] = {n_mtiles, 0, 0, 0}; then int4 per global token tile {expert, first_tile, n_tiles_of_expert, 0}
__global__ __launch_bounds__(MOE_MAX_EXPERTS) void tile_schedule_kernel(int N, const int32_t *__restrict__ counts,
                                                                        const uint8_t *__restrict__ mask,
                                                                        int32_t *__restrict__ sched)
{
    __shared__ int nmt[MOE_MAX_EXPERTS];
    __shared__ int first[MOE_MAX_EXPERTS];
    const int e = threadIdx.x;
    int n = 0;
    if (e < N && counts[e] > 0 && (mask == nullptr || mask[e] != 0)) n = (counts[e] + TM - 1) / TM;
    nmt[e] = n;
    __syncthreads();
    if (e == 0) {
        int run = 0;
        for (int j = 0; j < N; ++j) {
            first[j] = run;
            run += nmt[j];
        }
        sched[0] = run;
        sched[1] = sched[2] = sched[3] = 0;
    }
    __syncthreads();
    if (e < N) {
        int4 *tab = reinterpret_cast<int4 *>(sched + 4);
        for (int j = 0; j < n; ++j) tab[first[e] + j] = make_int4(e, first[e], n, 0);
    }
}

template <int MODE>   // 0: up (W1|W3 + SwiGLU -> act), 1: down (W2 -> y)
__global__ __launch_bounds__(256, 2) void ffn_tiled_kernel(
    int d, int I, int k, const uint16_t *__restrict__ xsrc,   // MODE 0: h [T,d]; MODE 1: act [R,I]
    const int32_t *__restrict__ perm, const int32_t *__restrict__ offsets, const int32_t *__restrict__ counts,
    const uint16_t *__restrict__ wa, const uint16_t *__restrict__ wb,   // MODE 0: w1, w3; MODE 1: w2, unused
    const int32_t *__restrict__ sched, uint16_t *__restrict__ out)      // MODE 0: act [R,I]; MODE 1: y [R,d]
{
    __shared__ __attribute__((aligned(16))) uint16_t Xs[TM * LDS_LD];
    __shared__ __attribute__((aligned(16))) uint16_t Ws[TW * LDS_LD];

    const int K = MODE == 0 ? d : I;          // contraction length
    const int NOUT = MODE == 0 ? I : d;       // output columns
    const int n_nt = MODE == 0 ? (I + 127) / 128 : (d + 255) / 256;

    // ---- which item ----------------------------------------------------------------------------
    const int n_mt = sched[0];
    const int total = n_mt * n_nt;
    const int pid = blockIdx.x;
    if (pid >= total) return;
    int L;
    {
        const int q = total / NUM_XCD, rem = total % NUM_XCD;
        const int xcd = pid % NUM_XCD, loc = pid / NUM_XCD;
        L = xcd < rem ? xcd * (q + 1) + loc : rem * (q + 1) + (xcd - rem) * q + loc;
    }
    const int4 ent = reinterpret_cast<const int4 *>(sched + 4)[L / n_nt];
    const int e = ent.x;
    const int local = L - ent.y * n_nt;
    const int mt = local % ent.z, nt = local / ent.z;
    const int row0 = offsets[e] + mt * TM;
    int nrows = counts[e] - mt * TM;
    nrows = nrows > TM ? TM : nrows;
    const int n0 = nt * (MODE == 0 ? 128 : 256);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave & 1, wn = wave >> 1;

    // ---- global -> LDS staging: thread owns 16-byte chunk (tid%8) of rows tid/8 + 32*i --------------
    const int lrow = tid >> 3, lchunk = tid & 7;
    const uint16_t *xptr[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int r = lrow + 32 * i;
        if (r >= nrows) r = nrows - 1;
        if (MODE == 0)
            xptr[i] = xsrc + (size_t)(perm[row0 + r] / k) * d + lchunk * 8;
        else
            xptr[i] = xsrc + (size_t)(row0 + r) * I + lchunk * 8;
    }
    const uint16_t *wptr[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        int r = lrow + 32 * i;
        if (MODE == 0) {
            int col = n0 + (r & 127);
            if (col >= I) col = I - 1;
            wptr[i] = (r < 128 ? wa : wb) + ((size_t)e * I + col) * d + lchunk * 8;
        } else {
            int col = n0 + r;
            if (col >= d) col = d - 1;
            wptr[i] = wa + ((size_t)e * d + col) * I + lchunk * 8;
        }
    }
    u32x4 xr[4], wr[8];
#define GLOAD(k0)                                                                                   \
    do {                                                                                            \
        _Pragma("unroll") for (int i_ = 0; i_ < 4; ++i_) xr[i_] = *reinterpret_cast<const u32x4 *>(xptr[i_] + (k0)); \
        _Pragma("unroll") for (int i_ = 0; i_ < 8; ++i_) wr[i_] = *reinterpret_cast<const u32x4 *>(wptr[i_] + (k0)); \
    } while (0)
#define LSTORE()                                                                                    \
    do {                                                                                            \
        _Pragma("unroll") for (int i_ = 0; i_ < 4; ++i_)                                            \
            *reinterpret_cast<u32x4 *>(&Xs[(lrow + 32 * i_) * LDS_LD + lchunk * 8]) = xr[i_];       \
        _Pragma("unroll") for (int i_ = 0; i_ < 8; ++i_)                                            \
            *reinterpret_cast<u32x4 *>(&Ws[(lrow + 32 * i_) * LDS_LD + lchunk * 8]) = wr[i_];       \
    } while (0)

    f32x16 acc[2][2][2];   // [weight group][weight frag][token frag]
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int c = 0; c < 2; ++c)
#pragma unroll
                for (int q = 0; q < 16; ++q) acc[a][b][c][q] = 0.f;

    const int l32 = lane & 31, kh = lane >> 5;
    const uint16_t *ws_base = &Ws[(wn * 64 + l32) * LDS_LD + kh * 8];
    const uint16_t *xs_base = &Xs[(wm * 64 + l32) * LDS_LD + kh * 8];

    GLOAD(0);
    LSTORE();
    __syncthreads();
    const int nk = K / TK;
    for (int kt = 0; kt < nk; ++kt) {
        if (kt + 1 < nk) GLOAD((kt + 1) * TK);
#pragma unroll
        for (int kk = 0; kk < TK / 16; ++kk) {
            bf16x8 wf[2][2], xf[2];
#pragma unroll
            for (int grp = 0; grp < 2; ++grp)
#pragma unroll
                for (int fi = 0; fi < 2; ++fi)
                    wf[grp][fi] = as_frag(*reinterpret_cast<const u32x4 *>(ws_base + (grp * 128 + fi * 32) * LDS_LD + kk * 16));
#pragma unroll
            for (int fj = 0; fj < 2; ++fj)
                xf[fj] = as_frag(*reinterpret_cast<const u32x4 *>(xs_base + (fj * 32) * LDS_LD + kk * 16));
#pragma unroll
            for (int grp = 0; grp < 2; ++grp)
#pragma unroll
                for (int fi = 0; fi < 2; ++fi)
#pragma unroll
                    for (int fj = 0; fj < 2; ++fj)
                        acc[grp][fi][fj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[grp][fi], xf[fj], acc[grp][fi][fj], 0, 0, 0);
        }
        __syncthreads();
        if (kt + 1 < nk) {
            LSTORE();
            __syncthreads();
        }
    }

    // ---- epilogue: lane holds, per fragment, columns 8b + 4*(lane/32) + 0..3 of token row lane%32 ----
#pragma unroll
    for (int fj = 0; fj < 2; ++fj) {
        const int tr = wm * 64 + fj * 32 + l32;
        if (tr >= nrows) continue;
        uint16_t *orow = out + (size_t)(row0 + tr) * NOUT;
#pragma unroll
        for (int fi = 0; fi < 2; ++fi) {
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const int wrow = wn * 64 + fi * 32 + 8 * b + 4 * kh;
                if (MODE == 0) {
                    const int col = n0 + wrow;
                    if (col < I) {
                        u32x2 o;
                        o.x = pack_bf16x2(silu_mul(acc[0][fi][fj][4 * b + 0], acc[1][fi][fj][4 * b + 0]),
                                          silu_mul(acc[0][fi][fj][4 * b + 1], acc[1][fi][fj][4 * b + 1]));
                        o.y = pack_bf16x2(silu_mul(acc[0][fi][fj][4 * b + 2], acc[1][fi][fj][4 * b + 2]),
                                          silu_mul(acc[0][fi][fj][4 * b + 3], acc[1][fi][fj][4 * b + 3]));
                        *reinterpret_cast<u32x2 *>(orow + col) = o;
                    }
                } else {
#pragma unroll
                    for (int grp = 0; grp < 2; ++grp) {
                        const int col = n0 + grp * 128 + wrow;
                        if (col < d) {
                            u32x2 o;
                            o.x = pack_bf16x2(acc[grp][fi][fj][4 * b + 0], acc[grp][fi][fj][4 * b + 1]);
                            o.y = pack_bf16x2(acc[grp][fi][fj][4 * b + 2], acc[grp][fi][fj][4 * b + 3]);
                            *reinterpret_cast<u32x2 *>(orow + col) = o;
                        }
                    }
                }
            }
        }
    }
}

int moe_ffn_tiled_impl(const moe_shape *s, const void *h, const int32_t *perm, const int32_t *offsets,
                       const int32_t *counts, const void *w1, const void *w3, const void *w2,
                       const uint8_t *expert_mask, void *y, void *workspace, int stages, hipStream_t st)
{
    const int d = s->d, I = s->I, N = s->N, k = s->k;
    const long R = (long)s->T * k;
    if (d % TK != 0 || I % TK != 0) return MOE_EUNSUPPORTED;
    moe_ws_layout L = moe_ws(s);
    uint16_t *act = (uint16_t *)((char *)workspace + L.act);
    int32_t *sched = (int32_t *)((char *)workspace + L.sched);
    const long max_mt = R / TM + (N < R ? N : R);

    if (stages & MOE_FFN_STAGE_UP) {
        hipLaunchKernelGGL(tile_schedule_kernel, dim3(1), dim3(MOE_MAX_EXPERTS), 0, st, N, counts, expert_mask, sched);
        MOE_CHECK_LAUNCH();
        const long n_nt = (I + 127) / 128;
        hipLaunchKernelGGL(ffn_tiled_kernel<0>, dim3((unsigned)(max_mt * n_nt)), dim3(256), 0, st, d, I, k,
                           (const uint16_t *)h, perm, offsets, counts, (const uint16_t *)w1, (const uint16_t *)w3, sched, act);
        MOE_CHECK_LAUNCH();
    }
    if (stages & MOE_FFN_STAGE_DOWN) {
        const long n_nt = (d + 255) / 256;
        hipLaunchKernelGGL(ffn_tiled_kernel<1>, dim3((unsigned)(max_mt * n_nt)), dim3(256), 0, st, d, I, k,
                           (const uint16_t *)act, perm, offsets, counts, (const uint16_t *)w2, (const uint16_t *)nullptr, sched,
                           (uint16_t *)y);
        MOE_CHECK_LAUNCH();
    }
    return MOE_OK;
}
