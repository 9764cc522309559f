// Grouped SwiGLU expert FFN for prefill-sized batches on gfx950.
//
// Two grouped GEMMs over the rows of the masked-on, non-empty experts:
//   up:    act[p, i] = silu(x_p . W1_e[i,:]) * (x_p . W3_e[i,:])      x_p = h[perm[p]/k, :] gathered in the tile load
//   down:  y[p, f]   = act[p,:] . W2_e[f,:]
//
// Design (what the counters said while this was built): with 128-row token tiles the kernel is bound by L2
// request throughput, not by MFMA issue, so the data path is shaped to ask L2 for as little as possible, in
// full 128-byte lines:
//   * Weights are consumed in the packed layout of moe_pack_weights: one MFMA 16x16x32 A fragment (16 weight
//     rows x 32 k) is 1 KB of contiguous memory in lane order.  Every wave owns a private set of weight rows,
//     so weights never pass through LDS: global_load_dwordx4 -> VGPR -> MFMA, prefetched 3 k32-steps ahead in
//     4 rotating register sets (the compiler's own vmcnt tracking keeps ~12 loads per wave in flight).
//   * The token tile (128 rows, shared by all 8 waves) is staged through LDS in k64 stages (16 KB each,
//     double buffered, 128-byte global requests), loaded two stages ahead so that waiting for it never
//     drains the weight prefetch queue (vmcnt retires in order).
//   * 8 waves per block (2 per SIMD, 128 fp32 accumulator registers each): one wave's barrier or load wait is
//     covered by the other's MFMAs, and the accumulators stay in place (no AGPR shuffling).
//   * The MFMA takes weight rows as A and token rows as B, so a lane ends up with 4 consecutive output columns
//     of one token: SwiGLU is applied in registers and the result leaves as one 8-byte store.
// A work item is (expert, 128-row token tile, weight tile); the item list is built on the device from
// counts/offsets/mask (tile_schedule_kernel), so empty and masked-off experts cost nothing and there is no host
// round trip.  Up to 128 tokens an expert has at most one token tile and every wave derives the list of working
// experts itself from two ballots, so no schedule kernel runs.  Block ids are remapped so that every XCD (own
// L2) works on a contiguous run of items ordered expert-major, weight tile, token tile: the token tiles that
// share a weight tile run side by side on one XCD (measured: the same items spread round-robin over the XCDs
// run up to 40 % slower, even with one token tile per expert).
// Tiles are rarely full: the launch bounds the 16-row subtiles by T and every block runs the body sized for its own
// row count (16, 32, 64, 96, 112 or 128 rows).
// What only the device knows (counts and mask) also shapes the launch there: with few working tiles the up projection
// switches to half-width items and the down projection splits the K range of its tiles over several items (fp32 partial
// sums, summed in split order by tiled_finish_kernel); with many, the schedule kernel picks the token-tile height of
// the down projection so that its items fill whole rounds of compute units.
// Each item walks K as a ring starting at an expert-dependent offset, so that the token tiles that share a weight tile
// stay in step (started at different points they run 18 % slower); the summation order is a function of the expert
// and of the number of K splits only, so results are reproducible for given inputs.
#include "moe_common.h"

#include <cstdlib>

#define TM MOE_TILE_M     // token rows per tile
#define NUM_XCD MOE_NUM_XCD
#define TILED_THREADS 512

// Tile tables, one per projection: int32 hdr[4] = {n_token_tiles, tile height, 0, 0}; then int4 per token tile
// {expert, first_tile, n_tiles_of_expert, 0}.  The up projection uses 128-row tiles.  The down projection has few
// items (8 column tiles of 512 per token tile at d = 4096), so the number of rounds the launch needs on 256 compute
// units moves its duration in steps: 27 token tiles are 216 items, one round with 40 units idle, and 30 tiles of 112
// rows are 240 items, still one round of shorter items.  The tile height of the down projection is therefore chosen
// here, on the device, from the workloads: 128, 112 or 96 rows, whichever gives the smallest (rounds x item time),
// with an item's time taken as proportional to (height + 64): its weight loads do not shrink with the tile.
__device__ __forceinline__ int sched_cost(int tiles, int n_ntc, int tm)
{
    const int items = tiles * n_ntc;
    const int rounds2 = items <= 512 ? 2 * ((items + 255) / 256) : (2 * items + 255) / 256 + 1;   // twice the rounds; beyond two rounds the last one fills unevenly anyway
    return rounds2 * (tm + 64);
}

__device__ __forceinline__ int wave_sum_int(int v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, MOE_WAVE);
    return v;
}

// exclusive prefix sum over the 128 threads of the block (two waves); *total receives the sum
__device__ __forceinline__ int block_exclusive_scan(int v, int *wave_total /* LDS, 2 ints */, int *total)
{
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    int incl = v;
#pragma unroll
    for (int o = 1; o < MOE_WAVE; o <<= 1) {
        const int t = __shfl_up(incl, o, MOE_WAVE);
        if (lane >= o) incl += t;
    }
    if (lane == MOE_WAVE - 1) wave_total[w] = incl;
    __syncthreads();
    *total = wave_total[0] + wave_total[1];
    return incl - v + (w == 1 ? wave_total[0] : 0);
}

__global__ __launch_bounds__(MOE_MAX_EXPERTS) void tile_schedule_kernel(int N, const int32_t *__restrict__ counts,
                                                                        const uint8_t *__restrict__ mask, int n_ntc_down,
                                                                        int32_t *__restrict__ sched_up,
                                                                        int32_t *__restrict__ sched_down)
{
    __shared__ int wsum[3][2], wtot[4][2];
    const int e = threadIdx.x, w = e >> 6;
    const int c = (e < N && counts[e] > 0 && (mask == nullptr || mask[e] != 0)) ? counts[e] : 0;
    const int n128 = (c + 127) / 128, n112 = (c + 111) / 112, n96 = (c + 95) / 96;
    const int s128 = wave_sum_int(n128), s112 = wave_sum_int(n112), s96 = wave_sum_int(n96);
    if ((e & 63) == 0) {
        wsum[0][w] = s128;
        wsum[1][w] = s112;
        wsum[2][w] = s96;
    }
    __syncthreads();
    // every thread takes the same decision from the same totals
    const int t128 = wsum[0][0] + wsum[0][1], t112 = wsum[1][0] + wsum[1][1], t96 = wsum[2][0] + wsum[2][1];
    int tm = 128, best = sched_cost(t128, n_ntc_down, 128);
    if (t128 * n_ntc_down >= 256) {                         // below that the K range is split instead
        const int c112 = sched_cost(t112, n_ntc_down, 112), c96 = sched_cost(t96, n_ntc_down, 96);
        if (c112 < best) { best = c112; tm = 112; }
        if (c96 < best) { best = c96; tm = 96; }
    }
    const int n_dn = tm == 128 ? n128 : tm == 112 ? n112 : n96;
    int tot_up, tot_dn;
    const int first_up = block_exclusive_scan(n128, wtot[0], &tot_up);
    const int first_dn = block_exclusive_scan(n_dn, wtot[1], &tot_dn);
    if (e == 0) {
        sched_up[0] = tot_up;
        sched_up[1] = TM;
        sched_up[2] = sched_up[3] = 0;
        sched_down[0] = tot_dn;
        sched_down[1] = tm;
        sched_down[2] = sched_down[3] = 0;
    }
    int4 *tab = reinterpret_cast<int4 *>(sched_up + 4);
#ifdef MOE_RAGGED_LAST
    {
        // full tiles of all experts first, then the ragged last tiles: a group is {expert, first list entry, tiles, first tile of the expert}
        const int nfull = c / TM, rag = (c % TM) != 0 ? 1 : 0;
        int tot_full, tot_rag;
        const int first_full = block_exclusive_scan(nfull, wtot[2], &tot_full);
        const int first_rag = tot_full + block_exclusive_scan(rag, wtot[3], &tot_rag);
        for (int j = 0; j < nfull; ++j) tab[first_full + j] = make_int4(e, first_full, nfull, 0);
        if (rag) tab[first_rag] = make_int4(e, first_rag, 1, nfull);
    }
#else
    for (int j = 0; j < n128; ++j) tab[first_up + j] = make_int4(e, first_up, n128, 0);
#endif
    tab = reinterpret_cast<int4 *>(sched_down + 4);
    for (int j = 0; j < n_dn; ++j) tab[first_dn + j] = make_int4(e, first_dn, n_dn, 0);
}

// Diagnostics: when a record buffer has been set (moe_debug_set_trace), thread 0 of every block of a tiled launch
// writes its begin / end time (constant 100 MHz clock), where it ran and what it worked on: the timeline of a launch.
// Costs one clock read per block and one scalar load of the pointer when unset.
#define MOE_TRACE_MAX_BLOCKS 65536
__device__ unsigned long long *g_moe_trace = nullptr;
extern "C" int moe_debug_set_trace(unsigned long long *records)
{
    return hipMemcpyToSymbol(HIP_SYMBOL(g_moe_trace), &records, sizeof(records)) == hipSuccess ? MOE_OK : MOE_ELAUNCH;
}
#define MOE_TRACE_BEGIN() const unsigned long long trace_t0_ = wall_clock64()
#define MOE_TRACE_END(mode_, e_, nrows_, nt_)                                                                   \
    do {                                                                                                        \
        unsigned long long *tr_ = g_moe_trace;                                                                  \
        if (tr_ != nullptr && threadIdx.x == 0 && blockIdx.x < MOE_TRACE_MAX_BLOCKS) {                          \
            unsigned hw_, xcc_;                                                                                 \
            asm volatile("s_getreg_b32 %0, hwreg(HW_REG_HW_ID)" : "=s"(hw_));                                   \
            asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc_));                                 \
            unsigned long long *r_ = tr_ + 8ull * (blockIdx.x + (mode_) * (unsigned long long)MOE_TRACE_MAX_BLOCKS); \
            r_[0] = trace_t0_; r_[1] = wall_clock64(); r_[2] = hw_; r_[3] = xcc_;                               \
            r_[4] = (e_); r_[5] = (nrows_); r_[6] = (nt_); r_[7] = 1;                                           \
        }                                                                                                       \
    } while (0)

// MODE 0: up (W1|W3 + SwiGLU -> act); a wave owns NF/2 fragments of W1 and the same NF/2 of W3.
// MODE 1: down (W2 -> y); a wave owns NF consecutive fragments of W2.
// Weight tile of a block: 8 waves x NF fragments x 16 rows.  NTT = 16-row token subtiles computed (rows past
// nrows are clamped copies whose results are dropped).
template <int MODE, int NF, int NTT, int NSETS, bool FENCED, int WAVES>
__device__ __forceinline__ void tile_body(uint16_t (*Xs)[2][TM * 32], int d, int I, int k, const uint16_t *__restrict__ xsrc,
                                          const int32_t *__restrict__ perm, const uint16_t *__restrict__ wa,
                                          const uint16_t *__restrict__ wb, uint16_t *__restrict__ out, int e, int nt,
                                          int row0, int nrows, int sp, int nsp, float *__restrict__ part, int R)
{
    constexpr int HF = MODE == 0 ? NF / 2 : NF;           // fragments per matrix per wave
    constexpr int WAVE_COLS = HF * 16;                     // output columns a wave produces
    constexpr int NT_COLS = WAVES * WAVE_COLS;             // output columns per block
    constexpr int RPP = WAVES * 8;                         // token rows one pass of the loader covers (8 threads per row)
    const int K = MODE == 0 ? d : I;
    const int NOUT = MODE == 0 ? I : d;
    const int n0 = nt * NT_COLS;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform: lets the weight addresses live in SGPRs
    const int li = lane & 15, lg = lane >> 4;
    const int kb_n = K / 32;                               // k32 blocks per weight row block
    const size_t rb_stride = (size_t)kb_n * 512;           // elements between consecutive 16-row blocks

    // ---- this wave's weight fragments: consecutive row blocks, so one pointer per matrix + a uniform stride
    // (wave-uniform byte base + a 32-bit lane offset: the loads take the scalar-base addressing form)
    const char *wp0, *wp1;
    const uint32_t wlane = lane * 16;
    {
        int col = n0 + wave * WAVE_COLS;
        if (col >= NOUT) col = NOUT - WAVE_COLS;           // a wave past the ragged edge recomputes the last columns
        // + the first k32 step of this item's share of K (MODE 1 with the K range split over nsp items)
        const size_t mat = (size_t)e * d * I + (size_t)(col >> 4) * rb_stride + (size_t)sp * (kb_n / nsp) * 512;
        wp0 = reinterpret_cast<const char *>(wa + mat);
        wp1 = MODE == 0 ? reinterpret_cast<const char *>(wb + mat) : wp0;
    }
    // ---- token tile loader: thread -> rows tid/8 + RPP j (j < XJ), 16-byte chunk tid%8 of the 128-byte k64 segment
    const int xc = tid & 7;
    constexpr int XJ = (NTT * 16 + RPP - 1) / RPP;         // loader passes over the token rows that are in use
    uint32_t xo[XJ];
#pragma unroll
    for (int j = 0; j < XJ; ++j) {
        int r = (tid >> 3) + RPP * j;
        if (r >= nrows) r = nrows - 1;
        if (MODE == 0)                                      // byte offsets: T*d < 2^31 elements keeps them in 32 bits
            xo[j] = ((uint32_t)(perm[row0 + r] / k) * (uint32_t)d + xc * 8) * 2u;
        else
            xo[j] = ((uint32_t)r * (uint32_t)I + xc * 8) * 2u;
    }
    const char *xbase = reinterpret_cast<const char *>(MODE == 0 ? xsrc : xsrc + (size_t)row0 * I + (size_t)sp * (kb_n / nsp) * 32);
    // LDS holds every 16-row x k32 subtile in MFMA fragment order with a swizzle: the 16 bytes of (row i, k chunk g) of
    // k32 half hf sit in slot 16 g + (i ^ g ^ 8 hf).  A fragment read is then one KB per wave, and the LDS serves a
    // 16-byte-per-lane read in four passes of 16 lanes -- lanes {0-3, 12-15, 20-23, 24-27} and so on, measured -- which
    // must hit 16 different 16-byte bank groups: i ^ g keeps that (4 clocks per read instead of 8 for plain rows), while
    // the 8 chunks of one row, which one store instruction of the loader carries in 8 adjacent lanes, land in 8
    // different bank groups (16 clocks per store instead of 64 for the unswizzled fragment order).
    uint16_t *xw = &Xs[0][xc >> 2][(tid >> 7) * 512 + ((xc & 3) * 16 + (((tid >> 3) & 15) ^ (xc & 3) ^ (xc >> 2) * 8)) * 8];   // + buffer * 2*TM*32 + j * RPP rows
    const uint16_t *xrd0 = &Xs[0][0][(lg * 16 + (li ^ lg)) * 8];       // + buffer * 2*TM*32 + t * 16 rows
    const uint16_t *xrd1 = &Xs[0][1][(lg * 16 + (li ^ lg ^ 8)) * 8];

    f32x4 acc[NF][NTT];
#pragma unroll
    for (int f = 0; f < NF; ++f)
#pragma unroll
        for (int t = 0; t < NTT; ++t) acc[f][t] = f32x4{0.f, 0.f, 0.f, 0.f};

    const int nk = kb_n / nsp;    // k32 steps of this item (a multiple of NSETS: the launch checks K)
    const int nst = nk / 2;       // k64 stages
    const int st0 = (int)(((unsigned)e * 5u) % (unsigned)nst);   // where this item's K ring starts (per expert: tiles that share rows or weights stay in step)
    static_assert(NSETS == 4 || NSETS == 8, "an even number of stages per unrolled round");
    u32x4 wr[NSETS][NF];          // W(step) lives in set step % NSETS, loaded NSETS - 1 steps ahead
    u32x4 xg[2][XJ];              // X(stage) lives in set stage % 2: loaded 2 stages ahead, stored to LDS 1 stage ahead
    bf16x8 xf[NTT];

    // Weight steps and token stages are loaded strictly in ring order, so one running position each replaces a
    // modulo per load: kw = k32 step of the next weight load, kx = k64 stage of the next token load.
    int kw = 2 * st0, kx = st0;
#ifdef MOE_NT_WEIGHTS
#define MOE_WLD(p) __builtin_nontemporal_load(p)
#else
#define MOE_WLD(p) (*(p))
#endif
#define WLOAD(set, s)                                                                            \
    do {                                                                                         \
        const size_t ko_ = (size_t)kw * 1024;                                                    \
        kw = kw + 1 == nk ? 0 : kw + 1;                                                          \
        _Pragma("unroll") for (int f = 0; f < HF; ++f) {                                         \
            wr[set][f] = MOE_WLD(reinterpret_cast<const u32x4 *>(wp0 + (f * rb_stride * 2 + ko_) + wlane)); \
            if (MODE == 0) wr[set][f + HF] = MOE_WLD(reinterpret_cast<const u32x4 *>(wp1 + (f * rb_stride * 2 + ko_) + wlane)); \
        }                                                                                        \
    } while (0)
#define XLOAD(set, st)                                                                           \
    do {                                                                                         \
        const size_t ko_ = (size_t)kx * 128;                                                     \
        kx = kx + 1 == nst ? 0 : kx + 1;                                                         \
        _Pragma("unroll") for (int j = 0; j < XJ; ++j)                                           \
            xg[set][j] = *reinterpret_cast<const u32x4 *>(xbase + ko_ + xo[j]);                  \
    } while (0)
#define XSTORE(buf)                                                                              \
    do {                                                                                         \
        _Pragma("unroll") for (int j = 0; j < XJ; ++j)                                           \
            *reinterpret_cast<u32x4 *>(xw + (buf) * (2 * TM * 32) + j * (RPP * 32)) = xg[buf][j]; \
    } while (0)
#define XREAD(buf, half)                                                                         \
    do {                                                                                         \
        _Pragma("unroll") for (int t = 0; t < NTT; ++t)                                          \
            xf[t] = as_frag(*reinterpret_cast<const u32x4 *>(((half) ? xrd1 : xrd0) + (buf) * (2 * TM * 32) + t * (16 * 32))); \
    } while (0)
    /* token subtile outermost: the first NF MFMAs need only the first LDS read, so the later reads land behind them */ \
#define MFMAS(set)                                                                               \
    do {                                                                                         \
        _Pragma("unroll") for (int t = 0; t < NTT; ++t)                                          \
            _Pragma("unroll") for (int f = 0; f < NF; ++f)                                       \
                acc[f][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_frag(wr[set][f]), xf[t], acc[f][t], 0, 0, 0); \
    } while (0)
    // FENCED: the compiler may not move the loads and LDS reads of a stage across its MFMA groups (measured: the wide
    // down-projection tile over a long K runs 4-6 % faster that way, short-K launches 4-8 % slower)
#define FENCE()                                                                                  \
    do {                                                                                         \
        if (FENCED) __builtin_amdgcn_sched_barrier(0);                                           \
    } while (0)
    // ... and the widest up-projection tile 3-6 % faster with the one fence between the first MFMA group of a stage and
    // the loads that follow it (compared inside one run on four layer shapes)
#define FENCE_MID()                                                                              \
    do {                                                                                         \
        if (FENCED || (MODE == 0 && NF == 4)) __builtin_amdgcn_sched_barrier(0);                 \
    } while (0)
    // Issue order asked of the scheduler for the full-size up-projection body (8 LDS fragment reads, 32 MFMAs and 6 or 4
    // global loads per half stage): two fragment reads ahead, then one read and one load after every 4 MFMAs.  Measured
    // inside one run: 5 % faster at 8192 tokens, where most tiles are full, the same at 2048.
#define SGB(mask, n) __builtin_amdgcn_sched_group_barrier(mask, n, 0)     /* 0x008 MFMA, 0x020 global load, 0x100 LDS read */
#define PIPE_HALF(n_loads)                                                                       \
    do {                                                                                         \
        if (MODE == 0 && NF == 4 && NTT == 8) {                                                  \
            SGB(0x100, 2);                                                                       \
            _Pragma("unroll") for (int i_ = 0; i_ < 6; ++i_) {                                   \
                SGB(0x008, 4);                                                                   \
                SGB(0x100, 1);                                                                   \
                if (i_ < (n_loads)) SGB(0x020, 1);                                               \
            }                                                                                    \
            SGB(0x008, 8);                                                                       \
        }                                                                                        \
    } while (0)
#define PIPE_FIRST() PIPE_HALF(6)       /* token loads of the stage + the weights of one step */
#define PIPE_SECOND() PIPE_HALF(4)
    // one stage: k32 steps in weight sets ws_ and ws_ + 1; its token rows are in LDS buffer buf
#define STAGE(buf, ws_)                                                                          \
    do {                                                                                         \
        __builtin_amdgcn_s_waitcnt(0xC07F);      /* lgkmcnt(0): this thread's LDS writes of the stage have landed */ \
        __builtin_amdgcn_s_barrier();                                                            \
        FENCE();                                                                                 \
        XLOAD(buf, 0);                            /* two stages ahead; its register set is in LDS now */          \
        WLOAD(((ws_) + NSETS - 1) % NSETS, 0);                                                   \
        XREAD(buf, 0);                                                                           \
        FENCE();                                                                                 \
        MFMAS(ws_);                                                                              \
        PIPE_FIRST();                                                                            \
        FENCE_MID();                                                                             \
        WLOAD(ws_, 0);                            /* = set (ws_ + NSETS) % NSETS */              \
        XREAD(buf, 1);                                                                           \
        FENCE();                                                                                 \
        MFMAS(((ws_) + 1) % NSETS);                                                              \
        PIPE_SECOND();                                                                           \
        XSTORE((buf) ^ 1);                        /* the next stage -> the other LDS buffer */   \
    } while (0)

    XLOAD(0, 0);
    XLOAD(1, 1);
#pragma unroll
    for (int u = 0; u < NSETS - 1; ++u) WLOAD(u, u);
    XSTORE(0);
    // a round of NSETS steps (NSETS / 2 stages, an even number, so the LDS buffer of a stage is a constant too)
    for (int s = 0; s < nk; s += NSETS) {
#pragma unroll
        for (int u = 0; u < NSETS; u += 2) STAGE((u >> 1) & 1, u);
    }
#undef STAGE
#undef PIPE_SECOND
#undef PIPE_FIRST
#undef PIPE_HALF
#undef SGB
#undef FENCE_MID
#undef FENCE
#undef MFMAS
#undef XREAD
#undef XSTORE
#undef XLOAD
#undef WLOAD
#undef MOE_WLD

    // ---- epilogue: in every 16x16 tile a lane holds weight rows 4*lg + 0..3 (= output columns) of token li
    const int colw = n0 + wave * WAVE_COLS;
    if (colw >= NOUT) return;                               // wave past the ragged edge: its columns were recomputed only
    if (MODE == 1 && nsp > 1) {
        // one of nsp partial sums over K: fp32, summed in split order by the finishing pass
#pragma unroll
        for (int t = 0; t < NTT; ++t) {
            const int tr = t * 16 + li;
            if (tr < nrows) {
                float *prow = part + ((size_t)sp * R + row0 + tr) * NOUT + colw + 4 * lg;
#pragma unroll
                for (int f = 0; f < HF; ++f) *reinterpret_cast<f32x4 *>(prow + f * 16) = acc[f][t];
            }
        }
        return;
    }
#pragma unroll
    for (int t = 0; t < NTT; ++t) {
        const int tr = t * 16 + li;
        if (tr < nrows) {
            uint16_t *orow = out + (size_t)(row0 + tr) * NOUT + colw + 4 * lg;
#pragma unroll
            for (int f = 0; f < HF; ++f) {
                u32x2 o;
                if (MODE == 0) {
                    o.x = pack_bf16x2(silu_mul(acc[f][t][0], acc[f + HF][t][0]), silu_mul(acc[f][t][1], acc[f + HF][t][1]));
                    o.y = pack_bf16x2(silu_mul(acc[f][t][2], acc[f + HF][t][2]), silu_mul(acc[f][t][3], acc[f + HF][t][3]));
                } else {
                    o.x = pack_bf16x2(acc[f][t][0], acc[f][t][1]);
                    o.y = pack_bf16x2(acc[f][t][2], acc[f][t][3]);
                }
                *reinterpret_cast<u32x2 *>(orow + f * 16) = o;
            }
        }
    }
}

// Whether the up projection runs its items at half width: twice as many items, each about 0.6 of the time (measured),
// so it pays when the rounds the launch needs on 256 compute units do not double: up to 128 items (one round either
// way), or just above a whole number of rounds (280 items: 2 rounds of wide items against 3 of narrow ones).
__device__ __forceinline__ bool up_items_narrow(int items)
{
    const int wide = (items + 255) / 256, narrow = (2 * items + 255) / 256;
    return narrow * 3 < wide * 5;
}

// NTT_MAX bounds the token subtiles a tile of this launch can need (from T); the block then runs the smallest
// body that covers its own rows, so a sparsely filled tile costs MFMA work for the rows it has.
template <int MODE, int NF, int NTT_MAX, bool DIRECT, int NSETS, bool FENCED, int WAVES>
__global__ __launch_bounds__(WAVES * 64, 2) void ffn_tiled_kernel(
    int d, int I, int k, int N, const uint16_t *__restrict__ xsrc,   // MODE 0: h [T,d]; MODE 1: act [R,I]
    const int32_t *__restrict__ perm, const int32_t *__restrict__ offsets, const int32_t *__restrict__ counts,
    const uint16_t *__restrict__ wa, const uint16_t *__restrict__ wb,   // MODE 0: packed w1, w3; MODE 1: packed w2, unused
    const int32_t *__restrict__ sched, const uint8_t *__restrict__ mask,   // DIRECT: mask instead of a schedule
    uint16_t *__restrict__ out,                                            // MODE 0: act [R,I]; MODE 1: y [R,d]
    int nsp_max, float *__restrict__ part, int R,   // MODE 1: up to nsp_max K splits per tile, partial sums in part [nsp,R,d] fp32
    int group)                                      // column tiles that alternate inside the item order of an expert (1: column tile major)
{
    __shared__ __attribute__((aligned(16))) uint16_t Xs[2][2][TM * 32];   // [buffer][k32 half][128 tokens x 32 k]
    // The up projection with its widest tile (NF = 4: 256 inner columns) can run its items with half that width instead:
    // also decided on the device (up_items_narrow).
    constexpr bool CAN_NARROW = MODE == 0 && NF == 4 && WAVES == 8;
    constexpr int NT_COLS = WAVES * 16 * (MODE == 0 ? NF / 2 : NF);
    int n_ntc = ((MODE == 0 ? I : d) + NT_COLS - 1) / NT_COLS;   // column tiles
    bool narrow = false;

    // ---- which item: (expert, token tile, column tile, K split).  The number of K splits follows from the number of
    // tiles that have work, which only the device knows (counts and mask live there)
    MOE_TRACE_BEGIN();
    int e, mt, nt, nsp = 1;
    if (DIRECT) {
        // at most one token tile per expert (T <= 128): no schedule has been built
        unsigned long long act_lo, act_hi;
        const int n_work = moe_working_experts(N, counts, mask, act_lo, act_hi);
        if (MODE == 1) nsp = moe_dev_splits(n_work * n_ntc, nsp_max);
        if (CAN_NARROW && up_items_narrow(n_work * n_ntc)) {
            narrow = true;
            n_ntc = (I + NT_COLS / 2 - 1) / (NT_COLS / 2);
        }
        if (!moe_item_of(act_lo, act_hi, n_ntc * nsp, blockIdx.x, e, nt)) return;
        mt = 0;
    } else {
        if (MODE == 1) nsp = moe_dev_splits(sched[0] * n_ntc, nsp_max);
        if (CAN_NARROW && up_items_narrow(sched[0] * n_ntc)) {
            narrow = true;
            n_ntc = (I + NT_COLS / 2 - 1) / (NT_COLS / 2);
        }
        const int n_nt = n_ntc * nsp;
        const int total = sched[0] * n_nt;
        const int pid = blockIdx.x;
        if (pid >= total) return;
        const int q = total / NUM_XCD, rem = total % NUM_XCD;
        const int xcd = pid % NUM_XCD, loc = pid / NUM_XCD;
        const int L = xcd < rem ? xcd * (q + 1) + loc : rem * (q + 1) + (xcd - rem) * q + loc;
        const int4 ent = reinterpret_cast<const int4 *>(sched + 4)[L / n_nt];
        e = ent.x;
        const int local = L - ent.y * n_nt;
        // Item order inside an expert: groups of `group` column tiles; inside a group the token tiles in turn, each with
        // the group's column tiles side by side.  Blocks that follow each other in the list start close in time, so the
        // blocks that share a token tile (same mt) and those that share a weight tile (same nt) both stay near each other.
        const int per_group = group * ent.z;
        const int g0 = local / per_group, within = local - g0 * per_group;
        const int gsz = min(group, n_nt - g0 * group);         // the last group may hold fewer column tiles
        mt = ent.w + within / gsz;
        nt = g0 * group + within % gsz;
    }
    const int sp = nt % nsp;      // column tile nt / nsp, K split nt % nsp
    nt /= nsp;
    const int tmk = (DIRECT || MODE == 0) ? TM : sched[1];      // token rows per tile of this launch
    const int row0 = offsets[e] + mt * tmk;
    int nrows = counts[e] - mt * tmk;
    nrows = nrows > tmk ? tmk : nrows;
#define BODY_NS(nf_, n, ns_) tile_body<MODE, nf_, n, ns_, FENCED, WAVES>(Xs, d, I, k, xsrc, perm, wa, wb, out, e, nt, row0, nrows, sp, nsp, part, R)
#define BODY_NF(nf_, n) BODY_NS(nf_, n, NSETS)
    // tiles with few token rows do little arithmetic per weight byte: their speed is the speed of the weight stream, so
    // they prefetch further ahead (8 register sets instead of 4; the accumulators of a short tile leave the room)
#ifdef MOE_DEEP_SMALL
    const bool deep_ok = NSETS == 4 && WAVES == 8 && (((MODE == 0 ? d : I) / 32 / nsp) % 8) == 0;
#else
    const bool deep_ok = false;
#endif
#define BODY_SMALL(nf_, n)                                         \
    do {                                                           \
        if (deep_ok) BODY_NS(nf_, n, 8);                           \
        else BODY_NF(nf_, n);                                      \
    } while (0)
#define BODIES(nf_)                                                \
    do {                                                           \
        if (NTT_MAX == 1 || nrows <= 16) BODY_SMALL(nf_, 1);       \
        else if (NTT_MAX == 2 || nrows <= 32) BODY_SMALL(nf_, 2);  \
        else if (NTT_MAX == 4 || nrows <= 64) BODY_SMALL(nf_, 4);  \
        else if (nrows <= 96) BODY_NF(nf_, 6);                     \
        else if (MODE == 1 && nrows <= 112) BODY_NF(nf_, 7);       \
        else BODY_NF(nf_, 8);                                      \
    } while (0)
    if constexpr (CAN_NARROW) {
        // a ragged last column tile that fits a half-width item runs as one (I = 1408: five items of 256 + one of 128)
        if (!narrow && nt == n_ntc - 1 && I % NT_COLS != 0 && I % NT_COLS <= NT_COLS / 2) {
            narrow = true;
            nt *= 2;
        }
        if (narrow) {
            BODIES(2);
            MOE_TRACE_END(MODE, e, nrows, nt);
            return;
        }
    }
    BODIES(NF);
    MOE_TRACE_END(MODE, e, nrows, nt);
#undef BODIES
#undef BODY_SMALL
#undef BODY_NF
#undef BODY_NS
}

// y[p,:] = bf16( sum over the K splits, in split order ), when the down projection of this launch split K (the same
// device-side decision as in ffn_tiled_kernel; nothing to do otherwise: the tiles wrote y themselves)
__global__ __launch_bounds__(256) void tiled_finish_kernel(int d, int R, int N, int n_ntc, int nsp_max, int direct,
                                                           const int32_t *__restrict__ sched, const float *__restrict__ partial,
                                                           const int32_t *__restrict__ offsets, const int32_t *__restrict__ counts,
                                                           const uint8_t *__restrict__ mask, uint16_t *__restrict__ y)
{
    int tiles;
    if (direct) {
        unsigned long long act_lo, act_hi;
        tiles = moe_working_experts(N, counts, mask, act_lo, act_hi);
    } else {
        tiles = sched[0];
    }
    const int nsp = moe_dev_splits(tiles * n_ntc, nsp_max);
    if (nsp == 1) return;
    const int e = blockIdx.y, j = blockIdx.x;
    if (j >= counts[e] || (mask != nullptr && mask[e] == 0)) return;
    const size_t p = (size_t)offsets[e] + j;
    for (int f = threadIdx.x * 4; f < d; f += 1024) {
        float4 a = *reinterpret_cast<const float4 *>(partial + p * d + f);
        for (int ks = 1; ks < nsp; ++ks) {
            const float4 b = *reinterpret_cast<const float4 *>(partial + ((size_t)ks * R + p) * d + f);
            a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w;
        }
        uint2 o;
        o.x = pack_bf16x2(a.x, a.y);
        o.y = pack_bf16x2(a.z, a.w);
        *reinterpret_cast<uint2 *>(y + p * d + f) = o;
    }
}

// measurement switch: how many column tiles alternate in the item order (see the kernel); 1 = column tile major
static int tiled_item_group(int mode)
{
    static const int up = getenv("MOE_TILED_GROUP_UP") ? atoi(getenv("MOE_TILED_GROUP_UP")) : 1;
    static const int dn = getenv("MOE_TILED_GROUP_DOWN") ? atoi(getenv("MOE_TILED_GROUP_DOWN")) : 1;
    const int g = mode == 0 ? up : dn;
    return g < 1 ? 1 : g;
}

template <int MODE, int NF, int NTT, bool DIRECT, int NSETS, bool FENCED, int WAVES>
static void launch_tiled(const moe_shape *s, long max_mt, const uint16_t *x, const int32_t *perm, const int32_t *offsets,
                         const int32_t *counts, const uint16_t *wa, const uint16_t *wb, const int32_t *sched,
                         const uint8_t *mask, uint16_t *out, int nsp_max, float *part, hipStream_t st)
{
    constexpr int cols = WAVES * 16 * (MODE == 0 ? NF / 2 : NF);
    const long n_ntc = ((MODE == 0 ? s->I : s->d) + cols - 1) / cols;
    const int R = s->T * s->k;
    // blocks for the most items the device-side choice of K splits can produce: with every tile at work it takes the
    // fewest splits that reach 256 items, with fewer tiles at work there are fewer items, so this bound covers both
    long n_nt = n_ntc * nsp_max;
    if (MODE == 0 && NF == 4 && WAVES == 8) n_nt = (s->I + cols / 2 - 1) / (cols / 2);   // ... or the half-width items of the up projection
    const long n_e = s->N < (long)s->T * s->k ? s->N : (long)s->T * s->k;   // DIRECT: experts that can be non-empty
    const dim3 grid((unsigned)((DIRECT ? n_e : max_mt) * n_nt));
    hipLaunchKernelGGL((ffn_tiled_kernel<MODE, NF, NTT, DIRECT, NSETS, FENCED, WAVES>), grid, dim3(WAVES * 64), 0, st, s->d, s->I, s->k,
                       s->N, x, perm, offsets, counts, wa, wb, sched, mask, out, nsp_max, part, R, tiled_item_group(MODE));
}

// Weight fragments per wave (NF), 16-row token subtiles per tile (NTT) and weight register sets (NSETS).  An expert
// never receives more rows than there are tokens, so T bounds the subtiles in use, and up to 128 tokens every expert
// has at most one token tile, which needs no schedule; narrow weight tiles keep every compute unit busy when there
// are few token tiles, and since a narrow tile leaves a wave only NF KB per step to ask for, it prefetches further
// ahead (8 register sets, K permitting; 16 measured no better: the token loads, two stages ahead, sit between the
// weight loads in the in-order vmcnt queue and bound the useful depth).
template <int MODE>
static void dispatch_tiled(const moe_shape *s, int nf, int waves, long max_mt, const uint16_t *x, const int32_t *perm,
                           const int32_t *offsets, const int32_t *counts, const uint16_t *wa, const uint16_t *wb,
                           const int32_t *sched, const uint8_t *mask, uint16_t *out, int nsp_max, float *part, hipStream_t st)
{
    const int K = MODE == 0 ? s->d : s->I;
    const bool deep = K % (256 * nsp_max) == 0 && K >= 2048;   // a short K does not pay for the longer prologue
#define GO(NF_, NTT_, D_, NS_, F_) launch_tiled<MODE, NF_, NTT_, D_, NS_, F_, 8>(s, max_mt, x, perm, offsets, counts, wa, wb, sched, mask, out, nsp_max, part, st)
    if (waves == 4) {
        // two independent 4-wave blocks per compute unit (scheduled launches with full-height tiles only)
        launch_tiled<MODE, 4, 8, false, 4, false, 4>(s, max_mt, x, perm, offsets, counts, wa, wb, sched, mask, out, nsp_max, part, st);
        return;
    }
#define GO3(NTT_, D_)                                                          \
    do {                                                                       \
        if constexpr (MODE == 1) {                                             \
            if (nf == 1) {                                                     \
                if (deep) GO(1, NTT_, D_, 8, false);                                  \
                else GO(1, NTT_, D_, 4, false);                                       \
                break;                                                         \
            }                                                                  \
            if (nf == 2) {                                                     \
                if (deep) GO(2, NTT_, D_, 8, false);                                  \
                else GO(2, NTT_, D_, 4, false);                                       \
                break;                                                         \
            }                                                                  \
        }                                                                      \
        if constexpr (MODE == 1 && !D_) {                                      \
            if (K >= 8192) {                                                   \
                GO(4, NTT_, D_, 4, true);                                      \
                break;                                                         \
            }                                                                  \
        }                                                                      \
        GO(4, NTT_, D_, 4, false);                                             \
    } while (0)
    if (s->T <= 16) GO3(1, true);
    else if (s->T <= 32) GO3(2, true);
    else if (s->T <= 64) GO3(4, true);
    else if (s->T <= TM) GO3(8, true);
    else GO3(8, false);
#undef GO3
#undef GO
}

int moe_ffn_tiled_impl(const moe_shape *s, const void *h, const int32_t *perm, const int32_t *offsets,
                       const int32_t *counts, const void *w1, const void *w3, const void *w2,
                       const uint8_t *expert_mask, void *y, void *workspace, int stages, hipStream_t st)
{
    const int d = s->d, I = s->I, N = s->N, k = s->k;
    const long R = (long)s->T * k;
    moe_ws_layout L = moe_ws(s);
    uint16_t *act = (uint16_t *)((char *)workspace + L.act);
    int32_t *sched = (int32_t *)((char *)workspace + L.sched);                     // up projection's tile table
    int32_t *sched_down = sched + moe_sched_table_bytes(s) / 4;
    const long max_mt = R / TM + (N < R ? N : R), max_mt_down = R / MOE_TILE_M_MIN + (N < R ? N : R);
    // token tiles to expect: every expert that can be non-empty has one, large experts have several
    const long est_mt = (R + TM - 1) / TM > (N < R ? N : R) ? (R + TM - 1) / TM : (N < R ? N : R);

    // the down projection's tile shape (needed by the schedule, which the up stage builds for both)
    int nf = s->T <= MOE_SKINNY_MAX_T ? 1
             : est_mt * ((d + 511) / 512) >= 256 ? 4 : est_mt * ((d + 255) / 256) >= 256 ? 2 : 1;
    // blocks of 4 waves, two of them per compute unit, for scheduled launches (experiment switch)
    static const int env_up = getenv("MOE_TILED_WAVES_UP") ? atoi(getenv("MOE_TILED_WAVES_UP")) : 0;
    static const int env_dn = getenv("MOE_TILED_WAVES_DOWN") ? atoi(getenv("MOE_TILED_WAVES_DOWN")) : 0;
    const int waves_up = s->T > TM && env_up == 4 ? 4 : 8;
    const int waves_down = s->T > TM && env_dn == 4 && nf == 4 ? 4 : 8;
    const int n_ntc = (d + 16 * waves_down * nf - 1) / (16 * waves_down * nf);
    // The tile tables are built at the start of every call, also of one that runs the down stage alone: that call then
    // never reads a table that an earlier call did not build or built from other counts or another mask.
    if (s->T > TM) {
        hipLaunchKernelGGL(tile_schedule_kernel, dim3(1), dim3(MOE_MAX_EXPERTS), 0, st, N, counts, expert_mask, n_ntc, sched,
                           sched_down);
        MOE_CHECK_LAUNCH();
    }
    if (stages & MOE_FFN_STAGE_UP) {
        dispatch_tiled<0>(s, 4, waves_up, max_mt, (const uint16_t *)h, perm, offsets, counts, (const uint16_t *)w1,
                          (const uint16_t *)w3, sched, expert_mask, act, 1, nullptr, st);
        MOE_CHECK_LAUNCH();
    }
    if (stages & MOE_FFN_STAGE_DOWN) {
        // nf: the widest weight tile that still leaves every compute unit a block (512 columns, then 256 columns), else
        // the narrowest (128 columns); and when even that leaves compute units idle -- few experts with rows, or few of
        // them masked on -- the K range of every tile is split over up to nsp_max items (decided on the device, which
        // knows counts and mask)
        const int nsp_max = moe_tiled_down_max_splits(s);
        float *part = (float *)((char *)workspace + L.partial);
        dispatch_tiled<1>(s, nf, waves_down, max_mt_down, (const uint16_t *)act, perm, offsets, counts, (const uint16_t *)w2,
                          (const uint16_t *)nullptr, sched_down, expert_mask, (uint16_t *)y, nsp_max, part, st);
        MOE_CHECK_LAUNCH();
        if (nsp_max > 1) {
            const int max_rows = s->T < (int)R ? s->T : (int)R;
            hipLaunchKernelGGL(tiled_finish_kernel, dim3(max_rows, N), dim3(256), 0, st, d, (int)R, N, n_ntc, nsp_max,
                               s->T <= TM ? 1 : 0, sched_down, part, offsets, counts, expert_mask, (uint16_t *)y);
            MOE_CHECK_LAUNCH();
        }
    }
    return MOE_OK;
}
