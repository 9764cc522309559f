// Gate, top-k, workload histogram, token permutation and next-layer workload prediction for gfx950.
//
// moe_route (Eq. 1 and the expert workload of Section "Greedy Assignment Strategy"):
//   gate_topk_kernel      16 tokens per block; logits by bf16 MFMA 16x16x32 straight from global memory
//                         (K split over the 8 waves, reduced through LDS), then softmax and top-k per token
//                         inside one wavefront: k rounds of a DPP max reduction + ballot.
//   hist_scan_perm_kernel one block per expert: register counts of the selections below / equal to the expert
//                         (= its offset and workload), then a ballot-based stable compaction of its rows.
//   Decode-sized batches (T <= 16, T*k <= 128) need no second kernel: the selecting block builds a 16-bit
//   token mask per expert in LDS, and workload, scan and permutation are popcounts of it.  With more than 16
//   experts the gate product of such a batch is first spread over one block per 16 experts and select_decode_kernel
//   (one wavefront per token) selects from the stored logits.
// moe_predict_workload (Section "Residual-Based Prefetching"):
//   the same kernels on the next layer's gate with bias'[e] = bias[e] + res_vec . W[e], so that
//   (h + res_vec) . W + bias = h . W + bias'.  Decode-sized: the fold happens inside the gate kernel and the
//   selecting block emits the workloads and their p largest.  Larger: fold_residual_kernel, gate_topk_kernel,
//   hist_top_kernel.
// moe_route_predict: both gates as two "jobs" of the same launches (blockIdx.z) at decode sizes.
#include "moe_common.h"

#define ROUTE_TOKENS 16      // tokens per block of gate_topk_kernel
#define ROUTE_THREADS 512
#define ROUTE_WAVES 8

// res_vec . W[e,:] over one wavefront: lane l takes the 8-element groups at 8l + 512m (d is a multiple of 128, so a
// group is whole or absent), each group accumulated in element order onto the lane's sum; the 64 partial sums are
// added by butterfly.  One definition for every caller, so the folded bias does not depend on the batch size.
__device__ __forceinline__ float residual_dot(int d, const float *__restrict__ res_vec, const uint16_t *__restrict__ w, int lane)
{
    float acc = 0.f;
    for (int j = lane * 8; j < d; j += 512) {
        const u32x4 pr = *reinterpret_cast<const u32x4 *>(w + j);
        const float4 r0 = *reinterpret_cast<const float4 *>(res_vec + j);
        const float4 r1 = *reinterpret_cast<const float4 *>(res_vec + j + 4);
        acc = fmaf(r0.x, bf16_lo(pr[0]), acc);
        acc = fmaf(r0.y, bf16_hi(pr[0]), acc);
        acc = fmaf(r0.z, bf16_lo(pr[1]), acc);
        acc = fmaf(r0.w, bf16_hi(pr[1]), acc);
        acc = fmaf(r1.x, bf16_lo(pr[2]), acc);
        acc = fmaf(r1.y, bf16_hi(pr[2]), acc);
        acc = fmaf(r1.z, bf16_lo(pr[3]), acc);
        acc = fmaf(r1.w, bf16_hi(pr[3]), acc);
    }
    return wave_sum(acc);
}

// The p largest workloads by descending value, equal values by ascending index; one wavefront, lane l holding the
// workloads c0 of expert l and c1 of expert l + 64.
__device__ __forceinline__ void top_p_of(int c0, int c1, int N, int p, int32_t *__restrict__ top, int lane)
{
    if (lane >= N) c0 = -1;
    if (lane + 64 >= N) c1 = -1;
    for (int s = 0; s < p; ++s) {
        int bc, bi;
        if (c0 >= c1) { bc = c0; bi = lane; } else { bc = c1; bi = lane + 64; }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            int oc = __shfl_xor(bc, o, MOE_WAVE);
            int oi = __shfl_xor(bi, o, MOE_WAVE);
            if (oc > bc || (oc == bc && oi < bi)) { bc = oc; bi = oi; }
        }
        if (bi == lane) c0 = -1;
        if (bi == lane + 64) c1 = -1;
        if (lane == 0) top[s] = bi;
    }
}

// ---------------------------------------------------------------------------------------------------
// Softmax + top-k of one token inside a wavefront: lane l holds the logits v0 of expert l and v1 of expert l + 64
// (-inf where there is no expert).  k rounds of: wave-wide max on the DPP crossbar, then the lowest expert index
// holding that value (ballot + find-first-set; the lower 64 experts are asked first), which is the tie rule "equal
// scores by ascending index".  Lane s < k returns the s-th selection and its softmax score; sel = sum of the k scores.
__device__ __forceinline__ void select_token(float v0, float v1, int N, int k, int lane, int &my_idx, float &my_p, float &sel)
{
    const float NEG = -__builtin_huge_valf();
    const float m = wave_max_dpp(fmaxf(v0, v1));
    const float p0 = v0 > NEG ? expf(v0 - m) : 0.f;
    const float p1 = v1 > NEG ? expf(v1 - m) : 0.f;
    const float den = wave_sum_dpp(p0 + p1);
    my_idx = 0;
    my_p = 0.f;
    sel = 0.f;
    float best = m;
    for (int s = 0; s < k; ++s) {
        if (s > 0) best = wave_max_dpp(fmaxf(v0, v1));
        const unsigned long long b0 = __ballot(v0 == best);
        const unsigned long long b1 = __ballot(v1 == best);
        int bi;
        if (b0 != 0ull) {
            bi = __ffsll((long long)b0) - 1;
            if (lane == bi) v0 = NEG;
        } else if (b1 != 0ull) {
            bi = __ffsll((long long)b1) - 1 + 64;
            if (lane + 64 == bi) v1 = NEG;
        } else {
            bi = N - 1;                                  // only reachable with NaN logits: stay in range
        }
        const float pb = expf(best - m) / den;           // uniform
        sel += pb;
        if (lane == s) { my_idx = bi; my_p = pb; }
    }
}

// Weight of a sigmoid-gated shared expert for one token, by one wavefront: c = 1 / (1 + exp(-(x . w_sg))).  One
// definition for every caller, so the value does not depend on which kernel evaluates it.
__device__ __forceinline__ float sigmoid_gate_of(const uint16_t *__restrict__ x, const uint16_t *__restrict__ w_sg, int d, int lane)
{
    float acc = 0.f;
    for (int j = lane * 8; j < d; j += 512) {
        uint4 a = *reinterpret_cast<const uint4 *>(x + j);
        uint4 b = *reinterpret_cast<const uint4 *>(w_sg + j);
        acc = fmaf(bf16_lo(a.x), bf16_lo(b.x), acc); acc = fmaf(bf16_hi(a.x), bf16_hi(b.x), acc);
        acc = fmaf(bf16_lo(a.y), bf16_lo(b.y), acc); acc = fmaf(bf16_hi(a.y), bf16_hi(b.y), acc);
        acc = fmaf(bf16_lo(a.z), bf16_lo(b.z), acc); acc = fmaf(bf16_hi(a.z), bf16_hi(b.z), acc);
        acc = fmaf(bf16_lo(a.w), bf16_lo(b.w), acc); acc = fmaf(bf16_hi(a.w), bf16_hi(b.w), acc);
    }
    acc = wave_sum(acc);
    return 1.0f / (1.0f + expf(-acc));
}

// Outputs of the wider layer (N + S experts, k + S slots per token: the S always-on shared experts appended, as
// append_shared_kernel writes them) that the selecting block of a decode-sized batch can write itself; S = 0: none.
struct shared_tail {
    int S, d;
    const uint16_t *h, *w_sg;          // w_sg null: weight 1
    int32_t *x_idx;
    float *x_w;
    int32_t *x_counts, *x_offsets, *x_perm, *x_inv;
};

// Histogram, scan and stable permutation of a decode-sized batch (T <= 16, R = T*k <= 128 selections in sel_idx, LDS)
// by one block.  A token selects an expert at most once, so the rows of expert e are one per selecting token, in
// token order: a 16-bit token mask per expert gives the workload (its popcount) and the rank of a row within its
// expert (the popcount below the token's bit) without any serial pass.  With perm == nullptr (a prediction) the
// workloads and the p largest of them are written instead.  Every thread of the block must call it.
// With X.S > 0 (routing only) the tables of the layer with its shared experts appended follow from the same LDS state:
// sel_w holds the combine weights of the R selections, cs is room for T floats.
__device__ __forceinline__ void decode_tables(const int *sel_idx, unsigned *tokmask, int *off_s, int T, int N, int k,
                                              int32_t *__restrict__ counts, int32_t *__restrict__ offsets,
                                              int32_t *__restrict__ perm, int32_t *__restrict__ inv_perm,
                                              int32_t *__restrict__ top, int p, const float *sel_w, float *cs,
                                              const shared_tail &X)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int R = T * k;
    if (threadIdx.x < MOE_MAX_EXPERTS) tokmask[threadIdx.x] = 0u;
    __syncthreads();
    int my_e = -1, my_t = 0;
    if ((int)threadIdx.x < R) {
        my_e = sel_idx[threadIdx.x];
        my_t = threadIdx.x / k;
        atomicOr(&tokmask[my_e], 1u << my_t);
    }
    __syncthreads();
    if (wave == 0) {
        // workloads of experts lane and lane + 64, and their exclusive prefix sums over all 128 slots
        const int c0 = lane < N ? __popc(tokmask[lane]) : 0;
        const int c1 = lane + 64 < N ? __popc(tokmask[lane + 64]) : 0;
        int s0 = c0, s1 = c1;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int u0 = __shfl_up(s0, o, MOE_WAVE), u1 = __shfl_up(s1, o, MOE_WAVE);
            if (lane >= o) { s0 += u0; s1 += u1; }
        }
        const int tot0 = __shfl(s0, 63, MOE_WAVE);
        if (lane < N) counts[lane] = c0;
        if (lane + 64 < N) counts[lane + 64] = c1;
        if (perm == nullptr) {
            // prediction: the workloads and the p largest of them (equal workloads by ascending index)
            top_p_of(c0, c1, N, p, top, lane);
        } else {
            off_s[lane] = s0 - c0;
            off_s[lane + 64] = tot0 + s1 - c1;
            if (lane < N) offsets[lane] = s0 - c0;
            if (lane + 64 < N) offsets[lane + 64] = tot0 + s1 - c1;
            if (lane == 0) offsets[N] = R;
        }
    }
    if (perm == nullptr) return;
    __syncthreads();
    int pos = 0;
    if ((int)threadIdx.x < R) {
        pos = off_s[my_e] + __popc(tokmask[my_e] & ((1u << my_t) - 1u));
        perm[pos] = threadIdx.x;
        inv_perm[threadIdx.x] = pos;
    }
    if (X.S <= 0) return;
    // ---- the same layer as N + S experts with k + S slots per token (what append_shared_kernel derives from the tables)
    const int S = X.S, kx = k + S, tid = threadIdx.x, nthreads = blockDim.x;
    for (int t = wave; t < T; t += nthreads >> 6) {
        const float c = X.w_sg != nullptr ? sigmoid_gate_of(X.h + (size_t)t * X.d, X.w_sg, X.d, lane) : 1.0f;
        if (lane == 0) cs[t] = c;
    }
    __syncthreads();
    if (tid < R) {                                             // routed slots keep their order; slot ids move to the wider stride
        const int o = my_t * kx + (tid - my_t * k);
        X.x_idx[o] = my_e;
        X.x_w[o] = sel_w[tid];
        X.x_inv[o] = pos;
        X.x_perm[pos] = tid + my_t * S;
    }
    for (int i = tid; i < T * S; i += nthreads) {              // shared expert j takes slot k + j of every token
        const int j = i / T, t = i - j * T;
        const int o = t * kx + k + j, row = R + j * T + t;
        X.x_idx[o] = N + j;
        X.x_w[o] = cs[t];
        X.x_inv[o] = row;
        X.x_perm[row] = o;
    }
    for (int e = tid; e < N + S; e += nthreads) {
        X.x_counts[e] = e < N ? __popc(tokmask[e]) : T;
        X.x_offsets[e] = e < N ? off_s[e] : R + (e - N) * T;
    }
    if (tid == 0) X.x_offsets[N + S] = R + S * T;
}

// One gate to evaluate: the layer's own (routing) or the next layer's (prediction).  A launch carries two jobs and
// blockIdx.z picks one, so that a decode step can route and predict in the same pair of launches.
struct gate_job {
    const uint16_t *gate_w;    // [N,d] bf16
    const float *bias;         // [N] or null
    const float *res_vec;      // non-null (decode-sized launches only): add res_vec . W[e] to the bias of expert e
    int norm_mode;
    int32_t *topk_idx;         // [T,k]
    float *topk_w;             // [T,k]
    int32_t *counts;           // non-null: single-block launch that also does the histogram (and, with perm, scan and permutation)
    int32_t *offsets, *perm, *inv_perm;
    const float *logits_in;    // non-null: skip the gate product, select from these [T,N] logits
    float *logits_out;         // non-null: only compute the logits of experts 16*NT*blockIdx.y .. and store them [T,N]
    int32_t *top;              // with counts and without perm: the p largest workloads
    int p;
    shared_tail x;             // x.S > 0 (with perm, decode-sized launches only): also write the tables with the shared experts appended
};

template <int NT>   // NT = ceil(N / 16) expert tiles
__global__ __launch_bounds__(ROUTE_THREADS) void gate_topk_kernel(int T, int d, int N, int k, const uint16_t *__restrict__ h,
                                                                  gate_job job0, gate_job job1)
{
    const gate_job &J = blockIdx.z == 0 ? job0 : job1;
    const uint16_t *__restrict__ gate_w = J.gate_w;
    const float *__restrict__ bias = J.bias;
    const float *__restrict__ res_vec = J.res_vec;
    const int norm_mode = J.norm_mode;
    int32_t *__restrict__ topk_idx = J.topk_idx;
    float *__restrict__ topk_w = J.topk_w;
    int32_t *__restrict__ counts = J.counts;
    int32_t *__restrict__ offsets = J.offsets;
    int32_t *__restrict__ perm = J.perm;
    int32_t *__restrict__ inv_perm = J.inv_perm;
    const float *__restrict__ logits_in = J.logits_in;
    float *__restrict__ logits_out = J.logits_out;
    int32_t *__restrict__ top = J.top;
    const int p = J.p;

    constexpr int NP = NT * 16;                       // padded expert count
    __shared__ float part[ROUTE_WAVES][ROUTE_TOKENS][NP + 1];   // per-wave partial logits
    __shared__ __attribute__((aligned(16))) float lg[ROUTE_TOKENS][NP + 4];   // reduced logits (+bias), rows 16-byte aligned

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int t0 = blockIdx.x * ROUTE_TOKENS;
    const int i = lane & 15, g = lane >> 4;
    const int e_base = logits_out != nullptr ? blockIdx.y * NP : 0;   // first expert of this block

    // ---- logits: D[token][expert] += A[token][k] * B[k][expert], 32 k per MFMA -------------------
    int tr = t0 + i;
    if (tr >= T) tr = T - 1;
    const uint16_t *hp = h + (size_t)tr * d + g * 8;
    const uint16_t *wp[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        int er = e_base + nt * 16 + i;
        if (er >= N) er = N - 1;
        wp[nt] = gate_w + (size_t)er * d + g * 8;
    }
    f32x4 acc[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) acc[nt] = f32x4{0.f, 0.f, 0.f, 0.f};

    // K is dealt to the 8 waves in 32-wide steps (step s -> wave s % 8); each wave issues the loads of four of
    // its steps before the first MFMA so that the block has ~8 x 4 x (1 + NT) loads in flight (eight at a time
    // measured no faster)
    constexpr int BATCH = 4;
    const int nsteps = logits_in != nullptr ? 0 : d >> 5;
    int s = wave;
    for (; s + (BATCH - 1) * ROUTE_WAVES < nsteps; s += BATCH * ROUTE_WAVES) {
        u32x4 a[BATCH], b[BATCH][NT];
#pragma unroll
        for (int u = 0; u < BATCH; ++u) {
            a[u] = *reinterpret_cast<const u32x4 *>(hp + (s + u * ROUTE_WAVES) * 32);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) b[u][nt] = *reinterpret_cast<const u32x4 *>(wp[nt] + (s + u * ROUTE_WAVES) * 32);
        }
        __builtin_amdgcn_sched_barrier(0);      // keep every load of the batch ahead of the first MFMA
#pragma unroll
        for (int u = 0; u < BATCH; ++u)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
                acc[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_frag(a[u]), as_frag(b[u][nt]), acc[nt], 0, 0, 0);
    }
    for (; s < nsteps; s += ROUTE_WAVES) {
        bf16x8 a = as_frag(*reinterpret_cast<const u32x4 *>(hp + s * 32));
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            bf16x8 b = as_frag(*reinterpret_cast<const u32x4 *>(wp[nt] + s * 32));
            acc[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc[nt], 0, 0, 0);
        }
    }
    // bias of the block's experts, with the residual vector folded in: (h + res_vec).W + b = h.W + (res_vec.W + b)
    __shared__ float bias_s[NP];
    if (logits_in == nullptr) {
        for (int el = wave; el < NP; el += ROUTE_WAVES) {
            const int e = e_base + el;
            float b = 0.f;
            if (e < N) {
                b = bias != nullptr ? bias[e] : 0.f;
                if (res_vec != nullptr) b = residual_dot(d, res_vec, gate_w + (size_t)e * d, lane) + b;
            }
            if (lane == 0) bias_s[el] = b;
        }
    }
    if (logits_in == nullptr) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int r = 0; r < 4; ++r)
                part[wave][4 * g + r][nt * 16 + i] = acc[nt][r];
    }
    __syncthreads();
    for (int idx = threadIdx.x; idx < ROUTE_TOKENS * NP; idx += ROUTE_THREADS) {
        int tt = idx / NP, e = idx % NP;
        float v;
        if (logits_in != nullptr) {
            v = (t0 + tt < T && e < N) ? logits_in[(size_t)(t0 + tt) * N + e] : 0.f;
        } else {
            v = ((part[0][tt][e] + part[1][tt][e]) + (part[2][tt][e] + part[3][tt][e])) +
                ((part[4][tt][e] + part[5][tt][e]) + (part[6][tt][e] + part[7][tt][e]));
            if (e_base + e < N) v += bias_s[e];
        }
        if (logits_out != nullptr) {
            if (t0 + tt < T && e_base + e < N) logits_out[(size_t)(t0 + tt) * N + e_base + e] = v;
        } else {
            lg[tt][e] = v;
        }
    }
    if (logits_out != nullptr) return;
    __syncthreads();

    // ---- softmax + top-k: one wave per token, lane l owns experts l and l+64.  k rounds of: wave-wide max on the
    // DPP crossbar, then the lowest expert index holding that value (ballot + find-first-set; the lower 64 experts
    // are asked first), which is the tie rule "equal scores by ascending index".
    for (int q = 0; q < ROUTE_TOKENS / ROUTE_WAVES; ++q) {
        const int tt = wave * (ROUTE_TOKENS / ROUTE_WAVES) + q;
        const int t = t0 + tt;
        if (t >= T) break;                                   // uniform per wave
        const float NEG = -__builtin_huge_valf();
        const float v0 = lane < N ? lg[tt][lane] : NEG;
        const float v1 = (NT > 4 && lane + 64 < N) ? lg[tt][lane + 64] : NEG;
        int my_idx;
        float my_p, sel;
        select_token(v0, v1, N, k, lane, my_idx, my_p, sel);
        if (lane < k) {
            topk_idx[(size_t)t * k + lane] = my_idx;
            topk_w[(size_t)t * k + lane] = norm_mode == MOE_NORM_RENORM ? my_p / sel : my_p;
            if (counts != nullptr) {                                                                  // keep for the tail below
                reinterpret_cast<int *>(&part[0][0][0])[tt * k + lane] = my_idx;
                (&part[1][0][0])[tt * k + lane] = norm_mode == MOE_NORM_RENORM ? my_p / sel : my_p;
            }
        }
    }
    if (counts == nullptr) return;

    // ---- decode-sized batch (one block, T <= 16): histogram, scan and stable permutation right here ----------
    __shared__ unsigned tokmask[MOE_MAX_EXPERTS];
    __shared__ int off_s[MOE_MAX_EXPERTS];
    decode_tables(reinterpret_cast<const int *>(&part[0][0][0]), tokmask, off_s, T, N, k, counts, offsets, perm, inv_perm, top, p,
                  &part[1][0][0], &part[2][0][0], J.x);
}

// Selection for a decode-sized batch from stored logits [T, N] (bias already added): one wavefront per token, then
// the tables of decode_tables.  One block of 16 waves per job (blockIdx.z).
#define SELECT_THREADS 1024
__global__ __launch_bounds__(SELECT_THREADS) void select_decode_kernel(int T, int N, int k, gate_job job0, gate_job job1)
{
    const gate_job &J = blockIdx.z == 0 ? job0 : job1;
    __shared__ int sel_idx[ROUTE_TOKENS * MOE_MAX_TOPK];
    __shared__ float sel_w[ROUTE_TOKENS * MOE_MAX_TOPK], cs[ROUTE_TOKENS];
    __shared__ unsigned tokmask[MOE_MAX_EXPERTS];
    __shared__ int off_s[MOE_MAX_EXPERTS];
    const int lane = threadIdx.x & 63, t = threadIdx.x >> 6;
    if (t < T) {
        const float NEG = -__builtin_huge_valf();
        const float *row = J.logits_in + (size_t)t * N;
        const float v0 = lane < N ? row[lane] : NEG;
        const float v1 = lane + 64 < N ? row[lane + 64] : NEG;
        int my_idx;
        float my_p, sel;
        select_token(v0, v1, N, k, lane, my_idx, my_p, sel);
        if (lane < k) {
            J.topk_idx[(size_t)t * k + lane] = my_idx;
            const float wgt = J.norm_mode == MOE_NORM_RENORM ? my_p / sel : my_p;
            J.topk_w[(size_t)t * k + lane] = wgt;
            sel_idx[t * k + lane] = my_idx;
            sel_w[t * k + lane] = wgt;
        }
    }
    __syncthreads();
    decode_tables(sel_idx, tokmask, off_s, T, N, k, J.counts, J.offsets, J.perm, J.inv_perm, J.top, J.p, sel_w, cs, J.x);
}

// Selection from stored logits [T, N] for any batch size: one wavefront per token, 16 tokens per block.
__global__ __launch_bounds__(SELECT_THREADS) void select_rows_kernel(int T, int N, int k, gate_job job0, gate_job job1)
{
    const gate_job &J = blockIdx.z == 0 ? job0 : job1;
    const int lane = threadIdx.x & 63;
    const int t = blockIdx.x * (SELECT_THREADS / 64) + (threadIdx.x >> 6);
    if (t >= T) return;
    const float NEG = -__builtin_huge_valf();
    const float *row = J.logits_in + (size_t)t * N;
    const float v0 = lane < N ? row[lane] : NEG;
    const float v1 = lane + 64 < N ? row[lane + 64] : NEG;
    int my_idx;
    float my_p, sel;
    select_token(v0, v1, N, k, lane, my_idx, my_p, sel);
    if (lane < k) {
        J.topk_idx[(size_t)t * k + lane] = my_idx;
        J.topk_w[(size_t)t * k + lane] = J.norm_mode == MOE_NORM_RENORM ? my_p / sel : my_p;
    }
}

// ---------------------------------------------------------------------------------------------------
// One block per expert e.  Pass 1 counts, in registers, the selections that are below e and equal to e (their
// block-wide sums are offsets[e] and counts[e]: no global zero-fill, no cross-block atomics, no shared bins to
// fight over); pass 2 places the rows of expert e in ascending r with wave ballots, so the permutation is stable
// and the same on every run.  Selections are read 16 K at a time, 64 per thread, all loads in flight at once;
// when T*k <= 16 K both passes work from the same registers.
#define HSP_PER_THREAD 64
#define HSP_SUPER (256 * HSP_PER_THREAD)
__global__ __launch_bounds__(256) void hist_scan_perm_kernel(
    int R, int N, const int32_t *__restrict__ topk_idx, int32_t *__restrict__ counts,
    int32_t *__restrict__ offsets, int32_t *__restrict__ perm, int32_t *__restrict__ inv_perm)
{
    __shared__ int red[2][4];
    __shared__ int wave_tot[HSP_PER_THREAD / 4][4];
    __shared__ int my_off;
    const int e = blockIdx.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;

    // entry j of this thread in super-chunk c0: r = c0 + (j/4)*1024 + wave*256 + (j%4)*64 + lane
    int v[HSP_PER_THREAD];
    auto load_super = [&](int c0) {
#pragma unroll
        for (int j = 0; j < HSP_PER_THREAD; ++j) {
            const int r = c0 + (j >> 2) * 1024 + wave * 256 + (j & 3) * 64 + lane;
            v[j] = r < R ? topk_idx[r] : -1;
        }
    };
    int below = 0, equal = 0;
    for (int c0 = 0; c0 < R; c0 += HSP_SUPER) {
        load_super(c0);
#pragma unroll
        for (int j = 0; j < HSP_PER_THREAD; ++j) {
            below += (unsigned)v[j] < (unsigned)e;          // padding entries are -1 = huge unsigned
            equal += v[j] == e;
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        below += __shfl_xor(below, o, MOE_WAVE);
        equal += __shfl_xor(equal, o, MOE_WAVE);
    }
    if (lane == 0) { red[0][wave] = below; red[1][wave] = equal; }
    __syncthreads();
    if (threadIdx.x == 0) {
        const int off = red[0][0] + red[0][1] + red[0][2] + red[0][3];
        const int cnt = red[1][0] + red[1][1] + red[1][2] + red[1][3];
        my_off = off;
        counts[e] = cnt;
        offsets[e] = off;
        if (e == N - 1) offsets[N] = off + cnt;
    }
    __syncthreads();
    int base = my_off;                                      // running output position, uniform
    const unsigned long long lower = (1ull << lane) - 1ull;
    for (int c0 = 0; c0 < R; c0 += HSP_SUPER) {
        if (R > HSP_SUPER) load_super(c0);                  // otherwise v[] still holds the only super-chunk
        unsigned long long bal[HSP_PER_THREAD];
#pragma unroll
        for (int c = 0; c < HSP_PER_THREAD / 4; ++c) {
            int tot = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                bal[4 * c + j] = __ballot(v[4 * c + j] == e);
                tot += __popcll(bal[4 * c + j]);
            }
            if (lane == 0) wave_tot[c][wave] = tot;
        }
        __syncthreads();
#pragma unroll
        for (int c = 0; c < HSP_PER_THREAD / 4; ++c) {
            int pos = base;
            for (int w = 0; w < wave; ++w) pos += wave_tot[c][w];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (v[4 * c + j] == e) {
                    const int r = c0 + c * 1024 + wave * 256 + j * 64 + lane;
                    const int p = pos + __popcll(bal[4 * c + j] & lower);
                    perm[p] = r;
                    inv_perm[r] = p;
                }
                pos += __popcll(bal[4 * c + j]);
            }
            base += wave_tot[c][0] + wave_tot[c][1] + wave_tot[c][2] + wave_tot[c][3];
        }
        __syncthreads();
    }
}

// ---------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(64) void fold_residual_kernel(int d, const float *__restrict__ res_vec,
                                                           const uint16_t *__restrict__ gate_w,
                                                           const float *__restrict__ bias, float *__restrict__ bias_out)
{
    const int e = blockIdx.x, lane = threadIdx.x;
    const float acc = residual_dot(d, res_vec, gate_w + (size_t)e * d, lane);
    if (lane == 0) bias_out[e] = acc + (bias != nullptr ? bias[e] : 0.f);
}

// Workload histogram of R predicted selections and its p largest entries.  One block of 16 wavefronts, each with a
// private LDS histogram (one shared set of 128 bins serialises on the popular experts), summed in wave order.
#define HT_THREADS 1024
__global__ __launch_bounds__(HT_THREADS) void hist_top_kernel(int R, int N, int p, const int32_t *__restrict__ idx,
                                                              int32_t *__restrict__ pred_counts, int32_t *__restrict__ top)
{
    __shared__ int sub[HT_THREADS / 64][MOE_MAX_EXPERTS];
    __shared__ int hist[MOE_MAX_EXPERTS];
    const int wave = threadIdx.x >> 6;
    for (int j = threadIdx.x; j < (HT_THREADS / 64) * MOE_MAX_EXPERTS; j += HT_THREADS) (&sub[0][0])[j] = 0;
    __syncthreads();
    for (int r = threadIdx.x; r < R; r += HT_THREADS) atomicAdd(&sub[wave][idx[r] & (MOE_MAX_EXPERTS - 1)], 1);
    __syncthreads();
    if (threadIdx.x < MOE_MAX_EXPERTS) {
        int c = 0;
#pragma unroll
        for (int w = 0; w < HT_THREADS / 64; ++w) c += sub[w][threadIdx.x];
        hist[threadIdx.x] = c;
        if ((int)threadIdx.x < N) pred_counts[threadIdx.x] = c;
    }
    __syncthreads();
    if (threadIdx.x < 64) top_p_of(hist[threadIdx.x], hist[threadIdx.x + 64], N, p, top, threadIdx.x);
}

// ---------------------------------------------------------------------------------------------------
__global__ void dense_route_kernel(int T, int S, int32_t *__restrict__ counts, int32_t *__restrict__ offsets,
                                   int32_t *__restrict__ perm)
{
    const int p = blockIdx.x * blockDim.x + threadIdx.x;
    if (p < T * S) {
        int e = p / T, t = p - e * T;
        perm[p] = t * S + e;
    }
    if (p < S) { counts[p] = T; offsets[p] = p * T; }
    if (p == 0) offsets[S] = S * T;
}

__global__ __launch_bounds__(256) void shared_gate_kernel(int T, int d, const uint16_t *__restrict__ h,
                                                          const uint16_t *__restrict__ w_sg, float *__restrict__ scale)
{
    const int lane = threadIdx.x & 63;
    const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= T) return;
    const float c = sigmoid_gate_of(h + (size_t)t * d, w_sg, d, lane);
    if (lane == 0) scale[t] = c;
}

// Tables of the layer seen as N + S experts with k + S slots per token: the S always-on experts become experts
// N .. N + S - 1 and take the last S slots of every token (weight 1, or the sigmoid gate of the token), so that one
// grouped launch computes routed and shared experts alike.  One wave per token; the routed rows keep their order and
// only their slot ids move to the wider stride.
__global__ __launch_bounds__(256) void append_shared_kernel(
    int T, int d, int N, int k, int S, const uint16_t *__restrict__ h, const uint16_t *__restrict__ w_sg,
    const int32_t *__restrict__ idx, const float *__restrict__ w, const int32_t *__restrict__ counts,
    const int32_t *__restrict__ offsets, const int32_t *__restrict__ perm, const int32_t *__restrict__ inv,
    int32_t *__restrict__ x_idx, float *__restrict__ x_w, int32_t *__restrict__ x_counts, int32_t *__restrict__ x_offsets,
    int32_t *__restrict__ x_perm, int32_t *__restrict__ x_inv)
{
    const int lane = threadIdx.x & 63;
    const int R = T * k, kx = k + S;
    const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t < T) {
        float c = 1.0f;
        if (w_sg != nullptr) c = sigmoid_gate_of(h + (size_t)t * d, w_sg, d, lane);
        if (lane < kx) {
            const int o = t * kx + lane;
            if (lane < k) {
                x_idx[o] = idx[t * k + lane];
                x_w[o] = w[t * k + lane];
                x_inv[o] = inv[t * k + lane];
            } else {
                const int row = R + (lane - k) * T + t;
                x_idx[o] = N + lane - k;
                x_w[o] = c;
                x_inv[o] = row;
                x_perm[row] = o;
            }
        }
    }
    for (int i = blockIdx.x * 256 + threadIdx.x; i < R; i += gridDim.x * 256) {
        const int v = perm[i];
        x_perm[i] = v + (v / k) * S;
    }
    if (blockIdx.x == 0) {
        for (int e = threadIdx.x; e < N + S; e += 256) {
            x_counts[e] = e < N ? counts[e] : T;
            x_offsets[e] = e < N ? offsets[e] : R + (e - N) * T;
        }
        if (threadIdx.x == 0) x_offsets[N + S] = R + S * T;
    }
}

// ---------------------------------------------------------------------------------------------------
// host side
static gate_job make_job(const void *gate_w, const float *bias, int norm_mode, int32_t *topk_idx, float *topk_w)
{
    gate_job j = {};
    j.gate_w = (const uint16_t *)gate_w;
    j.bias = bias;
    j.norm_mode = norm_mode;
    j.topk_idx = topk_idx;
    j.topk_w = topk_w;
    return j;
}

// Launches the gate kernels for one job, or for two jobs side by side (decode-sized batches only: both then take the
// same path).  ws_logits[i]: [max(T,16), N] scratch of job i for the paths that store logits, or null.
static int launch_gate_topk(const moe_shape *s, const void *h, hipStream_t st, int n_jobs, gate_job *jobs, float *const *ws_logits)
{
    const int NT = (s->N + 15) / 16;
    dim3 grid((s->T + ROUTE_TOKENS - 1) / ROUTE_TOKENS, 1, n_jobs), block(ROUTE_THREADS);
    const uint16_t *hp = (const uint16_t *)h;
    gate_job sel[2] = {jobs[0], jobs[n_jobs - 1]};
    if (s->T <= ROUTE_TOKENS && NT >= 2 && ws_logits[0] != nullptr) {
        // decode-sized batch with many experts: one block would stream the whole gate matrix alone, so the gate
        // product is spread over one block per 16 experts and the selection runs from the stored logits
        gate_job lg[2];
        for (int i = 0; i < 2; ++i) {
            const int ji = i < n_jobs ? i : n_jobs - 1;
            lg[i] = make_job(jobs[ji].gate_w, jobs[ji].bias, jobs[ji].norm_mode, nullptr, nullptr);
            lg[i].res_vec = jobs[ji].res_vec;
            lg[i].logits_out = ws_logits[ji];
            sel[i].logits_in = ws_logits[ji];
        }
        hipLaunchKernelGGL(gate_topk_kernel<1>, dim3(1, NT, n_jobs), block, 0, st, s->T, s->d, s->N, s->k, hp, lg[0], lg[1]);
        MOE_CHECK_LAUNCH();
        // T <= 16 and k <= 8: at most 128 selections, so the selecting block also builds the tables
        hipLaunchKernelGGL(select_decode_kernel, dim3(1, 1, n_jobs), dim3(SELECT_THREADS), 0, st, s->T, s->N, s->k, sel[0], sel[1]);
        MOE_CHECK_LAUNCH();
        return MOE_OK;
    }
    if (s->T > ROUTE_TOKENS && NT >= 4 && ws_logits[0] != nullptr) {
        // many experts: a block that evaluated all of them for its 16 tokens would leave half the chip idle and spend
        // its time on the gate rows, so the gate product runs as (token blocks x 32-expert slices) and the selection,
        // one wavefront per token, reads the stored logits
        gate_job lg[2];
        for (int i = 0; i < 2; ++i) {
            const int ji = i < n_jobs ? i : n_jobs - 1;
            lg[i] = make_job(jobs[ji].gate_w, jobs[ji].bias, jobs[ji].norm_mode, nullptr, nullptr);
            lg[i].logits_out = ws_logits[ji];
            sel[i].logits_in = ws_logits[ji];
        }
        hipLaunchKernelGGL(gate_topk_kernel<2>, dim3(grid.x, (s->N + 31) / 32, n_jobs), block, 0, st, s->T, s->d, s->N, s->k, hp,
                           lg[0], lg[1]);
        MOE_CHECK_LAUNCH();
        hipLaunchKernelGGL(select_rows_kernel, dim3((s->T + SELECT_THREADS / 64 - 1) / (SELECT_THREADS / 64), 1, n_jobs),
                           dim3(SELECT_THREADS), 0, st, s->T, s->N, s->k, sel[0], sel[1]);
        MOE_CHECK_LAUNCH();
        return MOE_OK;
    }
#define GT(n)                                                                                                  \
    case n:                                                                                                    \
        hipLaunchKernelGGL(gate_topk_kernel<n>, grid, block, 0, st, s->T, s->d, s->N, s->k, hp, sel[0], sel[1]); \
        break;
    switch (NT) {
        GT(1) GT(2) GT(3) GT(4) GT(5) GT(6) GT(7) GT(8)
    default:
        return MOE_EUNSUPPORTED;
    }
#undef GT
    MOE_CHECK_LAUNCH();
    return MOE_OK;
}

// [16, N] fp32 logits scratch number `which` (0: routing, 1: prediction) inside the routing workspace
static float *route_logits_scratch(const moe_shape *s, void *workspace, int which)
{
    if (workspace == nullptr) return nullptr;
    moe_ws_layout L = moe_ws(s);
    return (float *)((char *)workspace + L.route + moe_align256(MOE_MAX_EXPERTS * 4) + 2 * moe_align256((size_t)s->T * s->k * 4) +
                     (size_t)which * moe_logits_scratch_bytes(s));
}

static bool single_block_routing(const moe_shape *s) { return s->T <= ROUTE_TOKENS && s->T * s->k <= 128; }

static gate_job route_job(const moe_shape *s, const void *gate_w, const float *gate_bias, int norm_mode, int32_t *topk_idx,
                          float *topk_w, int32_t *counts, int32_t *offsets, int32_t *perm, int32_t *inv_perm)
{
    gate_job j = make_job(gate_w, gate_bias, norm_mode, topk_idx, topk_w);
    if (single_block_routing(s)) {     // one block: histogram, scan and permutation in the same launch
        j.counts = counts;
        j.offsets = offsets;
        j.perm = perm;
        j.inv_perm = inv_perm;
    }
    return j;
}

// prediction job of a decode-sized batch: residual folded inside the gate kernel, histogram and top-p in the selecting block
static gate_job predict_job(const moe_shape *s, const float *res_vec, const void *next_gate_w, const float *next_gate_bias, int p,
                            int32_t *pred_counts, int32_t *top_experts, void *workspace)
{
    moe_ws_layout L = moe_ws(s);
    char *ws = (char *)workspace + L.route;
    const size_t R = (size_t)s->T * s->k;
    int32_t *idx = (int32_t *)(ws + moe_align256(MOE_MAX_EXPERTS * 4));
    float *w = (float *)(ws + moe_align256(MOE_MAX_EXPERTS * 4) + moe_align256(R * 4));
    gate_job j = make_job(next_gate_w, next_gate_bias, MOE_NORM_NONE, idx, w);
    j.res_vec = res_vec;
    j.counts = pred_counts;
    j.top = top_experts;
    j.p = p;
    return j;
}

int moe_route_impl(const moe_shape *s, const void *h, const void *gate_w, const float *gate_bias, int norm_mode,
                   int32_t *topk_idx, float *topk_w, int32_t *counts, int32_t *offsets, int32_t *perm,
                   int32_t *inv_perm, void *workspace, hipStream_t st)
{
    gate_job j = route_job(s, gate_w, gate_bias, norm_mode, topk_idx, topk_w, counts, offsets, perm, inv_perm);
    float *wl[1] = {route_logits_scratch(s, workspace, 0)};
    int rc = launch_gate_topk(s, h, st, 1, &j, wl);
    if (rc != MOE_OK || single_block_routing(s)) return rc;
    hipLaunchKernelGGL(hist_scan_perm_kernel, dim3(s->N), dim3(256), 0, st, s->T * s->k, s->N, topk_idx, counts,
                       offsets, perm, inv_perm);
    MOE_CHECK_LAUNCH();
    return MOE_OK;
}

int moe_predict_impl(const moe_shape *s, const void *h, const float *res_vec, const void *next_gate_w,
                     const float *next_gate_bias, int p, int32_t *pred_counts, int32_t *top_experts, void *workspace,
                     hipStream_t st)
{
    if (single_block_routing(s)) {
        gate_job j = predict_job(s, res_vec, next_gate_w, next_gate_bias, p, pred_counts, top_experts, workspace);
        float *wl[1] = {route_logits_scratch(s, workspace, 1)};
        return launch_gate_topk(s, h, st, 1, &j, wl);
    }
    moe_ws_layout L = moe_ws(s);
    char *ws = (char *)workspace + L.route;
    float *bias2 = (float *)ws;
    size_t R = (size_t)s->T * s->k;
    int32_t *idx = (int32_t *)(ws + moe_align256(MOE_MAX_EXPERTS * 4));
    float *w = (float *)(ws + moe_align256(MOE_MAX_EXPERTS * 4) + moe_align256(R * 4));
    hipLaunchKernelGGL(fold_residual_kernel, dim3(s->N), dim3(64), 0, st, s->d, res_vec, (const uint16_t *)next_gate_w,
                       next_gate_bias, bias2);
    MOE_CHECK_LAUNCH();
    gate_job j = make_job(next_gate_w, bias2, MOE_NORM_NONE, idx, w);
    float *wl[1] = {route_logits_scratch(s, workspace, 1)};
    int rc = launch_gate_topk(s, h, st, 1, &j, wl);
    if (rc != MOE_OK) return rc;
    hipLaunchKernelGGL(hist_top_kernel, dim3(1), dim3(HT_THREADS), 0, st, (int)R, s->N, p, idx, pred_counts, top_experts);
    MOE_CHECK_LAUNCH();
    return MOE_OK;
}

// Routing of this layer and workload prediction of the next in one pass: at decode sizes the two gates are
// evaluated by the same two launches (blockIdx.z = 0 routes, 1 predicts); larger batches run one after the other.
int moe_route_predict_impl(const moe_shape *s, const void *h, const void *gate_w, const float *gate_bias, int norm_mode,
                           int32_t *topk_idx, float *topk_w, int32_t *counts, int32_t *offsets, int32_t *perm,
                           int32_t *inv_perm, const float *res_vec, const void *next_gate_w, const float *next_gate_bias,
                           int p, int32_t *pred_counts, int32_t *top_experts, void *workspace, hipStream_t st)
{
    if (!single_block_routing(s)) {
        int rc = moe_route_impl(s, h, gate_w, gate_bias, norm_mode, topk_idx, topk_w, counts, offsets, perm, inv_perm, workspace, st);
        if (rc != MOE_OK) return rc;
        return moe_predict_impl(s, h, res_vec, next_gate_w, next_gate_bias, p, pred_counts, top_experts, workspace, st);
    }
    gate_job jobs[2] = {route_job(s, gate_w, gate_bias, norm_mode, topk_idx, topk_w, counts, offsets, perm, inv_perm),
                        predict_job(s, res_vec, next_gate_w, next_gate_bias, p, pred_counts, top_experts, workspace)};
    float *wl[2] = {route_logits_scratch(s, workspace, 0), route_logits_scratch(s, workspace, 1)};
    return launch_gate_topk(s, h, st, 2, jobs, wl);
}

int moe_dense_route_impl(const moe_shape *s, int32_t *counts, int32_t *offsets, int32_t *perm, hipStream_t st)
{
    int n = s->T * s->N;
    hipLaunchKernelGGL(dense_route_kernel, dim3((n + 255) / 256), dim3(256), 0, st, s->T, s->N, counts, offsets, perm);
    MOE_CHECK_LAUNCH();
    return MOE_OK;
}

int moe_append_shared_impl(const moe_shape *, int, const void *, const void *, const int32_t *, const float *, const int32_t *,
                           const int32_t *, const int32_t *, const int32_t *, int32_t *, float *, int32_t *, int32_t *, int32_t *,
                           int32_t *, hipStream_t);

// moe_route followed by moe_append_shared; at decode sizes the selecting block writes both sets of tables
int moe_route_shared_impl(const moe_shape *s, int n_shared, const void *h, const void *gate_w, const float *gate_bias, int norm_mode,
                          const void *w_sg, int32_t *topk_idx, float *topk_w, int32_t *counts, int32_t *offsets, int32_t *perm,
                          int32_t *inv_perm, int32_t *x_topk_idx, float *x_topk_w, int32_t *x_counts, int32_t *x_offsets,
                          int32_t *x_perm, int32_t *x_inv_perm, void *workspace, hipStream_t st)
{
    if (!single_block_routing(s)) {
        int rc = moe_route_impl(s, h, gate_w, gate_bias, norm_mode, topk_idx, topk_w, counts, offsets, perm, inv_perm, workspace, st);
        if (rc != MOE_OK) return rc;
        return moe_append_shared_impl(s, n_shared, h, w_sg, topk_idx, topk_w, counts, offsets, perm, inv_perm, x_topk_idx, x_topk_w,
                                      x_counts, x_offsets, x_perm, x_inv_perm, st);
    }
    gate_job j = route_job(s, gate_w, gate_bias, norm_mode, topk_idx, topk_w, counts, offsets, perm, inv_perm);
    j.x.S = n_shared;
    j.x.d = s->d;
    j.x.h = (const uint16_t *)h;
    j.x.w_sg = (const uint16_t *)w_sg;
    j.x.x_idx = x_topk_idx;
    j.x.x_w = x_topk_w;
    j.x.x_counts = x_counts;
    j.x.x_offsets = x_offsets;
    j.x.x_perm = x_perm;
    j.x.x_inv = x_inv_perm;
    float *wl[1] = {route_logits_scratch(s, workspace, 0)};
    return launch_gate_topk(s, h, st, 1, &j, wl);
}

int moe_shared_gate_impl(const moe_shape *s, const void *h, const void *w_sg, float *scale, hipStream_t st)
{
    hipLaunchKernelGGL(shared_gate_kernel, dim3((s->T + 3) / 4), dim3(256), 0, st, s->T, s->d, (const uint16_t *)h,
                       (const uint16_t *)w_sg, scale);
    MOE_CHECK_LAUNCH();
    return MOE_OK;
}

int moe_append_shared_impl(const moe_shape *s, int n_shared, const void *h, const void *w_sg, const int32_t *topk_idx,
                           const float *topk_w, const int32_t *counts, const int32_t *offsets, const int32_t *perm,
                           const int32_t *inv_perm, int32_t *x_topk_idx, float *x_topk_w, int32_t *x_counts,
                           int32_t *x_offsets, int32_t *x_perm, int32_t *x_inv_perm, hipStream_t st)
{
    hipLaunchKernelGGL(append_shared_kernel, dim3((s->T + 3) / 4), dim3(256), 0, st, s->T, s->d, s->N, s->k, n_shared,
                       (const uint16_t *)h, (const uint16_t *)w_sg, topk_idx, topk_w, counts, offsets, perm, inv_perm, x_topk_idx,
                       x_topk_w, x_counts, x_offsets, x_perm, x_inv_perm);
    MOE_CHECK_LAUNCH();
    return MOE_OK;
}
