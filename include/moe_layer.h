/*
 * moe_layer.h -- C ABI of the MI355X (gfx950) MoE expert-layer library.
 *
 * The library computes, on one GPU, the MoE layer that the DALI paper's offloading framework
 * schedules: the gate of Eq. 1, the per-expert token workload that drives its Greedy Assignment
 * (Alg. 1) and Workload-Aware Cache Replacement (Alg. 2), the residual-based next-layer workload
 * prediction, the expert FFNs of the experts an assignment vector G places on this GPU, and the
 * weighted combine of Eq. 2.
 *
 * Conventions (all entry points):
 *   - Pointers marked [device] are HIP device pointers, pointers marked [host] are host pointers.
 *     The caller owns every buffer, including the workspace; the library allocates nothing, keeps
 *     no pointer after a call returns and never synchronises the device.
 *   - Every call only enqueues kernels on `stream` (a hipStream_t passed as void*; NULL = the
 *     default stream) and returns.  Outputs are valid once the stream reaches that point.
 *   - "bf16" is bfloat16 stored as 16-bit words; all matrices are row-major and densely packed.
 *   - Return value: MOE_OK (0) or a negative error code.  Arguments are validated on the host
 *     before anything is launched; on an error nothing has been enqueued and no device memory has
 *     been touched.  moe_strerror() names a code.
 *   - Same inputs give bit-identical outputs from run to run (no floating-point atomics; the
 *     token permutation is stable).
 *
 * Shape limits: 1 <= k <= 8, k <= N <= 128, T >= 1, T*k < 2^31, T*d < 2^31, d a multiple of 128 (<= 8192),
 * I a multiple of 128.
 */
#ifndef MOE_LAYER_H
#define MOE_LAYER_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MOE_OK            0
#define MOE_EINVAL       -1   /* null pointer, size out of range, misaligned pointer */
#define MOE_EUNSUPPORTED -2   /* a valid request this build has no kernel for */
#define MOE_ELAUNCH      -3   /* the HIP runtime refused a launch (hipGetLastError) */
#define MOE_EWORKSPACE   -4   /* workspace pointer not 256-byte aligned */
#define MOE_ETOOLARGE    -5   /* moe_expert_ffn_static: the shape needs more scratch than the static array holds */

#define MOE_MAX_EXPERTS 128
#define MOE_MAX_TOPK      8

/* how the k selected scores become combine weights */
#define MOE_NORM_NONE   0     /* G(x)_i = softmax over all N experts at the selected expert (Eq. 1 as printed) */
#define MOE_NORM_RENORM 1     /* the k selected scores divided by their sum (= softmax over the k logits) */

/* which expert-FFN kernels to use */
#define MOE_FFN_AUTO   0      /* skinny when T <= 16 and d <= 4096, tiled otherwise */
#define MOE_FFN_TILED  1      /* LDS-tiled bf16 MFMA grouped GEMMs (prefill) */
#define MOE_FFN_SKINNY 2      /* weight-streaming path for at most 16 rows per expert (decode); needs T <= 16, d <= 4096 */

/* layout of the expert weight arrays w1, w3, w2 that the caller passes to the expert-FFN entry points */
#define MOE_WEIGHTS_ROWMAJOR 0  /* [N,I,d] / [N,d,I] row-major: not consumed by any kernel of this build (pack them first) */
#define MOE_WEIGHTS_PACKED   1  /* the MFMA-fragment order written by moe_pack_weights */

typedef struct moe_shape {
    int32_t T;              /* tokens in the batch */
    int32_t d;              /* hidden size */
    int32_t N;              /* routed experts in the layer */
    int32_t k;              /* experts selected per token */
    int32_t I;              /* expert FFN inner size */
    int32_t ffn_path;       /* MOE_FFN_* */
    int32_t weight_layout;  /* MOE_WEIGHTS_*: what the caller says w1, w3, w2 hold.  The library cannot tell the two
                               layouts apart by looking, so the caller states it: a zero-initialised shape (row-major)
                               makes moe_expert_ffn* return MOE_EUNSUPPORTED instead of multiplying garbage.  Read by
                               the expert-FFN entry points only. */
} moe_shape;

const char *moe_strerror(int code);

/* Bytes of device workspace that any call with this shape may use.  [host] pointers only. */
int moe_workspace_bytes(const moe_shape *s, size_t *bytes);

/*
 * Gate, top-k, workload histogram and token permutation (Section "Mixture of Experts (MoE)", Eq. 1;
 * the expert workload w_i of Section "Greedy Assignment Strategy").
 *
 *   logits[t,e] = sum_j h[t,j] * gate_w[e,j] (+ gate_bias[e]),  fp32 accumulation;
 *   scores      = softmax(logits[t,:]) over the N experts;
 *   topk_idx[t,0..k) = the k experts with the highest score, by descending score, equal scores by
 *                      ascending expert index;
 *   topk_w[t,s] = score of topk_idx[t,s]            (MOE_NORM_NONE)
 *               = that score / sum of the k scores  (MOE_NORM_RENORM);
 *   counts[e]   = number of (t,s) pairs with topk_idx[t,s] = e   (the expert workload);
 *   offsets[e]  = counts[0] + ... + counts[e-1], offsets[N] = T*k;
 *   perm[offsets[e] + j] = the j-th smallest r = t*k+s routed to expert e (stable grouping);
 *   inv_perm[perm[p]] = p.
 *
 * h [T,d] bf16 [device]; gate_w [N,d] bf16 [device] (row e = column e of the paper's d x N matrix W_g);
 * gate_bias [N] fp32 [device] or NULL; topk_idx [T,k] int32, topk_w [T,k] fp32, counts [N] int32,
 * offsets [N+1] int32, perm [T*k] int32, inv_perm [T*k] int32: all [device] outputs.
 * workspace [device], 256-byte aligned, >= moe_workspace_bytes() of the same shape, or NULL (then gates with many
 * experts take a slower path that evaluates all experts of 16 tokens in one block; the results are the same).
 */
int moe_route(const moe_shape *s, const void *h, const void *gate_w, const float *gate_bias, int norm_mode,
              int32_t *topk_idx, float *topk_w, int32_t *counts, int32_t *offsets, int32_t *perm,
              int32_t *inv_perm, void *workspace, void *stream);

/*
 * Residual-based next-layer workload prediction (Section "Residual-Based Prefetching", its two
 * equations and the sentence after them): the next layer's gate is applied to h + res_vec (res_vec
 * shared by all tokens), the tokens routed to each predicted expert are counted, and the p experts
 * with the highest predicted workload are listed.
 *
 *   pred_counts[e]   = number of (t,s) pairs whose predicted expert is e (s < k);
 *   top_experts[0..p) = experts by descending pred_counts, equal counts by ascending index.
 *
 * The logits are evaluated as h.W + (res_vec.W + bias), which equals (h + res_vec).W + bias up to
 * fp32 rounding; h + res_vec is never rounded to bf16.
 * h [T,d] bf16, res_vec [d] fp32 (16-byte aligned), next_gate_w [N,d] bf16, next_gate_bias [N] fp32 or NULL,
 * pred_counts [N] int32 out, top_experts [p] int32 out (1 <= p <= N): all [device].
 */
int moe_predict_workload(const moe_shape *s, const void *h, const float *res_vec, const void *next_gate_w,
                         const float *next_gate_bias, int p, int32_t *pred_counts, int32_t *top_experts,
                         void *workspace, void *stream);

/*
 * moe_route of this layer and moe_predict_workload for the next one in a single call, with the results of the two
 * calls made one after the other (same arguments, same outputs, bit for bit).  The features h are the input of
 * both gates (Section "Residual-Based Prefetching": the prediction uses the current layer's features), so at decode
 * sizes (T <= 16 and T*k <= 128) the two gates are evaluated side by side by the same pair of launches; larger
 * batches run the two calls in sequence.  workspace is required (not NULL).
 */
int moe_route_predict(const moe_shape *s, const void *h, const void *gate_w, const float *gate_bias, int norm_mode,
                      int32_t *topk_idx, float *topk_w, int32_t *counts, int32_t *offsets, int32_t *perm,
                      int32_t *inv_perm, const float *res_vec, const void *next_gate_w, const float *next_gate_bias,
                      int p, int32_t *pred_counts, int32_t *top_experts, void *workspace, void *stream);

/*
 * Expert weights are consumed in a packed, MFMA-fragment-ordered layout (the expert weights are static, so this
 * is done once when they are loaded).  moe_pack_weights converts n_mats row-major [rows, K] bf16 matrices:
 *
 *   packed[m][rb][kb][l][j] = src[m][16*rb + (l % 16)][32*kb + 8*(l / 16) + j]
 *   for rb < rows/16, kb < K/32, l < 64, j < 8
 *
 * i.e. every 1 KB block holds 16 rows x 32 k in the lane order of the A operand of v_mfma_f32_16x16x32_bf16.
 * rows must be a multiple of 16 and K a multiple of 32; src and dst [device], distinct, 16-byte aligned.
 * w1 and w3 are packed with (n_mats = N, rows = I, K = d), w2 with (n_mats = N, rows = d, K = I).
 */
int moe_pack_weights(int n_mats, int rows, int K, const void *src, void *dst, void *stream);

/*
 * Expert FFNs of the experts placed on this GPU (the experts with G_i = 1 in Section "Greedy
 * Assignment Strategy"; every selected expert is applied to the token's hidden state x,
 * Section "Mixture of Experts (MoE)").  For every expert e with expert_mask[e] != 0 and
 * counts[e] > 0, and each of its rows p in [offsets[e], offsets[e+1]):
 *
 *   x = h[perm[p] / k, :],   y[p,:] = W2_e ( silu(W1_e x) * (W3_e x) ),  silu(g) = g / (1 + exp(-g)).
 *
 * bf16 inputs, fp32 accumulation; the inner activation is rounded to bf16 once before the second
 * product.  Rows of experts that are masked off are not written.
 * h [T,d] bf16; perm [T*k], offsets [N+1], counts [N] int32 as produced by moe_route (or
 * moe_dense_route); w1, w3: [N,I,d] bf16 and w2: [N,d,I] bf16, all three PACKED by moe_pack_weights, and
 * s->weight_layout = MOE_WEIGHTS_PACKED says so (any other value: MOE_EUNSUPPORTED, nothing launched);
 * expert_mask [N] uint8 (NULL = all on);
 * y [T*k,d] bf16 out, in permuted row order: all [device].
 * The host cannot see the tables, so they are trusted: the kernels index h, y and the workspace with perm,
 * offsets and counts unchecked, and tables that do not describe a routing of T*k rows (offsets[e] + counts[e]
 * <= T*k, perm a permutation of 0 .. T*k-1) lead outside the buffers.  Only host-visible arguments are validated.
 */
int moe_expert_ffn(const moe_shape *s, const void *h, const int32_t *perm, const int32_t *offsets,
                   const int32_t *counts, const void *w1, const void *w3, const void *w2,
                   const uint8_t *expert_mask, void *y, void *workspace, void *stream);

/*
 * The same computation in two separately launchable halves, for callers that want to time or overlap them:
 * MOE_FFN_STAGE_UP writes the bf16 inner activations silu(W1 x) * (W3 x) of all rows into the workspace,
 * MOE_FFN_STAGE_DOWN multiplies them by W2 into y.  A DOWN call must follow an UP call with the same
 * arguments and workspace on the same stream; one that does not stays within its buffers (every call
 * builds its own tile tables from counts and expert_mask) but multiplies whatever activations the
 * workspace holds.  MOE_FFN_STAGE_ALL is moe_expert_ffn.
 */
#define MOE_FFN_STAGE_UP   1
#define MOE_FFN_STAGE_DOWN 2
#define MOE_FFN_STAGE_ALL  3
int moe_expert_ffn_stage(const moe_shape *s, const void *h, const int32_t *perm, const int32_t *offsets,
                         const int32_t *counts, const void *w1, const void *w3, const void *w2,
                         const uint8_t *expert_mask, void *y, void *workspace, int stages, void *stream);

/*
 * moe_expert_ffn for callers that cannot allocate device memory or carry a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and bit-identical results, but
 * the scratch (inner activations, split-K partial sums, tile tables) lives in an array that is part of the library's
 * code object: moe_static_scratch_bytes() bytes (32 MiB) on every GPU the library runs on, held until the process ends.
 * The call allocates and frees nothing.
 *   - Shapes whose moe_workspace_bytes() exceeds moe_static_scratch_bytes() are rejected with MOE_ETOOLARGE before
 *     anything is launched (all decode shapes fit: T <= 16 needs at most 3.7 MB + 8.4 MB at d = 4096, I = 14336;
 *     prefill shapes fit while T*k*I*2 bytes of activations do).
 *   - All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (different streams or
 *     threads) race; calls in stream order do not.  Nothing in the array has to start at zero: every call builds its
 *     own tile tables and writes each activation and partial sum before reading it.
 *   - The array's device address is looked up on the first call on each device (hipGetSymbolAddress, no allocation);
 *     the device that is current at the call must be the one that owns the other buffers.
 */
size_t moe_static_scratch_bytes(void);
int moe_expert_ffn_static(const moe_shape *s, const void *h, const int32_t *perm, const int32_t *offsets,
                          const int32_t *counts, const void *w1, const void *w3, const void *w2,
                          const uint8_t *expert_mask, void *y, void *stream);

/*
 * Weighted combine (Eq. 2, restricted to the experts with G_i = 1):
 *
 *   out[t,:] = sum_{s<k, expert_mask[topk_idx[t,s]] != 0} topk_w[t,s] * y[inv_perm[t*k+s], :]
 *            + shared_scale[t] * sum_{m<n_shared} shared_y[m*T + t, :]
 *
 * fp32 sum, rounded once to bf16.  The weights are not renormalised over the masked-on subset, so
 * the outputs of complementary masks add up to the whole layer (mutual-exclusion constraint on C, G).
 * y [T*k,d] bf16; topk_idx [T,k]; topk_w [T,k]; inv_perm [T*k]; expert_mask [N] uint8 or NULL;
 * shared_y [n_shared*T, d] bf16 or NULL (expert-major, as moe_expert_ffn writes it under
 * moe_dense_route); shared_scale [T] fp32 or NULL (= 1); out [T,d] bf16: all [device].  s->I unused.
 */
int moe_combine(const moe_shape *s, const void *y, const int32_t *topk_idx, const float *topk_w,
                const int32_t *inv_perm, const uint8_t *expert_mask, const void *shared_y, int n_shared,
                const float *shared_scale, void *out, void *stream);

/*
 * Routing tables of always-on shared experts (the "shared experts" column of the model table in
 * Section "Experimental Setup"): every token goes to each of the s->N (= s->k) shared experts, so
 * counts[e] = T, offsets[e] = e*T, perm[e*T + t] = t*k + e.  Lets moe_expert_ffn run them as a
 * dense layer.  Requires s->k == s->N.  All pointers [device] outputs.
 */
int moe_dense_route(const moe_shape *s, int32_t *counts, int32_t *offsets, int32_t *perm, void *stream);

/*
 * Per-token scale of a sigmoid-gated shared expert: scale[t] = 1 / (1 + exp(-(h[t,:] . w_sg))).
 * h [T,d] bf16, w_sg [d] bf16, scale [T] fp32 out: all [device].  Uses s->T and s->d only.
 */
int moe_shared_gate(const moe_shape *s, const void *h, const void *w_sg, float *scale, void *stream);

/*
 * Shared experts inside the grouped launches.  The always-on shared experts of the model table in Section
 * "Experimental Setup" enter Eq. 2 as further terms of the same sum, so a layer with N routed experts (k per token)
 * and n_shared shared ones is a layer of N + n_shared experts in which every token takes k + n_shared slots, the last
 * n_shared of them fixed.  Given the tables moe_route wrote for shape (T, N, k), this call writes the tables of that
 * wider layer:
 *
 *   x_topk_idx[t, s] = topk_idx[t, s] (s < k),  N + (s - k) (s >= k)
 *   x_topk_w[t, s]   = topk_w[t, s]   (s < k),  c(t)        (s >= k),  c(t) = 1, or 1/(1+exp(-(h[t,:] . w_sg)))
 *   x_counts[e]      = counts[e] (e < N),  T (e >= N);   x_offsets = their exclusive scan
 *   x_perm           = the routed rows in their order, then expert N + j's rows t = 0..T-1 (slot ids t*(k+n_shared)+s)
 *   x_inv_perm       = its inverse
 *
 * moe_expert_ffn and moe_combine then run with shape (T, d, N + n_shared, k + n_shared, I), weight arrays holding the
 * shared experts' matrices after the routed ones, and a mask of N + n_shared entries.  A shared expert whose inner
 * size is m * I is m shared experts of inner size I with the same weight c(t): its W1 and W3 rows and its W2 columns
 * split into m consecutive blocks (SwiGLU acts on each inner unit separately, and the down projection sums over them).
 *
 * s: the routed shape (s->I unused).  h [T,d] bf16 and w_sg [d] bf16, both 16-byte aligned, or w_sg = NULL for
 * c(t) = 1 (h is then not read).  Inputs as written by moe_route; outputs x_topk_idx, x_topk_w [T, k+n_shared],
 * x_counts [N+n_shared], x_offsets [N+n_shared+1], x_perm, x_inv_perm [T*(k+n_shared)]: all [device], none may
 * alias an input.  Errors: MOE_EINVAL for n_shared < 1, N + n_shared > MOE_MAX_EXPERTS, k + n_shared > MOE_MAX_TOPK,
 * a NULL table pointer or a misaligned h / w_sg.
 */
int moe_append_shared(const moe_shape *s, int n_shared, const void *h, const void *w_sg, const int32_t *topk_idx,
                      const float *topk_w, const int32_t *counts, const int32_t *offsets, const int32_t *perm,
                      const int32_t *inv_perm, int32_t *x_topk_idx, float *x_topk_w, int32_t *x_counts, int32_t *x_offsets,
                      int32_t *x_perm, int32_t *x_inv_perm, void *stream);

/*
 * moe_route followed by moe_append_shared in one call, with the results of the two calls made one after the other
 * (same arguments, same outputs, bit for bit: the routed tables AND the tables of the wider layer).  At decode sizes
 * (T <= 16 and T*k <= 128) the block that selects the experts writes both sets of tables, so the step has one launch
 * fewer; larger batches run the two calls in sequence.  Arguments as for the two calls (h is always read: it feeds the
 * gate); workspace as for moe_route (may be NULL).  Errors: the union of the two calls' checks.
 */
int moe_route_shared(const moe_shape *s, int n_shared, const void *h, const void *gate_w, const float *gate_bias, int norm_mode,
                     const void *w_sg, int32_t *topk_idx, float *topk_w, int32_t *counts, int32_t *offsets, int32_t *perm,
                     int32_t *inv_perm, int32_t *x_topk_idx, float *x_topk_w, int32_t *x_counts, int32_t *x_offsets,
                     int32_t *x_perm, int32_t *x_inv_perm, void *workspace, void *stream);

/*
 * Calibration of res_vec (Section "Residual-Based Prefetching", the res_vec equation): the mean, over the tokens
 * of a calibration set, of the difference between a token's input feature at the next MoE layer and at this one.
 *
 *   moe_res_vec_accumulate:  acc_sum[j] += sum over r < n of ( h_next[r,j] - h_cur[r,j] )      (float64)
 *   moe_res_vec_finish:      res_vec[j]  = (float)( acc_sum[j] / n_total )
 *
 * The calibration set may arrive in any number of batches: zero acc_sum once, accumulate every batch, finish with
 * the total number of tokens.  Sums are formed in a fixed order (no atomics), in float64.
 * h_cur, h_next [n,d] bf16 [device], 16-byte aligned, the same n tokens row by row; acc_sum [d] float64 [device],
 * in/out; workspace [device], 8-byte aligned, >= moe_res_vec_workspace_bytes(d) bytes; res_vec [d] fp32 [device]
 * out.  d a multiple of 8, 8 <= d <= 8192; n >= 0 (n = 0 changes nothing); n_total >= 1.
 * Errors: MOE_EINVAL for a NULL or misaligned pointer or a size out of range.
 */
size_t moe_res_vec_workspace_bytes(int d);
int moe_res_vec_accumulate(int n, int d, const void *h_cur, const void *h_next, double *acc_sum, void *workspace,
                           void *stream);
int moe_res_vec_finish(int d, const double *acc_sum, int64_t n_total, float *res_vec, void *stream);

/*
 * Diagnostics (not a step of the method): timeline of the tiled expert-FFN launches.  With records != NULL, every
 * block of the tiled up / down projection kernels launched afterwards on the current device writes one record of
 * 8 uint64: {begin, end (100 MHz constant clock), HW_ID register, XCC_ID register, expert, token rows of the tile,
 * column tile, 1} at records[8 * (block index + 65536 * projection)], projection 0 = up, 1 = down; blocks with an
 * index of 65536 or more write nothing.  records [device]: 2 * 65536 * 8 uint64 (8 MiB), zeroed by the caller, who
 * keeps it alive until moe_debug_set_trace(NULL).  One setting per device; launches on other streams see it too.
 */
int moe_debug_set_trace(unsigned long long *records);

/* ------------------------------------------------------------------------------------------------------------
 * Host-side scheduling policies fed by the workload histograms (all pointers [host]; nothing touches the GPU).
 * ------------------------------------------------------------------------------------------------------------ */

/*
 * Expected execution time of every expert on either side (Section "Greedy Assignment Strategy"):
 *   t_cpu[e] = cpu_compute[min(counts[e], wmax)],
 *   t_gpu[e] = max(Trans, gpu_compute[min(counts[e], wmax)]),  Trans = 0 if cached[e] else trans_time,
 * and both are 0 for counts[e] = 0 (not activated).  gpu_compute, cpu_compute: [wmax+1] profiled time tables
 * indexed by workload; cached [N] uint8 or NULL (nothing cached).
 */
int moe_expert_times(int N, const int32_t *counts, const uint8_t *cached, float trans_time, const float *gpu_compute,
                     const float *cpu_compute, int wmax, float *t_gpu, float *t_cpu);

/*
 * Greedy Assignment (Alg. 1): visit the experts in descending |t_gpu - t_cpu| (equal differences by ascending
 * index) and give each to the side with the smaller running total after adding it (the GPU when equal); experts
 * with t_gpu = t_cpu = 0 stay unassigned.  G, C: [N] uint8 outputs (G is the expert_mask of moe_expert_ffn);
 * T_gpu, T_cpu: the two totals (may be NULL).  The GPU-memory constraint is not checked, as in the algorithm.
 */
int moe_greedy_assign(int N, const float *t_gpu, const float *t_cpu, uint8_t *G, uint8_t *C, float *T_gpu, float *T_cpu);

/*
 * Workload-Aware Cache Replacement (Alg. 2), one token step of one layer.  score [N] int64 and on_gpu [N] uint8
 * are the persistent state (start with score = 0, *step_in_window = 0 and the initial cache in on_gpu).
 * workload [N] is this step's expert workload (summed over the sequences of the batch).  After every w_size steps
 * the u_size highest-score experts off the GPU replace the u_size lowest-score experts on it (the text's reading
 * of the algorithm's second TopK; equal scores by ascending index on both sides; min(u_size, experts on, experts off)
 * when a side has fewer), the i-th evicted paired with the i-th loaded; then the scores are reset.
 * mode = MOE_CACHE_ALWAYS is the algorithm as printed: the exchange happens whatever the scores are.
 * mode = MOE_CACHE_GUARDED is a variant that is not in the paper: the pairs are taken in that order only while the
 * incoming score is larger than the outgoing one.
 * evicted / loaded [u_size] receive the swapped ids, *n_swapped their number (0 on steps that do not close a window).
 * Errors: MOE_EINVAL for N outside 1..MOE_MAX_EXPERTS, w_size < 1, u_size < 0, an unknown mode, a NULL pointer
 * (evicted / loaded may be NULL when u_size = 0).
 */
#define MOE_CACHE_ALWAYS  0
#define MOE_CACHE_GUARDED 1
int moe_cache_step(int N, int w_size, int u_size, int mode, const int32_t *workload, int64_t *score, uint8_t *on_gpu,
                   int32_t *step_in_window, int32_t *evicted, int32_t *loaded, int32_t *n_swapped);

#ifdef __cplusplus
}
#endif
#endif /* MOE_LAYER_H */
