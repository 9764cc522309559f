/*
 * CPU oracle of the MoE expert layer.  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, per-token evaluation of the layer as the paper defines it, used to check the
 * HIP library and to time a CPU baseline.  It shares no code with the HIP path and must never be
 * called from it.  All floating-point inputs arrive as bfloat16 bit patterns (uint16) or float32
 * and are widened exactly; every sum is accumulated in double.
 *
 * What each function follows:
 *   oracle_logits      gate product x . W_g of Section "Mixture of Experts (MoE)" (the argument of
 *                      Eq. 1), optionally on the corrected features h + res_vec of the
 *                      residual-based prefetching equation (Section "Residual-Based Prefetching").
 *   oracle_select      Eq. 1: softmax over the N experts and the k highest-scoring experts.
 *   oracle_histogram   the expert workload w_i = number of tokens routed to expert i
 *                      (Introduction; Section "Greedy Assignment Strategy").
 *   oracle_top_p       the p highest-workload predicted experts chosen for prefetching
 *                      (Section "Residual-Based Prefetching", last sentence before its figure).
 *   oracle_expert_rows E(x)_i for one (token, expert) pair: a SwiGLU feed-forward network
 *                      W2 (silu(W1 x) * (W3 x)); the paper only names a feed-forward network as the usual choice.
 *   oracle_layer       Eq. 2 restricted to the experts with G_i = 1 (the assignment vector of
 *                      Section "Greedy Assignment Strategy", mutual-exclusion constraint), plus the
 *                      always-on shared experts of the model table in "Experimental Setup".
 *   oracle_res_vec     the res_vec equation of Section "Residual-Based Prefetching".
 *
 * No blocking, grouping, permutation or fused step: one token at a time, one expert at a time.
 * The only parallelism is an OpenMP "parallel for" over tokens.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static inline float bf16_to_f32(uint16_t b)
{
    uint32_t u = ((uint32_t)b) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* logits[t,e] = float( sum_j x[t,j] * W_g[e,j] ) + bias[e], with x = h, or x = float(h + res_vec)
 * when res_vec is given (the sum formed in float32 and not rounded further).
 * gate_w is [N,d]: row e holds column e of the paper's d x N matrix. */
void oracle_logits(int T, int d, int N, const uint16_t *h, const uint16_t *gate_w, const float *bias,
                   const float *res_vec, float *logits)
{
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        for (int e = 0; e < N; ++e) {
            double acc = 0.0;
            for (int j = 0; j < d; ++j) {
                float x = bf16_to_f32(h[(size_t)t * d + j]);
                if (res_vec)
                    x = x + res_vec[j];
                acc += (double)x * (double)bf16_to_f32(gate_w[(size_t)e * d + j]);
            }
            float l = (float)acc;
            if (bias)
                l = l + bias[e];
            logits[(size_t)t * N + e] = l;
        }
    }
}

/* For each token: scores = softmax(logits) over all N experts; the k experts with the highest
 * score, ordered by descending score, equal scores by ascending expert index (softmax is monotone,
 * so the order is taken on the logits).  norm_mode 0: weight = score of the selected expert;
 * norm_mode 1: the k selected scores divided by their sum. */
void oracle_select(int T, int N, int k, const float *logits, int norm_mode, int32_t *topk_idx, float *topk_w)
{
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        const float *l = logits + (size_t)t * N;
        double *p = (double *)malloc(sizeof(double) * N);
        char *taken = (char *)calloc(N, 1);
        double mx = l[0];
        for (int e = 1; e < N; ++e)
            if (l[e] > mx)
                mx = l[e];
        double den = 0.0;
        for (int e = 0; e < N; ++e) {
            p[e] = exp((double)l[e] - mx);
            den += p[e];
        }
        for (int e = 0; e < N; ++e)
            p[e] /= den;
        double sel_sum = 0.0;
        for (int s = 0; s < k; ++s) {
            int best = -1;
            for (int e = 0; e < N; ++e) {
                if (taken[e])
                    continue;
                if (best < 0 || l[e] > l[best])
                    best = e; /* strict '>' keeps the lower index among equals */
            }
            taken[best] = 1;
            topk_idx[(size_t)t * k + s] = best;
            sel_sum += p[best];
        }
        for (int s = 0; s < k; ++s) {
            double g = p[topk_idx[(size_t)t * k + s]];
            if (norm_mode == 1)
                g /= sel_sum;
            topk_w[(size_t)t * k + s] = (float)g;
        }
        free(p);
        free(taken);
    }
}

/* counts[e] = number of (token, slot) pairs routed to expert e. */
void oracle_histogram(int R, int N, const int32_t *topk_idx, int32_t *counts)
{
    for (int e = 0; e < N; ++e)
        counts[e] = 0;
    for (int r = 0; r < R; ++r)
        counts[topk_idx[r]] += 1;
}

/* The p experts with the largest counts, by descending count, equal counts by ascending index. */
void oracle_top_p(int N, const int32_t *counts, int p, int32_t *top)
{
    char *taken = (char *)calloc(N, 1);
    for (int s = 0; s < p; ++s) {
        int best = -1;
        for (int e = 0; e < N; ++e) {
            if (taken[e])
                continue;
            if (best < 0 || counts[e] > counts[best])
                best = e;
        }
        taken[best] = 1;
        top[s] = best;
    }
    free(taken);
}

/* y = W2 ( silu(W1 x) * (W3 x) ) for one token row x (bf16 bits) and one expert.
 * w1, w3: [I,d]; w2: [d,I]; all row-major bf16 bits.  act is scratch of I doubles. */
static void expert_row(int d, int I, const uint16_t *x, const uint16_t *w1, const uint16_t *w3,
                       const uint16_t *w2, double *act, double *y)
{
    for (int i = 0; i < I; ++i) {
        double g = 0.0, u = 0.0;
        for (int j = 0; j < d; ++j) {
            double xj = (double)bf16_to_f32(x[j]);
            g += (double)bf16_to_f32(w1[(size_t)i * d + j]) * xj;
            u += (double)bf16_to_f32(w3[(size_t)i * d + j]) * xj;
        }
        act[i] = g / (1.0 + exp(-g)) * u;
    }
    for (int c = 0; c < d; ++c) {
        double acc = 0.0;
        for (int i = 0; i < I; ++i)
            acc += (double)bf16_to_f32(w2[(size_t)c * I + i]) * act[i];
        y[c] = acc;
    }
}

/* Expert outputs for a list of tokens: y[n, s, :] = E_{idx[tok_n, s]}(h[tok_n]) if that expert's
 * mask bit is set, else zeros.  y is [n_tok, k, d] doubles.  mask may be NULL (all experts on). */
void oracle_expert_rows(int d, int N, int k, int I, const uint16_t *h, const int32_t *topk_idx,
                        const uint16_t *w1, const uint16_t *w3, const uint16_t *w2, const uint8_t *mask,
                        int n_tok, const int32_t *tokens, double *y)
{
    (void)N;
#pragma omp parallel for schedule(dynamic, 1) collapse(2)
    for (int n = 0; n < n_tok; ++n) {
        for (int s = 0; s < k; ++s) {
            int t = tokens[n];
            int e = topk_idx[(size_t)t * k + s];
            double *yo = y + ((size_t)n * k + s) * d;
            if (mask && !mask[e]) {
                for (int c = 0; c < d; ++c)
                    yo[c] = 0.0;
                continue;
            }
            double *act = (double *)malloc(sizeof(double) * I);
            expert_row(d, I, h + (size_t)t * d, w1 + (size_t)e * I * d, w3 + (size_t)e * I * d,
                       w2 + (size_t)e * d * I, act, yo);
            free(act);
        }
    }
}

/* Layer output for a list of tokens:
 *   out[n,:] = sum_{s<k, mask[idx[t,s]]=1} topk_w[t,s] * E_{idx[t,s]}(h[t])
 *            + sum_{m<n_shared} c_m(t) * Eshared_m(h[t])
 * with t = tokens[n].  The routed weights are NOT renormalised over the masked-on subset, so the
 * outputs of complementary masks add up to the full layer (each expert is on exactly one side).
 * shared_mode: 0 = no shared experts, 1 = c_m = 1, 2 = c = sigmoid(h[t] . w_sg) (w_sg: [d] bf16).
 * sw1, sw3: [n_shared, I_sh, d]; sw2: [n_shared, d, I_sh].  out is [n_tok, d] doubles. */
void oracle_layer(int d, int N, int k, int I, const uint16_t *h, const int32_t *topk_idx, const float *topk_w,
                  const uint16_t *w1, const uint16_t *w3, const uint16_t *w2, const uint8_t *mask,
                  int shared_mode, int n_shared, int I_sh, const uint16_t *sw1, const uint16_t *sw3,
                  const uint16_t *sw2, const uint16_t *w_sg, int n_tok, const int32_t *tokens, double *out)
{
    (void)N;
#pragma omp parallel for schedule(dynamic, 1)
    for (int n = 0; n < n_tok; ++n) {
        int t = tokens[n];
        const uint16_t *x = h + (size_t)t * d;
        double *o = out + (size_t)n * d;
        double *y = (double *)malloc(sizeof(double) * d);
        int Imax = I > I_sh ? I : I_sh;
        double *act = (double *)malloc(sizeof(double) * Imax);
        for (int c = 0; c < d; ++c)
            o[c] = 0.0;
        for (int s = 0; s < k; ++s) {
            int e = topk_idx[(size_t)t * k + s];
            if (mask && !mask[e])
                continue;
            expert_row(d, I, x, w1 + (size_t)e * I * d, w3 + (size_t)e * I * d, w2 + (size_t)e * d * I, act, y);
            double g = (double)topk_w[(size_t)t * k + s];
            for (int c = 0; c < d; ++c)
                o[c] += g * y[c];
        }
        if (shared_mode != 0) {
            double cm = 1.0;
            if (shared_mode == 2) {
                double z = 0.0;
                for (int j = 0; j < d; ++j)
                    z += (double)bf16_to_f32(x[j]) * (double)bf16_to_f32(w_sg[j]);
                cm = 1.0 / (1.0 + exp(-z));
            }
            for (int m = 0; m < n_shared; ++m) {
                expert_row(d, I_sh, x, sw1 + (size_t)m * I_sh * d, sw3 + (size_t)m * I_sh * d,
                           sw2 + (size_t)m * d * I_sh, act, y);
                for (int c = 0; c < d; ++c)
                    o[c] += cm * y[c];
            }
        }
        free(act);
        free(y);
    }
}

/* res_vec[j] = (1/n) sum_i ( h_next[i,j] - h_cur[i,j] ) over n calibration tokens. */
void oracle_res_vec(int n, int d, const uint16_t *h_cur, const uint16_t *h_next, float *res_vec)
{
    for (int j = 0; j < d; ++j) {
        double acc = 0.0;
        for (int i = 0; i < n; ++i)
            acc += (double)bf16_to_f32(h_next[(size_t)i * d + j]) - (double)bf16_to_f32(h_cur[(size_t)i * d + j]);
        res_vec[j] = (float)(acc / (double)n);
    }
}
