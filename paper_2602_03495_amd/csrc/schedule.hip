// Host-side scheduling policies that consume the workload histograms of moe_route: the paper's Greedy Assignment
// (Alg. 1) and Workload-Aware Cache Replacement (Alg. 2).  Plain integer / float work over N <= 128 experts per
// layer; nothing here touches the GPU.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <numeric>

#include "moe_layer.h"

extern "C" {

// Expected per-expert times from workloads (Section "Greedy Assignment Strategy": t_gpu(w) = max(Trans(w), compute(w)),
// Trans(w) = 0 for w = 0 and for experts already cached on the GPU, else trans_time).
int moe_expert_times(int N, const int32_t *counts, const uint8_t *cached, float trans_time, const float *gpu_compute,
                     const float *cpu_compute, int wmax, float *t_gpu, float *t_cpu)
{
    if (N < 1 || N > MOE_MAX_EXPERTS || !counts || !gpu_compute || !cpu_compute || wmax < 0 || !t_gpu || !t_cpu) return MOE_EINVAL;
    for (int e = 0; e < N; ++e) {
        const int w = counts[e];
        if (w < 0) return MOE_EINVAL;
        if (w == 0) {                                        // not activated: costs nothing on either side
            t_gpu[e] = 0.f;
            t_cpu[e] = 0.f;
            continue;
        }
        const int wi = w < wmax ? w : wmax;                  // tables are clamped at their last entry
        const float trans = (cached != nullptr && cached[e]) ? 0.f : trans_time;
        t_gpu[e] = std::max(trans, gpu_compute[wi]);
        t_cpu[e] = cpu_compute[wi];
    }
    return MOE_OK;
}

// Alg. 1: experts in descending order of |t_gpu - t_cpu| (equal differences: ascending index); each goes to the side whose
// running total stays smaller, the GPU on a tie; experts with both times zero are not assigned.
int moe_greedy_assign(int N, const float *t_gpu, const float *t_cpu, uint8_t *G, uint8_t *C, float *T_gpu_out, float *T_cpu_out)
{
    if (N < 1 || N > MOE_MAX_EXPERTS || !t_gpu || !t_cpu || !G || !C) return MOE_EINVAL;
    int order[MOE_MAX_EXPERTS];
    std::iota(order, order + N, 0);
    std::stable_sort(order, order + N, [&](int a, int b) { return std::fabs(t_gpu[a] - t_cpu[a]) > std::fabs(t_gpu[b] - t_cpu[b]); });
    float Tg = 0.f, Tc = 0.f;
    for (int e = 0; e < N; ++e) G[e] = C[e] = 0;
    for (int i = 0; i < N; ++i) {
        const int e = order[i];
        const float g = t_gpu[e], c = t_cpu[e];
        if (g == 0.f && c == 0.f) continue;
        if (Tg + g <= Tc + c) {
            G[e] = 1;
            Tg += g;
        } else {
            C[e] = 1;
            Tc += c;
        }
    }
    if (T_gpu_out) *T_gpu_out = Tg;
    if (T_cpu_out) *T_cpu_out = Tc;
    return MOE_OK;
}

// Alg. 2, one token step: score += workload; when the window of w_size steps is complete, u_size experts change sides:
// the highest-score experts not on the GPU replace the lowest-score experts on the GPU, then the scores are reset.
// Ties: lower index first.  MOE_CACHE_GUARDED (a variant, not the paper's) stops at the first pair whose incoming score
// is not larger than the outgoing one.
int moe_cache_step(int N, int w_size, int u_size, int mode, const int32_t *workload, int64_t *score, uint8_t *on_gpu,
                   int32_t *step_in_window, int32_t *evicted, int32_t *loaded, int32_t *n_swapped)
{
    if (N < 1 || N > MOE_MAX_EXPERTS || w_size < 1 || u_size < 0 || !workload || !score || !on_gpu || !step_in_window || !n_swapped)
        return MOE_EINVAL;
    if (u_size > 0 && (!evicted || !loaded)) return MOE_EINVAL;
    if (mode != MOE_CACHE_ALWAYS && mode != MOE_CACHE_GUARDED) return MOE_EINVAL;
    *n_swapped = 0;
    for (int e = 0; e < N; ++e) score[e] += workload[e];
    *step_in_window += 1;
    if (*step_in_window < w_size) return MOE_OK;
    int cpu_ids[MOE_MAX_EXPERTS], gpu_ids[MOE_MAX_EXPERTS], nc = 0, ng = 0;
    for (int e = 0; e < N; ++e) (on_gpu[e] ? gpu_ids[ng++] : cpu_ids[nc++]) = e;
    std::stable_sort(cpu_ids, cpu_ids + nc, [&](int a, int b) { return score[a] > score[b]; });   // highest first
    std::stable_sort(gpu_ids, gpu_ids + ng, [&](int a, int b) { return score[a] < score[b]; });   // lowest first
    const int u = std::min(u_size, std::min(nc, ng));
    for (int i = 0; i < u; ++i) {
        const int in = cpu_ids[i], out = gpu_ids[i];
        if (mode == MOE_CACHE_GUARDED && score[in] <= score[out]) break;   // no gain from this or any later pair
        on_gpu[out] = 0;
        on_gpu[in] = 1;
        evicted[*n_swapped] = out;
        loaded[*n_swapped] = in;
        *n_swapped += 1;
    }
    for (int e = 0; e < N; ++e) score[e] = 0;
    *step_in_window = 0;
    return MOE_OK;
}

}   // extern "C"
