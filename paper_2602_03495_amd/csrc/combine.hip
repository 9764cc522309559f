// Weighted combine of the expert outputs (Eq. 2 restricted to the experts placed on this GPU) for gfx950.
// One block per token; each thread owns 8 consecutive hidden features (one 16-byte bf16 load per source row),
// sums in fp32 in slot order and rounds once to bf16.  A gather, so no atomics and no ordering effects.
#include "moe_common.h"

__device__ __forceinline__ void fma8(float (&acc)[8], float w, uint4 v)
{
    acc[0] = fmaf(w, bf16_lo(v.x), acc[0]); acc[1] = fmaf(w, bf16_hi(v.x), acc[1]);
    acc[2] = fmaf(w, bf16_lo(v.y), acc[2]); acc[3] = fmaf(w, bf16_hi(v.y), acc[3]);
    acc[4] = fmaf(w, bf16_lo(v.z), acc[4]); acc[5] = fmaf(w, bf16_hi(v.z), acc[5]);
    acc[6] = fmaf(w, bf16_lo(v.w), acc[6]); acc[7] = fmaf(w, bf16_hi(v.w), acc[7]);
}

__global__ __launch_bounds__(256) void combine_kernel(int T, int d, int k, const uint16_t *__restrict__ y,
                                                      const int32_t *__restrict__ topk_idx, const float *__restrict__ topk_w,
                                                      const int32_t *__restrict__ inv_perm, const uint8_t *__restrict__ mask,
                                                      const uint16_t *__restrict__ shared_y, int n_shared,
                                                      const float *__restrict__ shared_scale, uint16_t *__restrict__ out)
{
    const int t = blockIdx.x;
    __shared__ float w_s[MOE_MAX_TOPK];
    __shared__ int p_s[MOE_MAX_TOPK];
    if (threadIdx.x < k) {
        const int r = t * k + threadIdx.x;
        const int e = topk_idx[r];
        const bool on = mask == nullptr || mask[e] != 0;
        w_s[threadIdx.x] = topk_w[r];
        p_s[threadIdx.x] = on ? inv_perm[r] : -1;
    }
    __syncthreads();
    const float sc = (n_shared > 0 && shared_scale != nullptr) ? shared_scale[t] : 1.0f;
    for (int f = threadIdx.x * 8; f < d; f += 256 * 8) {
        float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        for (int s = 0; s < k; ++s) {
            const int p = p_s[s];
            if (p >= 0) fma8(acc, w_s[s], *reinterpret_cast<const uint4 *>(y + (size_t)p * d + f));
        }
        for (int m = 0; m < n_shared; ++m)
            fma8(acc, sc, *reinterpret_cast<const uint4 *>(shared_y + ((size_t)m * T + t) * d + f));
        uint4 o;
        o.x = pack_bf16x2(acc[0], acc[1]);
        o.y = pack_bf16x2(acc[2], acc[3]);
        o.z = pack_bf16x2(acc[4], acc[5]);
        o.w = pack_bf16x2(acc[6], acc[7]);
        *reinterpret_cast<uint4 *>(out + (size_t)t * d + f) = o;
    }
}

int moe_combine_impl(const moe_shape *s, const void *y, const int32_t *topk_idx, const float *topk_w,
                     const int32_t *inv_perm, const uint8_t *expert_mask, const void *shared_y, int n_shared,
                     const float *shared_scale, void *out, hipStream_t st)
{
    hipLaunchKernelGGL(combine_kernel, dim3(s->T), dim3(256), 0, st, s->T, s->d, s->k, (const uint16_t *)y, topk_idx,
                       topk_w, inv_perm, expert_mask, (const uint16_t *)shared_y, shared_y ? n_shared : 0, shared_scale,
                       (uint16_t *)out);
    MOE_CHECK_LAUNCH();
    return MOE_OK;
}
