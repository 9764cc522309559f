// extern "C" boundary of the library: argument validation on the host, then the kernel launchers.
#include "moe_common.h"

#include <mutex>

int moe_route_impl(const moe_shape *, const void *, const void *, const float *, int, int32_t *, float *, int32_t *,
                   int32_t *, int32_t *, int32_t *, void *, hipStream_t);
int moe_predict_impl(const moe_shape *, const void *, const float *, const void *, const float *, int, int32_t *,
                     int32_t *, void *, hipStream_t);
int moe_dense_route_impl(const moe_shape *, int32_t *, int32_t *, int32_t *, hipStream_t);
int moe_shared_gate_impl(const moe_shape *, const void *, const void *, float *, hipStream_t);
int moe_append_shared_impl(const moe_shape *, int, const void *, const void *, const int32_t *, const float *, const int32_t *,
                           const int32_t *, const int32_t *, const int32_t *, int32_t *, float *, int32_t *, int32_t *, int32_t *,
                           int32_t *, hipStream_t);
int moe_route_shared_impl(const moe_shape *, int, const void *, const void *, const float *, int, const void *, int32_t *, float *,
                          int32_t *, int32_t *, int32_t *, int32_t *, int32_t *, float *, int32_t *, int32_t *, int32_t *, int32_t *,
                          void *, hipStream_t);
int moe_ffn_tiled_impl(const moe_shape *, const void *, const int32_t *, const int32_t *, const int32_t *, const void *,
                       const void *, const void *, const uint8_t *, void *, void *, int, hipStream_t);
int moe_ffn_skinny_impl(const moe_shape *, const void *, const int32_t *, const int32_t *, const int32_t *, const void *,
                        const void *, const void *, const uint8_t *, void *, void *, int, hipStream_t);
int moe_combine_impl(const moe_shape *, const void *, const int32_t *, const float *, const int32_t *, const uint8_t *,
                     const void *, int, const float *, void *, hipStream_t);

int moe_pack_weights_impl(int, int, int, const void *, void *, hipStream_t);
int moe_route_predict_impl(const moe_shape *, const void *, const void *, const float *, int, int32_t *, float *, int32_t *,
                           int32_t *, int32_t *, int32_t *, const float *, const void *, const float *, int, int32_t *, int32_t *,
                           void *, hipStream_t);
size_t moe_res_vec_ws_bytes(int);
int moe_res_vec_accumulate_impl(int, int, const void *, const void *, double *, void *, hipStream_t);
int moe_res_vec_finish_impl(int, const double *, long long, float *, hipStream_t);

static bool aligned16(const void *p) { return ((uintptr_t)p & 15u) == 0; }

// ---- scratch of the entry point that allocates nothing -----------------------------------------------------------
// One array per GPU, part of the loaded code object, held until the process ends.  In host code the array's name is
// only a handle: its device address is looked up once per device and that address is what the kernels receive.
#define MOE_STATIC_SCRATCH_BYTES ((size_t)32 << 20)
#define MOE_MAX_DEVICES 64
static __device__ __align__(256) unsigned char moe_static_scratch[MOE_STATIC_SCRATCH_BYTES];
static void *g_scratch_ptr[MOE_MAX_DEVICES];      // device address of the current device's copy, looked up on first use
static std::mutex g_scratch_lock;

static int static_scratch(void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MOE_MAX_DEVICES) return MOE_ELAUNCH;
    std::lock_guard<std::mutex> hold(g_scratch_lock);
    if (g_scratch_ptr[dev] == nullptr) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(moe_static_scratch)) != hipSuccess || p == nullptr) return MOE_ELAUNCH;
        if (((uintptr_t)p & 255u) != 0) return MOE_EWORKSPACE;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return MOE_OK;
}

// sizes every entry point relies on
static int check_shape(const moe_shape *s, bool need_I)
{
    if (s == nullptr) return MOE_EINVAL;
    if (s->T < 1 || s->N < 1 || s->N > MOE_MAX_EXPERTS || s->k < 1 || s->k > MOE_MAX_TOPK || s->k > s->N) return MOE_EINVAL;
    if ((long long)s->T * s->k >= (1ll << 31)) return MOE_EINVAL;
    if (s->d < 128 || s->d > 8192 || s->d % 128 != 0) return MOE_EINVAL;
    if (need_I && (s->I < 128 || s->I % 128 != 0)) return MOE_EINVAL;
    if ((long long)s->T * s->d >= (1ll << 31)) return MOE_EINVAL;
    return MOE_OK;
}

extern "C" {

const char *moe_strerror(int code)
{
    switch (code) {
    case MOE_OK: return "ok";
    case MOE_EINVAL: return "invalid argument (null or misaligned pointer, or a size out of range)";
    case MOE_EUNSUPPORTED: return "request not supported by this build (shape outside the chosen FFN path, or expert weights not declared as packed by moe_pack_weights: set moe_shape.weight_layout = MOE_WEIGHTS_PACKED)";
    case MOE_ELAUNCH: return "HIP kernel launch failed";
    case MOE_EWORKSPACE: return "workspace pointer must be 256-byte aligned";
    case MOE_ETOOLARGE: return "shape needs more scratch than the library's static scratch array holds (see moe_static_scratch_bytes)";
    default: return "unknown error code";
    }
}

int moe_workspace_bytes(const moe_shape *s, size_t *bytes)
{
    if (bytes == nullptr) return MOE_EINVAL;
    int rc = check_shape(s, true);
    if (rc != MOE_OK) return rc;
    *bytes = moe_ws(s).total;
    return MOE_OK;
}

int moe_route(const moe_shape *s, const void *h, const void *gate_w, const float *gate_bias, int norm_mode,
              int32_t *topk_idx, float *topk_w, int32_t *counts, int32_t *offsets, int32_t *perm, int32_t *inv_perm,
              void *workspace, void *stream)
{
    int rc = check_shape(s, false);
    if (rc != MOE_OK) return rc;
    if (!h || !gate_w || !topk_idx || !topk_w || !counts || !offsets || !perm || !inv_perm) return MOE_EINVAL;
    if (!aligned16(h) || !aligned16(gate_w)) return MOE_EINVAL;
    if (norm_mode != MOE_NORM_NONE && norm_mode != MOE_NORM_RENORM) return MOE_EINVAL;
    if (workspace != nullptr && ((uintptr_t)workspace & 255u) != 0) return MOE_EWORKSPACE;
    if (workspace != nullptr && (s->I < 128 || s->I % 128 != 0)) return MOE_EINVAL;    // the workspace layout depends on I
    return moe_route_impl(s, h, gate_w, gate_bias, norm_mode, topk_idx, topk_w, counts, offsets, perm, inv_perm, workspace,
                          (hipStream_t)stream);
}

int moe_predict_workload(const moe_shape *s, const void *h, const float *res_vec, const void *next_gate_w,
                         const float *next_gate_bias, int p, int32_t *pred_counts, int32_t *top_experts, void *workspace,
                         void *stream)
{
    int rc = check_shape(s, true);
    if (rc != MOE_OK) return rc;
    if (!h || !res_vec || !next_gate_w || !pred_counts || !top_experts || !workspace) return MOE_EINVAL;
    if (!aligned16(res_vec)) return MOE_EINVAL;
    if (!aligned16(h) || !aligned16(next_gate_w)) return MOE_EINVAL;
    if (p < 1 || p > s->N) return MOE_EINVAL;
    if (((uintptr_t)workspace & 255u) != 0) return MOE_EWORKSPACE;
    return moe_predict_impl(s, h, res_vec, next_gate_w, next_gate_bias, p, pred_counts, top_experts, workspace,
                            (hipStream_t)stream);
}

int moe_expert_ffn_stage(const moe_shape *s, const void *h, const int32_t *perm, const int32_t *offsets,
                         const int32_t *counts, const void *w1, const void *w3, const void *w2, const uint8_t *expert_mask,
                         void *y, void *workspace, int stages, void *stream)
{
    if (stages < 1 || stages > MOE_FFN_STAGE_ALL) return MOE_EINVAL;
    int rc = check_shape(s, true);
    if (rc != MOE_OK) return rc;
    if (!h || !perm || !offsets || !counts || !w1 || !w3 || !w2 || !y || !workspace) return MOE_EINVAL;
    if (!aligned16(h) || !aligned16(w1) || !aligned16(w3) || !aligned16(w2) || !aligned16(y)) return MOE_EINVAL;
    if (((uintptr_t)workspace & 255u) != 0) return MOE_EWORKSPACE;
    // every kernel reads the weights in the packed fragment order; row-major arrays would be multiplied as garbage
    if (s->weight_layout != MOE_WEIGHTS_PACKED) return MOE_EUNSUPPORTED;
    int path = s->ffn_path;
    // the decode path keeps a wave's share of the hidden dimension in registers: at most 4096 wide
    if (path == MOE_FFN_AUTO)
        path = s->T <= MOE_SKINNY_MAX_T && s->d <= MOE_SKINNY_WAVES * MOE_SKINNY_MAX_STEPS * 32 ? MOE_FFN_SKINNY : MOE_FFN_TILED;
    if (path == MOE_FFN_SKINNY)
        return moe_ffn_skinny_impl(s, h, perm, offsets, counts, w1, w3, w2, expert_mask, y, workspace, stages, (hipStream_t)stream);
    if (path == MOE_FFN_TILED)
        return moe_ffn_tiled_impl(s, h, perm, offsets, counts, w1, w3, w2, expert_mask, y, workspace, stages, (hipStream_t)stream);
    return MOE_EINVAL;
}

int moe_expert_ffn(const moe_shape *s, const void *h, const int32_t *perm, const int32_t *offsets, const int32_t *counts,
                   const void *w1, const void *w3, const void *w2, const uint8_t *expert_mask, void *y, void *workspace,
                   void *stream)
{
    return moe_expert_ffn_stage(s, h, perm, offsets, counts, w1, w3, w2, expert_mask, y, workspace, MOE_FFN_STAGE_ALL, stream);
}

size_t moe_static_scratch_bytes(void) { return MOE_STATIC_SCRATCH_BYTES; }

int moe_expert_ffn_static(const moe_shape *s, const void *h, const int32_t *perm, const int32_t *offsets, const int32_t *counts,
                          const void *w1, const void *w3, const void *w2, const uint8_t *expert_mask, void *y, void *stream)
{
    int rc = check_shape(s, true);
    if (rc != MOE_OK) return rc;
    if (s->weight_layout != MOE_WEIGHTS_PACKED) return MOE_EUNSUPPORTED;
    if (moe_ws(s).total > MOE_STATIC_SCRATCH_BYTES) return MOE_ETOOLARGE;
    void *scratch = nullptr;
    rc = static_scratch(&scratch);
    if (rc != MOE_OK) return rc;
    return moe_expert_ffn_stage(s, h, perm, offsets, counts, w1, w3, w2, expert_mask, y, scratch, MOE_FFN_STAGE_ALL, stream);
}

int moe_combine(const moe_shape *s, const void *y, const int32_t *topk_idx, const float *topk_w, const int32_t *inv_perm,
                const uint8_t *expert_mask, const void *shared_y, int n_shared, const float *shared_scale, void *out,
                void *stream)
{
    int rc = check_shape(s, false);
    if (rc != MOE_OK) return rc;
    if (!y || !topk_idx || !topk_w || !inv_perm || !out) return MOE_EINVAL;
    if (!aligned16(y) || !aligned16(out) || (shared_y && !aligned16(shared_y))) return MOE_EINVAL;
    if (n_shared < 0 || (shared_y && n_shared < 1)) return MOE_EINVAL;
    return moe_combine_impl(s, y, topk_idx, topk_w, inv_perm, expert_mask, shared_y, n_shared, shared_scale, out,
                            (hipStream_t)stream);
}

int moe_pack_weights(int n_mats, int rows, int K, const void *src, void *dst, void *stream)
{
    if (n_mats < 1 || rows < 16 || rows % 16 != 0 || K < 32 || K % 32 != 0) return MOE_EINVAL;
    if (!src || !dst || src == dst || !aligned16(src) || !aligned16(dst)) return MOE_EINVAL;
    return moe_pack_weights_impl(n_mats, rows, K, src, dst, (hipStream_t)stream);
}

int moe_dense_route(const moe_shape *s, int32_t *counts, int32_t *offsets, int32_t *perm, void *stream)
{
    int rc = check_shape(s, false);
    if (rc != MOE_OK) return rc;
    if (s->k != s->N) return MOE_EINVAL;
    if (!counts || !offsets || !perm) return MOE_EINVAL;
    return moe_dense_route_impl(s, counts, offsets, perm, (hipStream_t)stream);
}

int moe_shared_gate(const moe_shape *s, const void *h, const void *w_sg, float *scale, void *stream)
{
    if (s == nullptr || s->T < 1 || s->d < 128 || s->d > 8192 || s->d % 128 != 0) return MOE_EINVAL;
    if (!h || !w_sg || !scale || !aligned16(h) || !aligned16(w_sg)) return MOE_EINVAL;
    return moe_shared_gate_impl(s, h, w_sg, scale, (hipStream_t)stream);
}

int moe_append_shared(const moe_shape *s, int n_shared, const void *h, const void *w_sg, const int32_t *topk_idx,
                      const float *topk_w, const int32_t *counts, const int32_t *offsets, const int32_t *perm,
                      const int32_t *inv_perm, int32_t *x_topk_idx, float *x_topk_w, int32_t *x_counts, int32_t *x_offsets,
                      int32_t *x_perm, int32_t *x_inv_perm, void *stream)
{
    int rc = check_shape(s, false);
    if (rc != MOE_OK) return rc;
    if (n_shared < 1 || s->N + n_shared > MOE_MAX_EXPERTS || s->k + n_shared > MOE_MAX_TOPK) return MOE_EINVAL;
    if ((long long)s->T * (s->k + n_shared) >= (1ll << 31)) return MOE_EINVAL;
    if (!topk_idx || !topk_w || !counts || !offsets || !perm || !inv_perm) return MOE_EINVAL;
    if (!x_topk_idx || !x_topk_w || !x_counts || !x_offsets || !x_perm || !x_inv_perm) return MOE_EINVAL;
    if (w_sg != nullptr && (h == nullptr || !aligned16(h) || !aligned16(w_sg))) return MOE_EINVAL;
    return moe_append_shared_impl(s, n_shared, h, w_sg, topk_idx, topk_w, counts, offsets, perm, inv_perm, x_topk_idx, x_topk_w,
                                  x_counts, x_offsets, x_perm, x_inv_perm, (hipStream_t)stream);
}

int moe_route_shared(const moe_shape *s, int n_shared, const void *h, const void *gate_w, const float *gate_bias, int norm_mode,
                     const void *w_sg, int32_t *topk_idx, float *topk_w, int32_t *counts, int32_t *offsets, int32_t *perm,
                     int32_t *inv_perm, int32_t *x_topk_idx, float *x_topk_w, int32_t *x_counts, int32_t *x_offsets,
                     int32_t *x_perm, int32_t *x_inv_perm, void *workspace, void *stream)
{
    int rc = check_shape(s, false);
    if (rc != MOE_OK) return rc;
    if (!h || !gate_w || !topk_idx || !topk_w || !counts || !offsets || !perm || !inv_perm) return MOE_EINVAL;
    if (!aligned16(h) || !aligned16(gate_w)) return MOE_EINVAL;
    if (norm_mode != MOE_NORM_NONE && norm_mode != MOE_NORM_RENORM) return MOE_EINVAL;
    if (workspace != nullptr && ((uintptr_t)workspace & 255u) != 0) return MOE_EWORKSPACE;
    if (workspace != nullptr && (s->I < 128 || s->I % 128 != 0)) return MOE_EINVAL;
    if (n_shared < 1 || s->N + n_shared > MOE_MAX_EXPERTS || s->k + n_shared > MOE_MAX_TOPK) return MOE_EINVAL;
    if ((long long)s->T * (s->k + n_shared) >= (1ll << 31)) return MOE_EINVAL;
    if (!x_topk_idx || !x_topk_w || !x_counts || !x_offsets || !x_perm || !x_inv_perm) return MOE_EINVAL;
    if (w_sg != nullptr && !aligned16(w_sg)) return MOE_EINVAL;
    return moe_route_shared_impl(s, n_shared, h, gate_w, gate_bias, norm_mode, w_sg, topk_idx, topk_w, counts, offsets, perm, inv_perm,
                                 x_topk_idx, x_topk_w, x_counts, x_offsets, x_perm, x_inv_perm, workspace, (hipStream_t)stream);
}

int moe_route_predict(const moe_shape *s, const void *h, const void *gate_w, const float *gate_bias, int norm_mode,
                      int32_t *topk_idx, float *topk_w, int32_t *counts, int32_t *offsets, int32_t *perm,
                      int32_t *inv_perm, const float *res_vec, const void *next_gate_w, const float *next_gate_bias,
                      int p, int32_t *pred_counts, int32_t *top_experts, void *workspace, void *stream)
{
    int rc = check_shape(s, true);
    if (rc != MOE_OK) return rc;
    if (!h || !gate_w || !topk_idx || !topk_w || !counts || !offsets || !perm || !inv_perm) return MOE_EINVAL;
    if (!res_vec || !next_gate_w || !pred_counts || !top_experts || !workspace) return MOE_EINVAL;
    if (!aligned16(h) || !aligned16(gate_w) || !aligned16(next_gate_w) || !aligned16(res_vec)) return MOE_EINVAL;
    if (norm_mode != MOE_NORM_NONE && norm_mode != MOE_NORM_RENORM) return MOE_EINVAL;
    if (p < 1 || p > s->N) return MOE_EINVAL;
    if (((uintptr_t)workspace & 255u) != 0) return MOE_EWORKSPACE;
    return moe_route_predict_impl(s, h, gate_w, gate_bias, norm_mode, topk_idx, topk_w, counts, offsets, perm, inv_perm, res_vec,
                                  next_gate_w, next_gate_bias, p, pred_counts, top_experts, workspace, (hipStream_t)stream);
}

size_t moe_res_vec_workspace_bytes(int d) { return d > 0 ? moe_res_vec_ws_bytes(d) : 0; }

int moe_res_vec_accumulate(int n, int d, const void *h_cur, const void *h_next, double *acc_sum, void *workspace,
                           void *stream)
{
    if (n < 0 || d < 8 || d > 8192 || d % 8 != 0) return MOE_EINVAL;
    if (!acc_sum || !workspace || ((uintptr_t)acc_sum & 7u) != 0 || ((uintptr_t)workspace & 7u) != 0) return MOE_EINVAL;
    if (n > 0 && (!h_cur || !h_next || !aligned16(h_cur) || !aligned16(h_next))) return MOE_EINVAL;
    return moe_res_vec_accumulate_impl(n, d, h_cur, h_next, acc_sum, workspace, (hipStream_t)stream);
}

int moe_res_vec_finish(int d, const double *acc_sum, int64_t n_total, float *res_vec, void *stream)
{
    if (d < 8 || d > 8192 || d % 8 != 0 || n_total < 1 || !acc_sum || !res_vec) return MOE_EINVAL;
    return moe_res_vec_finish_impl(d, acc_sum, (long long)n_total, res_vec, (hipStream_t)stream);
}

}   // extern "C"
