// Weight packing for gfx950: row-major [n_mats, rows, K] bf16 -> MFMA-fragment order.
//
// Packed layout: [n_mats][rows/16][K/32][64 lanes][8 bf16].  The 1 KB block (m, rb, kb) holds weight rows
// 16 rb .. 16 rb + 15 and k = 32 kb .. 32 kb + 31; lane l = 16 g + i of it holds row 16 rb + i, k = 32 kb + 8 g .. + 7,
// which is exactly what lane l feeds to the A operand of v_mfma_f32_16x16x32_bf16.  Walking K for one row block
// is a contiguous stream, and every fragment load is eight full 128-byte lines.
#include "moe_common.h"

__global__ __launch_bounds__(256) void pack_weights_kernel(int rows, int K, const uint16_t *__restrict__ src,
                                                           uint16_t *__restrict__ dst, size_t n_chunks)
{
    const size_t c = (size_t)blockIdx.x * 256 + threadIdx.x;     // one 16-byte chunk of the destination per thread
    if (c >= n_chunks) return;
    const int kb_n = K / 32;
    const size_t per_mat = (size_t)rows * K / 8;
    const size_t m = c / per_mat, r = c % per_mat;
    const size_t tile = r / 64;
    const int lane = (int)(r % 64);
    const size_t rb = tile / kb_n;
    const int kb = (int)(tile % kb_n);
    const int i = lane & 15, g = lane >> 4;
    const uint16_t *sp = src + (m * rows + rb * 16 + i) * K + kb * 32 + g * 8;
    *reinterpret_cast<u32x4 *>(dst + c * 8) = *reinterpret_cast<const u32x4 *>(sp);
}

int moe_pack_weights_impl(int n_mats, int rows, int K, const void *src, void *dst, hipStream_t st)
{
    const size_t n_chunks = (size_t)n_mats * rows * K / 8;
    const size_t blocks = (n_chunks + 255) / 256;
    if (blocks > 0x7fffffffull) return MOE_EUNSUPPORTED;
    hipLaunchKernelGGL(pack_weights_kernel, dim3((unsigned)blocks), dim3(256), 0, st, rows, K, (const uint16_t *)src,
                       (uint16_t *)dst, n_chunks);
    MOE_CHECK_LAUNCH();
    return MOE_OK;
}
