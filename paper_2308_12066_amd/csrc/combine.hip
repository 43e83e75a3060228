// Weighted combine (Sec. II-B: the gate's probabilities weigh the outputs of the activated
// experts): y[t] = sum_j prob[t,j] * y_perm[row_of[t*k+j]], gathered per token so that no
// atomics are needed and the sum order (j ascending) is fixed.  Optionally also writes the
// residual stand-in x_next = x_res + y that feeds the next MoE block.
#include "pgmoe_internal.h"

namespace pgmoe {

template <typename XT>
struct Vec4;
template <>
struct Vec4<float> {
    typedef float4 type;
};
template <>
struct Vec4<__bf16> {
    typedef __bf16 type __attribute__((ext_vector_type(4)));
};

template <typename XT, int VEC>
__global__ __launch_bounds__(256) void combine_kernel(const XT *__restrict__ y_perm, const int32_t *__restrict__ row_of,
                                                       const float *__restrict__ prob, int d, int k, XT *__restrict__ y,
                                                       const XT *__restrict__ x_res, XT *__restrict__ x_next) {
    const int t = blockIdx.x;
    for (int c = (blockIdx.y * 256 + threadIdx.x) * VEC; c < d; c += gridDim.y * 256 * VEC) {
        float acc[VEC];
#pragma unroll
        for (int v = 0; v < VEC; ++v) acc[v] = 0.f;
        for (int j = 0; j < k; ++j) {
            const float p = prob[(size_t)t * k + j];
            const XT *src = y_perm + (size_t)row_of[(size_t)t * k + j] * d + c;
            if (VEC == 4) {
                const typename Vec4<XT>::type v4 = *reinterpret_cast<const typename Vec4<XT>::type *>(src);
                acc[0] = fmaf(p, (float)v4.x, acc[0]);
                acc[1] = fmaf(p, (float)v4.y, acc[1]);
                acc[2] = fmaf(p, (float)v4.z, acc[2]);
                acc[3] = fmaf(p, (float)v4.w, acc[3]);
            } else {
                acc[0] = fmaf(p, (float)src[0], acc[0]);
            }
        }
        const size_t o = (size_t)t * d + c;
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
            if (y) y[o + v] = (XT)acc[v];
            if (x_next) x_next[o + v] = (XT)((float)x_res[o + v] + acc[v]);
        }
    }
}

template <typename XT>
static void launch_t(const pgmoe_config &c, const void *y_perm, const int32_t *row_of, const float *prob, int T, void *y,
                     const void *x_res, void *x_next, hipStream_t s) {
    const int d = c.d_model;
    if (d % 4 == 0) {
        const int gy = (d / 4 + 255) / 256;
        hipLaunchKernelGGL((combine_kernel<XT, 4>), dim3(T, gy), dim3(256), 0, s, (const XT *)y_perm, row_of, prob, d,
                           c.top_k, (XT *)y, (const XT *)x_res, (XT *)x_next);
    } else {
        const int gy = (d + 255) / 256;
        hipLaunchKernelGGL((combine_kernel<XT, 1>), dim3(T, gy), dim3(256), 0, s, (const XT *)y_perm, row_of, prob, d,
                           c.top_k, (XT *)y, (const XT *)x_res, (XT *)x_next);
    }
}

int launch_combine(pgmoe_ctx *ctx, const void *y_perm, const int32_t *row_of, const float *prob, int T, void *y,
                   const void *x_res, void *x_next, hipStream_t s) {
    if (ctx->cfg.dtype == PGMOE_F32)
        launch_t<float>(ctx->cfg, y_perm, row_of, prob, T, y, x_res, x_next, s);
    else
        launch_t<__bf16>(ctx->cfg, y_perm, row_of, prob, T, y, x_res, x_next, s);
    PG_HIP(ctx, hipGetLastError());
    return PGMOE_OK;
}

}  // namespace pgmoe
