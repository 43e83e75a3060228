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

// Combine straight from the FFN's unreduced float32 partials: for every selected row the P
// partials are added exactly as ffn_reduce_kernel<PL> adds them (PL interleaved sub-sums, then
// the sub-sums in ascending order), rounded to bf16 as y_perm would have been, and only then
// weighted and accumulated, so the result is bit-identical to reduce + combine.
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));

template <int PL>
__global__ __launch_bounds__(256) void combine_partials_kernel(const float *__restrict__ partial, int P, int n_rows,
                                                                const int32_t *__restrict__ row_of,
                                                                const float *__restrict__ prob, int d, int k,
                                                                __bf16 *__restrict__ y, const __bf16 *__restrict__ x_res,
                                                                __bf16 *__restrict__ x_next) {
    // 256 threads = PL p-lanes x COLS float4 columns of one token (same split as ffn_reduce_kernel<PL>)
    constexpr int COLS = 256 / PL;
    __shared__ floatx4 sub[PL][COLS + 1];
    const int t = blockIdx.x;
    const int col = threadIdx.x % COLS, pl = threadIdx.x / COLS;
    const int c4 = blockIdx.y * COLS + col;
    const bool live = c4 < d / 4;
    const size_t plane4 = (size_t)n_rows * d / 4;
    floatx4 acc = floatx4{0.f, 0.f, 0.f, 0.f};
    // the residual is needed last: request it first, so that its latency is not paid at the end
    bf16x4 res = bf16x4{0, 0, 0, 0};
    if (x_next && pl == 0 && live) res = *reinterpret_cast<const bf16x4 *>(x_res + (size_t)t * d + 4 * (size_t)c4);
    for (int j = 0; j < k; ++j) {
        floatx4 s = floatx4{0.f, 0.f, 0.f, 0.f};
        const float p_j = prob[(size_t)t * k + j];  // used after the reduction: requested with the row index
        if (live) {
            const floatx4 *src = reinterpret_cast<const floatx4 *>(partial) + (size_t)row_of[(size_t)t * k + j] * (d / 4) + c4;
            // eight partials are requested at a time and then added in ascending order (the order
            // of ffn_reduce_kernel); a plain loop waits for every load before it issues the next
            constexpr int U = 8;
            for (int p0 = pl; p0 < P; p0 += PL * U) {
                floatx4 v[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int p = p0 + u * PL;
                    v[u] = src[(size_t)(p < P ? p : pl) * plane4];  // past the end: a valid address, value unused
                }
#pragma unroll
                for (int u = 0; u < U; ++u)
                    if (p0 + u * PL < P) s += v[u];
            }
        }
        if (PL > 1) {
            __syncthreads();  // previous round's readers are done with sub
            sub[pl][col] = s;
            __syncthreads();
            if (pl == 0) {
                s = sub[0][col];
#pragma unroll
                for (int l = 1; l < PL; ++l) s += sub[l][col];
            }
        }
        if (pl == 0) {
            const float p = p_j;
            acc.x = fmaf(p, (float)(__bf16)s.x, acc.x);
            acc.y = fmaf(p, (float)(__bf16)s.y, acc.y);
            acc.z = fmaf(p, (float)(__bf16)s.z, acc.z);
            acc.w = fmaf(p, (float)(__bf16)s.w, acc.w);
        }
    }
    if (pl != 0 || !live) return;
    const size_t o = (size_t)t * d + 4 * (size_t)c4;
    if (y) {
        bf16x4 v;
        v.x = (__bf16)acc.x; v.y = (__bf16)acc.y; v.z = (__bf16)acc.z; v.w = (__bf16)acc.w;
        *reinterpret_cast<bf16x4 *>(y + o) = v;
    }
    if (x_next) {
        const bf16x4 r = res;
        bf16x4 v;
        v.x = (__bf16)((float)r.x + acc.x); v.y = (__bf16)((float)r.y + acc.y);
        v.z = (__bf16)((float)r.z + acc.z); v.w = (__bf16)((float)r.w + acc.w);
        *reinterpret_cast<bf16x4 *>(x_next + o) = v;
    }
}

int launch_combine_partials(pgmoe_ctx *ctx, const float *partial, int P, int n_rows, const int32_t *row_of,
                            const float *prob, int T, void *y, const void *x_res, void *x_next, hipStream_t s) {
    const pgmoe_config &c = ctx->cfg;
    const int pl = reduce_lanes(P);
    const int cols = 256 / pl;
    const dim3 grid(T, (c.d_model / 4 + cols - 1) / cols);
#define PG_CP(PL_)                                                                                                   \
    hipLaunchKernelGGL(combine_partials_kernel<PL_>, grid, dim3(256), 0, s, partial, P, n_rows, row_of, prob, c.d_model, \
                       c.top_k, (__bf16 *)y, (const __bf16 *)x_res, (__bf16 *)x_next)
    if (pl == 1) PG_CP(1);
    else if (pl == 4) PG_CP(4);
    else PG_CP(16);
#undef PG_CP
    PG_HIP(ctx, hipGetLastError());
    return PGMOE_OK;
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
