// Gate / pre-gate: logits z = x.W (+ bias), softmax over the experts, top-k on the logits
// (Sec. II-B: the gate gives every expert a probability per token and the best ones are
// activated; Sec. IV-B: the same function, placed in block N, routes block N+1).
//
// One workgroup handles GATE_TB tokens.  The token rows are staged in LDS as float32 in
// chunks of GATE_DC features; thread (g, e) owns expert column e and every G-th feature
// row, so a wavefront reads W in contiguous runs.  The G partial sums per (token, expert)
// are added in fixed order (bit-reproducible), then one wavefront per token does the
// softmax and k rounds of arg-max with DPP-free shuffles.
#include "pgmoe_internal.h"

namespace pgmoe {

constexpr int GATE_TB = 8;
constexpr int GATE_DC = 1024;
constexpr int GATE_THREADS = 256;

__device__ inline float to_float(float v) { return v; }
__device__ inline float to_float(__bf16 v) { return (float)v; }

// (value, index) arg-max over the wavefront; equal values keep the lower index.
__device__ inline void wave_argmax(float &v, int &i) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const float ov = __shfl_xor(v, off);
        const int oi = __shfl_xor(i, off);
        if (ov > v || (ov == v && oi < i)) {
            v = ov;
            i = oi;
        }
    }
}

template <typename XT>
__global__ __launch_bounds__(GATE_THREADS) void gate_topk_kernel(
    const XT *__restrict__ x, const XT *__restrict__ w, const float *__restrict__ bias, int T, int d, int E, int k,
    int32_t *__restrict__ idx_out, float *__restrict__ prob_out, float *__restrict__ probs_out, uint32_t *flags) {
    __shared__ float xs[GATE_TB * GATE_DC];
    __shared__ float part[GATE_THREADS * GATE_TB];  // [G][TB][E], G*E <= 256
    __shared__ float zs[GATE_TB * PGMOE_MAX_EXPERTS];

    const int tid = threadIdx.x;
    const int t0 = blockIdx.x * GATE_TB;
    const int nt = min(GATE_TB, T - t0);
    const int G = GATE_THREADS / E;
    const int g = tid / E, e = tid - g * E;
    const bool active = g < G;

    float acc[GATE_TB];
#pragma unroll
    for (int t = 0; t < GATE_TB; ++t) acc[t] = 0.f;

    for (int c0 = 0; c0 < d; c0 += GATE_DC) {
        const int dc = min(GATE_DC, d - c0);
        __syncthreads();
        for (int i = tid; i < GATE_TB * dc; i += GATE_THREADS) {
            const int t = i / dc, c = i - t * dc;
            xs[t * GATE_DC + c] = t < nt ? to_float(x[(size_t)(t0 + t) * d + c0 + c]) : 0.f;
        }
        __syncthreads();
        if (active) {
            for (int i = g; i < dc; i += G) {
                const float wv = to_float(w[(size_t)(c0 + i) * E + e]);
#pragma unroll
                for (int t = 0; t < GATE_TB; ++t) acc[t] = fmaf(xs[t * GATE_DC + i], wv, acc[t]);
            }
        }
    }
    if (active) {
#pragma unroll
        for (int t = 0; t < GATE_TB; ++t) part[(g * GATE_TB + t) * E + e] = acc[t];
    }
    __syncthreads();
    for (int o = tid; o < GATE_TB * E; o += GATE_THREADS) {
        const int t = o / E, ee = o - t * E;
        float s = 0.f;
        for (int gg = 0; gg < G; ++gg) s += part[(gg * GATE_TB + t) * E + ee];
        zs[t * PGMOE_MAX_EXPERTS + ee] = s + (bias ? bias[ee] : 0.f);
    }
    __syncthreads();

    // softmax + top-k: one wavefront per token; lane holds experts lane, lane+64, lane+128, lane+192
    const int lane = tid & 63, wave = tid >> 6;
    for (int t = wave; t < nt; t += GATE_THREADS / 64) {
        float v[4];
        bool saw_nan = false;
        float m = -INFINITY;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int ee = lane + 64 * q;
            float z = ee < E ? zs[t * PGMOE_MAX_EXPERTS + ee] : -INFINITY;
            if (z != z) {
                z = -INFINITY;
                saw_nan = true;
            }
            v[q] = z;
            m = fmaxf(m, z);
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
        float p[4], s = 0.f;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            p[q] = (lane + 64 * q < E) ? expf(v[q] - m) : 0.f;
            s += p[q];
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) s += __shfl_xor(s, off);
        const float inv = 1.f / s;
        const size_t tok = (size_t)(t0 + t);
        if (probs_out) {
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (lane + 64 * q < E) probs_out[tok * E + lane + 64 * q] = p[q] * inv;
        }
        if (__any(saw_nan) && lane == 0) atomicOr(flags, kFlagNaN);

        unsigned taken = 0;
        for (int j = 0; j < k; ++j) {
            float bv = -INFINITY;
            int bi = 0x7fffffff;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int ee = lane + 64 * q;
                // strict > keeps the lowest index of this lane; untaken -inf entries still compete by index
                if (ee < E && !(taken >> q & 1) && (bi == 0x7fffffff || v[q] > bv)) {
                    bv = v[q];
                    bi = ee;
                }
            }
            wave_argmax(bv, bi);
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (lane + 64 * q == bi) taken |= 1u << q;
            if (lane == 0) {
                idx_out[tok * k + j] = bi;
                prob_out[tok * k + j] = expf(bv - m) * inv;
            }
        }
    }
}

int launch_gate(pgmoe_ctx *ctx, const void *x, const void *w, const float *bias, int T, int32_t *idx,
                float *prob, float *probs, hipStream_t s) {
    const pgmoe_config &c = ctx->cfg;
    const int grid = (T + GATE_TB - 1) / GATE_TB;
    if (c.dtype == PGMOE_F32)
        hipLaunchKernelGGL(gate_topk_kernel<float>, dim3(grid), dim3(GATE_THREADS), 0, s, (const float *)x,
                           (const float *)w, bias, T, c.d_model, c.n_experts, c.top_k, idx, prob, probs, ctx->dev_flags);
    else
        hipLaunchKernelGGL(gate_topk_kernel<__bf16>, dim3(grid), dim3(GATE_THREADS), 0, s, (const __bf16 *)x,
                           (const __bf16 *)w, bias, T, c.d_model, c.n_experts, c.top_k, idx, prob, probs, ctx->dev_flags);
    PG_HIP(ctx, hipGetLastError());
    return PGMOE_OK;
}

}  // namespace pgmoe
