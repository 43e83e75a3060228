// Gate / pre-gate: logits z = x.W (+ bias), softmax over the experts, top-k on the logits
// (Sec. II-B: the gate gives every expert a probability per token and the best ones are
// activated; Sec. IV-B: the same function, placed in block N, routes block N+1).
//
// Three kernels share one softmax / top-k routine (16 lanes per token, k rounds of arg-max with
// shuffles, ties to the lowest index, NaN ranks as -infinity and raises a flag):
//   gate_topk_mfma_kernel  bf16, E a multiple of 8: logits on the matrix cores, 16 tokens per
//                          workgroup, W transposed in registers (no LDS staging on the way in);
//   gate_topk_vec_kernel   f32 (and bf16 when the matrix-core kernel does not apply) for
//                          power-of-two E: token rows staged in LDS as float32, threads split W
//                          by expert columns and feature rows and fold their partial sums in a
//                          fixed order (bit-reproducible);
//   gate_topk_kernel       the scalar version of that for any other E.
#include <cstdlib>

#include "gate_small.h"
#include "pgmoe_internal.h"

namespace pgmoe {

constexpr int GATE_TB = 8;
constexpr int GATE_DC = 1024;
constexpr int GATE_THREADS = 256;

__device__ inline float to_float(float v) { return v; }
__device__ inline float to_float(__bf16 v) { return (float)v; }

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

    softmax_topk(zs, PGMOE_MAX_EXPERTS, t0, nt, E, k, idx_out, prob_out, probs_out, flags);
}

// Fast path for E in {8, 16, 32, 64, 128, 256}: thread (rg, cv) owns the 8 experts 8*cv..8*cv+7
// (one 16-byte load of a W row for bf16, two for f32) and every RG-th feature row, so the 256
// threads sweep W in fully contiguous 4 KiB strides.  The RG partial sums per expert are folded
// with a fixed butterfly inside the wavefront and then across the 4 wavefronts in order.
template <typename XT, int TB>
__global__ __launch_bounds__(GATE_THREADS) void gate_topk_vec_kernel(
    const XT *__restrict__ x, const XT *__restrict__ w, const float *__restrict__ bias, int T, int d, int E, int k,
    int32_t *__restrict__ idx_out, float *__restrict__ prob_out, float *__restrict__ probs_out, uint32_t *flags) {
    __shared__ float xs[TB * GATE_DC];
    __shared__ float part[4 * TB * PGMOE_MAX_EXPERTS];
    __shared__ float zs[TB * PGMOE_MAX_EXPERTS];
    typedef XT vec8 __attribute__((ext_vector_type(8)));

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int t0 = blockIdx.x * TB;
    const int nt = min(TB, T - t0);
    const int CV = E >> 3;            // 8-expert column vectors per row (power of two, <= 32)
    const int RG = GATE_THREADS / CV; // row groups
    const int cv = tid & (CV - 1), rg = tid / CV;

    float acc[TB][8];
#pragma unroll
    for (int t = 0; t < TB; ++t)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[t][j] = 0.f;

    for (int c0 = 0; c0 < d; c0 += GATE_DC) {
        const int dc = min(GATE_DC, d - c0);
        __syncthreads();
        for (int i = tid; i < TB * dc; i += GATE_THREADS) {
            const int t = i / dc, c = i - t * dc;
            xs[t * GATE_DC + c] = t < nt ? to_float(x[(size_t)(t0 + t) * d + c0 + c]) : 0.f;
        }
        __syncthreads();
        const vec8 *wv = reinterpret_cast<const vec8 *>(w + (size_t)c0 * E) + cv;
#pragma unroll 4
        for (int i = rg; i < dc; i += RG) {
            const vec8 v = wv[(size_t)i * CV];
            float xr[TB];
#pragma unroll
            for (int t = 0; t < TB; ++t) xr[t] = xs[t * GATE_DC + i];
#pragma unroll
            for (int t = 0; t < TB; ++t)
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[t][j] = fmaf(xr[t], to_float(v[j]), acc[t][j]);
        }
    }
    // fold the row groups that live in this wavefront (lanes with equal cv are CV apart)
    for (int off = 32; off >= CV; off >>= 1) {
#pragma unroll
        for (int t = 0; t < TB; ++t)
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[t][j] += __shfl_xor(acc[t][j], off);
    }
    if (lane < CV) {
#pragma unroll
        for (int t = 0; t < TB; ++t)
#pragma unroll
            for (int j = 0; j < 8; ++j) part[(wave * TB + t) * PGMOE_MAX_EXPERTS + 8 * lane + j] = acc[t][j];
    }
    __syncthreads();
    for (int o = tid; o < TB * E; o += GATE_THREADS) {
        const int t = o / E, e = o - t * E;
        float sum = part[t * PGMOE_MAX_EXPERTS + e];
#pragma unroll
        for (int wv2 = 1; wv2 < 4; ++wv2) sum += part[(wv2 * TB + t) * PGMOE_MAX_EXPERTS + e];
        zs[t * PGMOE_MAX_EXPERTS + e] = sum + (bias ? bias[e] : 0.f);
    }
    __syncthreads();
    softmax_topk(zs, PGMOE_MAX_EXPERTS, t0, nt, E, k, idx_out, prob_out, probs_out, flags);
}

// The smallest gate as a kernel of its own (its body lives in gate_small.h).
__global__ __launch_bounds__(GS_THREADS) void gate_small_kernel(
    int E, const __bf16 *__restrict__ x, const __bf16 *__restrict__ w, const float *__restrict__ bias, int T, int d, int k,
    int32_t *__restrict__ idx_out, float *__restrict__ prob_out, float *__restrict__ probs_out, uint32_t *flags,
    int32_t *__restrict__ row_of, int32_t *__restrict__ offsets, int32_t *__restrict__ src_row) {
    gate_small_dispatch(E, x, w, bias, T, d, k, idx_out, prob_out, probs_out, flags, row_of, offsets, src_row);
}

// Matrix-core path (bf16, E a multiple of 8, d_model a multiple of 32): the gate is a skinny
// GEMM [T,d] x [d,E].  A workgroup takes 16 tokens (one matrix-core tile); its NW wavefronts
// (eight for E <= 128, four above) split the d_model reduction (k-tile kt goes to wavefront
// kt % NW) and their partial logits are added in LDS in wavefront order.  Nothing is staged through LDS on the way in:
//   * the token operand (16 tokens x 32 k) is one 16-byte load per lane straight from x;
//   * W is row-major [d,E], an expert's weights are strided, but lane (n, g) can load rows
//     32*kt + 8*g .. +7 of the eight experts 8*n .. 8*n+7 with eight contiguous 16-byte loads and
//     transpose the 8x8 block in registers.  Product q (q = 0..7) then takes from every lane the
//     eight k-values of expert 8*n + q: that is a valid operand for the 16 experts
//     {q, 8+q, 16+q, ...}, i.e. output column n of product q is expert 8*n + q.  Eight products
//     cover 128 experts per k-tile; E = 256 takes a second pass.
typedef __bf16 gbf16x8 __attribute__((ext_vector_type(8)));
typedef float gfloatx4 __attribute__((ext_vector_type(4)));
constexpr int GM_TOK = 16;  // tokens per workgroup
constexpr int GATE_ROUTE_MAX = 256;  // most (token, choice) pairs the gate kernel groups by itself

template <int NP, int NW>  // NP: passes of 128 experts (1: E <= 128, 2: E <= 256); NW: wavefronts that split d_model
__global__ __launch_bounds__(NW * 64) void gate_topk_mfma_kernel(
    const __bf16 *__restrict__ x, const __bf16 *__restrict__ w, const float *__restrict__ bias, int T, int d, int E, int k,
    int32_t *__restrict__ idx_out, float *__restrict__ prob_out, float *__restrict__ probs_out, uint32_t *flags,
    int32_t *__restrict__ row_of, int32_t *__restrict__ offsets, int32_t *__restrict__ src_row) {  // routing outputs: see below
    extern __shared__ __attribute__((aligned(16))) char gsm[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 15, g = lane >> 4;
    const int t0 = blockIdx.x * GM_TOK;
    const int nt = min(GM_TOK, T - t0);
    const int KT = d >> 5;
    const int ncv = E >> 3;           // 8-expert column vectors per W row
    const int ecols = NP * 128;       // logit columns kept per token in LDS
    constexpr int NT = NW * 64;                              // threads
    float *part = reinterpret_cast<float *>(gsm);            // [NW][GM_TOK][ecols]
    float *zs = part + NW * GM_TOK * ecols;                  // [GM_TOK][ecols]

    gfloatx4 acc[NP][8];
#pragma unroll
    for (int p = 0; p < NP; ++p)
#pragma unroll
        for (int q = 0; q < 8; ++q) acc[p][q] = gfloatx4{0.f, 0.f, 0.f, 0.f};

    const __bf16 *xrow = x + (size_t)(t0 + (n < nt ? n : 0)) * d + 8 * g;  // rows past the batch read its first token; their logits are never used
    // Register prefetch ring, PF k-tiles deep: the operands of k-tile i + PF are requested when
    // k-tile i is consumed, so a wavefront pays the memory latency once, not once per k-tile.
    // Every request is an unconditional load from a clamped (always valid) address, so nothing
    // makes the compiler wait for one load before it issues the next: a stage past the last
    // k-tile reads the last one again and has its token operand zeroed when it is used (it adds
    // nothing), column vectors past E read the last real one (their logits are never used).
    constexpr int PF = NP == 1 ? 3 : 2;
    const gbf16x8 zero8 = gbf16x8{0, 0, 0, 0, 0, 0, 0, 0};
    gbf16x8 a_buf[PF], rows_buf[PF][NP][8];
    auto request = [&](int kt, gbf16x8 &a, gbf16x8 (&rows)[NP][8]) {
        const int ktc = min(kt, KT - 1);
        a = *reinterpret_cast<const gbf16x8 *>(xrow + ktc * 32);
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            const int cv = min(n + 16 * p, ncv - 1);
            const gbf16x8 *src = reinterpret_cast<const gbf16x8 *>(w + (size_t)(ktc * 32 + 8 * g) * E) + cv;
#pragma unroll
            for (int j = 0; j < 8; ++j) rows[p][j] = src[(size_t)j * ncv];
        }
    };
#pragma unroll
    for (int st = 0; st < PF; ++st) request(wave + NW * st, a_buf[st], rows_buf[st]);
    // the instruction scheduler must not move these loads down to their uses to save registers
    // (that would pay the memory latency once per stage): nothing crosses this point
    __builtin_amdgcn_sched_barrier(0);
    for (int kt0 = wave; kt0 < KT; kt0 += NW * PF) {
#pragma unroll
        for (int st = 0; st < PF; ++st) {
            const gbf16x8 a = kt0 + NW * st < KT ? a_buf[st] : zero8;
            gbf16x8 cells[NP][8];
#pragma unroll
            for (int p = 0; p < NP; ++p)
#pragma unroll
                for (int q = 0; q < 8; ++q)
#pragma unroll
                    for (int j = 0; j < 8; ++j) cells[p][q][j] = rows_buf[st][p][j][q];
            request(kt0 + NW * (st + PF), a_buf[st], rows_buf[st]);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int p = 0; p < NP; ++p)
#pragma unroll
                for (int q = 0; q < 8; ++q)
                    acc[p][q] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, cells[p][q], acc[p][q], 0, 0, 0);
        }
    }
    // lane holds tokens 4*g + r (r = 0..3), column n of product q = expert 8*(n + 16*p) + q.  The
    // partial logits are parked as [wave][p][q][lane][r] (one 16-byte LDS write per accumulator
    // tile) and added over the wavefronts in wave order.
#pragma unroll
    for (int p = 0; p < NP; ++p)
#pragma unroll
        for (int q = 0; q < 8; ++q)
            reinterpret_cast<gfloatx4 *>(part)[(((size_t)wave * NP + p) * 8 + q) * 64 + lane] = acc[p][q];
    __syncthreads();
    constexpr int PLANE = NP * 8 * 4 * 64;  // floats per wavefront
    for (int o = tid; o < PLANE; o += NT) {
        const int r = o & 3, l = (o >> 2) & 63, q = (o >> 8) & 7, p = o >> 11;
        const int e = 8 * ((l & 15) + 16 * p) + q, tokl = 4 * (l >> 4) + r;
        float sum = part[o];
#pragma unroll
        for (int wv = 1; wv < NW; ++wv) sum += part[wv * PLANE + o];
        zs[tokl * ecols + e] = sum + ((bias && e < E) ? bias[e] : 0.f);
    }
    __syncthreads();
    // Decode-sized batch (the whole batch in this one workgroup, at most GATE_ROUTE_MAX
    // selections): group the tokens by expert right here instead of in a kernel of its own.
    // Same integers as route_kernel: counts, exclusive prefix sum, stable rank, inverse map.
    const bool route = row_of != nullptr;   // uniform; the host passes it only for a single-workgroup launch
    int32_t *r_idx = reinterpret_cast<int32_t *>(part);      // [n]   (the partial planes are dead by now)
    int32_t *r_cnt = r_idx + GATE_ROUTE_MAX;                 // [E]
    int32_t *r_off = r_cnt + PGMOE_MAX_EXPERTS;              // [E]
    softmax_topk<8 * NP>(zs, ecols, t0, nt, E, k, idx_out, prob_out, probs_out, flags, route ? r_idx : nullptr);
    if (!route) return;
    group_in_workgroup(r_idx, r_cnt, r_off, nt * k, E, k, NT, row_of, offsets, src_row);
}

template <typename XT>
static void launch_gate_t(const pgmoe_config &c, const XT *x, const XT *w, const float *bias, int T, int32_t *idx,
                          float *prob, float *probs, uint32_t *flags, hipStream_t s) {
    const int E = c.n_experts;
    const bool vec = E >= 8 && E <= PGMOE_MAX_EXPERTS && (E & (E - 1)) == 0;
    if (!vec) {
        hipLaunchKernelGGL(gate_topk_kernel<XT>, dim3((T + GATE_TB - 1) / GATE_TB), dim3(GATE_THREADS), 0, s, x, w, bias, T,
                           c.d_model, E, c.top_k, idx, prob, probs, flags);
        return;
    }
    // tokens per workgroup: as few as keeps about 64 workgroups busy (each re-reads W from L2)
#define PG_GATE(TB_)                                                                                                  \
    hipLaunchKernelGGL((gate_topk_vec_kernel<XT, TB_>), dim3((T + TB_ - 1) / TB_), dim3(GATE_THREADS), 0, s, x, w, bias, T, \
                       c.d_model, E, c.top_k, idx, prob, probs, flags)
    if (T <= 64) PG_GATE(1);
    else if (T <= 128) PG_GATE(2);
    else if (T <= 256) PG_GATE(4);
    else PG_GATE(8);
#undef PG_GATE
}

static int launch_gate_mfma(pgmoe_ctx *ctx, const __bf16 *x, const __bf16 *w, const float *bias, int T, int32_t *idx,
                            float *prob, float *probs, hipStream_t s, int32_t *row_of, int32_t *offsets, int32_t *src_row,
                            bool *routed) {
    const pgmoe_config &c = ctx->cfg;
    const int np = c.n_experts <= 128 ? 1 : 2;
    const dim3 grid((T + GM_TOK - 1) / GM_TOK);
    // grouping inside the gate kernel: one workgroup holds the whole batch and the selections fit
    const bool route = row_of && offsets && src_row && grid.x == 1 && T * c.top_k <= GATE_ROUTE_MAX;
    if (!route) row_of = offsets = src_row = nullptr;
    if (routed) *routed = route;
    if (gate_small_applies(c, T)) {
        hipLaunchKernelGGL(gate_small_kernel, dim3(1), dim3(GS_THREADS), 0, s, c.n_experts, x, w, bias, T, c.d_model, c.top_k, idx,
                           prob, probs, ctx->dev_flags, row_of, offsets, src_row);
        PG_HIP(ctx, hipGetLastError());
        return PGMOE_OK;
    }
    // eight wavefronts split d_model: with a three-deep prefetch ring each of them has all its
    // k-tiles (d_model <= 768) in flight at once, i.e. the kernel pays the memory latency once
#define PG_GATE_MFMA(NP_, NW_)                                                                                          \
    do {                                                                                                                \
        auto kern = gate_topk_mfma_kernel<NP_, NW_>;                                                                    \
        const size_t lds = (size_t)(NW_ + 1) * GM_TOK * NP_ * 128 * sizeof(float); /* NW partial planes + the logits */ \
        if (int rc_ = allow_dynamic_lds(ctx, reinterpret_cast<const void *>(kern), lds)) return rc_;                    \
        hipLaunchKernelGGL(kern, grid, dim3(NW_ * 64), lds, s, x, w, bias, T, c.d_model, c.n_experts, c.top_k, idx, prob, probs, \
                           ctx->dev_flags, row_of, offsets, src_row);                                                   \
    } while (0)
    if (np == 1) PG_GATE_MFMA(1, 8);
    else PG_GATE_MFMA(2, 4);
#undef PG_GATE_MFMA
    PG_HIP(ctx, hipGetLastError());
    return PGMOE_OK;
}

int launch_gate(pgmoe_ctx *ctx, const void *x, const void *w, const float *bias, int T, int32_t *idx,
                float *prob, float *probs, hipStream_t s, int32_t *row_of, int32_t *offsets, int32_t *src_row, bool *routed) {
    const pgmoe_config &c = ctx->cfg;
    if (routed) *routed = false;
    if (c.dtype == PGMOE_BF16 && c.n_experts % 8 == 0 && c.d_model % 32 == 0)
        return launch_gate_mfma(ctx, (const __bf16 *)x, (const __bf16 *)w, bias, T, idx, prob, probs, s,
                                row_of, offsets, src_row, routed);
    if (c.dtype == PGMOE_F32)
        launch_gate_t<float>(c, (const float *)x, (const float *)w, bias, T, idx, prob, probs, ctx->dev_flags, s);
    else
        launch_gate_t<__bf16>(c, (const __bf16 *)x, (const __bf16 *)w, bias, T, idx, prob, probs, ctx->dev_flags, s);
    PG_HIP(ctx, hipGetLastError());
    return PGMOE_OK;
}

}  // namespace pgmoe
