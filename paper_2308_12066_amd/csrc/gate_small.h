// Device code shared by the gate kernels (gate.hip) and by the decode-sized expert-FFN kernel
// (ffn.hip), which can carry the next block's pre-gate as one extra workgroup: reductions over a
// group of 16 lanes, softmax / top-k, token grouping inside a workgroup, and the body of the
// smallest gate (at most GS_TOK tokens, 8 or 16 experts).
#ifndef PGMOE_GATE_SMALL_H
#define PGMOE_GATE_SMALL_H
#include "pgmoe_internal.h"

namespace pgmoe {

// Reductions over a group of 16 lanes (one DPP row) by rotating the row by 8, 4, 2 and 1 lanes:
// every lane ends with the reduction over all 16, each step is one VALU operation (no LDS
// crossbar traffic as with a shuffle).  All 64 lanes of the wavefront must be active.
template <int N>
__device__ inline int row_ror(int v) {
    return __builtin_amdgcn_update_dpp(0, v, 0x120 + N, 0xf, 0xf, false);  // row_ror:N
}
template <int N>
__device__ inline float row_ror(float v) {
    return __int_as_float(row_ror<N>(__float_as_int(v)));
}
__device__ inline float group_max(float m) {
    m = fmaxf(m, row_ror<8>(m));
    m = fmaxf(m, row_ror<4>(m));
    m = fmaxf(m, row_ror<2>(m));
    return fmaxf(m, row_ror<1>(m));
}
__device__ inline float group_sum(float s) {  // fixed order: bit-reproducible
    s += row_ror<8>(s);
    s += row_ror<4>(s);
    s += row_ror<2>(s);
    return s + row_ror<1>(s);
}
template <int N>
__device__ inline void argmax_step(float &v, int &i) {
    const float ov = row_ror<N>(v);
    const int oi = row_ror<N>(i);
    if (ov > v || (ov == v && oi < i)) {
        v = ov;
        i = oi;
    }
}
// (value, index) arg-max over the group; equal values keep the lower index.
__device__ inline void group_argmax(float &v, int &i) {
    argmax_step<8>(v, i);
    argmax_step<4>(v, i);
    argmax_step<2>(v, i);
    argmax_step<1>(v, i);
}

// Softmax over the E logits of each token and k rounds of arg-max (ties to the lowest index,
// NaN ranks as -infinity and raises the NaN flag).  zs: LDS [tokens][zstride] logits.
// Sixteen lanes per token, so a wavefront works on four tokens at once; lane s of a group holds
// experts s, s+16, s+32, ...: NQ of them (compile time, E <= 16*NQ), fully unrolled without a
// branch per slice (a skipped slice of a 16-slice version still costs its branch, some 60 clocks,
// which is what a batch-1 gate with 8 experts then spends its time on).
template <int NQ>
__device__ inline void softmax_topk_n(const float *zs, int zstride, int t0, int nt, int E, int k,
                                      int32_t *__restrict__ idx_out, float *__restrict__ prob_out,
                                      float *__restrict__ probs_out, uint32_t *flags, int32_t *idx_lds) {
    const int tid = threadIdx.x;
    const int sub = tid & 15, grp = tid >> 4;  // 16 lanes per group
    bool any_nan = false;
    for (int tb = 0; tb < nt; tb += (int)blockDim.x / 16) {
        if (tb + (grp & ~3) >= nt) continue;  // none of this wavefront's four tokens exists (uniform over the wavefront)
        const int t = tb + grp;
        const bool live = t < nt;  // idle groups of a live wavefront just skip the writes
        float v[NQ];
        float m = -INFINITY;
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
            const int ee = sub + 16 * q;
            float z = (live && ee < E) ? zs[t * zstride + ee] : -INFINITY;
            if (z != z) {
                z = -INFINITY;
                any_nan = true;
            }
            v[q] = z;
            m = fmaxf(m, z);
        }
        m = group_max(m);
        float p[NQ], s = 0.f;
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
            p[q] = (sub + 16 * q < E) ? expf(v[q] - m) : 0.f;
            s += p[q];
        }
        s = group_sum(s);
        const float inv = 1.f / s;
        const size_t tok = (size_t)(t0 + t);
        if (probs_out && live) {
#pragma unroll
            for (int q = 0; q < NQ; ++q)
                if (sub + 16 * q < E) probs_out[tok * E + sub + 16 * q] = p[q] * inv;
        }
        unsigned taken = 0;
        for (int j = 0; j < k; ++j) {
            float bv = -INFINITY;
            int bi = 0x7fffffff;
#pragma unroll
            for (int q = 0; q < NQ; ++q) {
                const int ee = sub + 16 * q;
                // strict > keeps the lowest index of this lane; untaken -inf entries still compete by index
                if (ee < E && !(taken >> q & 1) && (bi == 0x7fffffff || v[q] > bv)) {
                    bv = v[q];
                    bi = ee;
                }
            }
            group_argmax(bv, bi);
            if ((bi & 15) == sub) taken |= 1u << (bi >> 4);  // the lane that holds the winner retires it
            if (sub == 0 && live) {
                idx_out[tok * k + j] = bi;
                prob_out[tok * k + j] = expf(bv - m) * inv;
                if (idx_lds) idx_lds[t * k + j] = bi;
            }
        }
    }
    if (__any(any_nan) && (tid & 63) == 0) atomicOr(flags, kFlagNaN);
}

// MAXQ: the most slices the calling kernel can need (E <= 16*MAXQ there).
template <int MAXQ = 16>
__device__ inline void softmax_topk(const float *zs, int zstride, int t0, int nt, int E, int k,
                                    int32_t *__restrict__ idx_out, float *__restrict__ prob_out,
                                    float *__restrict__ probs_out, uint32_t *flags,
                                    int32_t *idx_lds = nullptr) {  // nullable: LDS copy [nt*k] of the chosen indices
#define PG_SOFTMAX(NQ_) softmax_topk_n<NQ_>(zs, zstride, t0, nt, E, k, idx_out, prob_out, probs_out, flags, idx_lds)
    if (E <= 16) PG_SOFTMAX(1);  // uniform over the kernel
    else if (E <= 32) PG_SOFTMAX(2);
    else if (E <= 64) PG_SOFTMAX(4);
    else if (MAXQ <= 8 || E <= 128) PG_SOFTMAX(8);
    else PG_SOFTMAX(16);
#undef PG_SOFTMAX
}

// Token grouping inside a gate kernel whose single workgroup holds the whole (decode-sized)
// batch: the same integers as route_kernel (counts, exclusive prefix sum, stable rank, inverse
// map), from the LDS copy r_idx[n_sel] of the chosen experts.  r_cnt, r_off: LDS [E] each.
__device__ inline void group_in_workgroup(const int32_t *r_idx, int32_t *r_cnt, int32_t *r_off, int n_sel, int E, int k,
                                          int n_threads, int32_t *__restrict__ row_of, int32_t *__restrict__ offsets,
                                          int32_t *__restrict__ src_row) {
    const int tid = threadIdx.x;
    __syncthreads();
    for (int e = tid; e < E; e += n_threads) {
        int c = 0;
        for (int i = 0; i < n_sel; ++i) c += r_idx[i] == e ? 1 : 0;
        r_cnt[e] = c;
    }
    __syncthreads();
    for (int e = tid; e < E; e += n_threads) {
        int o = 0;
        for (int q = 0; q < e; ++q) o += r_cnt[q];
        r_off[e] = o;
        offsets[e] = o;
    }
    if (tid == 0) offsets[E] = n_sel;
    __syncthreads();
    for (int i = tid; i < n_sel; i += n_threads) {
        const int e = r_idx[i];
        int rank = 0;
        for (int q = 0; q < i; ++q) rank += r_idx[q] == e ? 1 : 0;
        const int r = r_off[e] + rank;
        row_of[i] = r;
        src_row[r] = i / k;
    }
}

// Smallest gates (bf16, at most GS_TOK tokens, 8 or 16 experts: batch-1 decode of the 8-expert
// models): latency is everything, the arithmetic is a few thousand multiply-adds.  One workgroup;
// thread i owns rows 8i .. 8i+7 of W (whole rows: E contiguous values) and the matching eight
// features of every token, all requested at once; partial logits are summed over the 16 lanes
// of a row by rotation, then over the rows of all wavefronts in LDS in ascending order.
constexpr int GS_TOK = 4;
constexpr int GS_THREADS = 256;
typedef __bf16 gs_bf16x8 __attribute__((ext_vector_type(8)));

template <int EV, int NTOK>  // EV = E / 8 (1 or 2); NTOK = tokens the arithmetic is unrolled for (T <= NTOK <= GS_TOK)
__device__ inline void gate_small_body(
    const __bf16 *__restrict__ x, const __bf16 *__restrict__ w, const float *__restrict__ bias, int T, int d, int k,
    int32_t *__restrict__ idx_out, float *__restrict__ prob_out, float *__restrict__ probs_out, uint32_t *flags,
    int32_t *__restrict__ row_of, int32_t *__restrict__ offsets, int32_t *__restrict__ src_row) {
    constexpr int E = 8 * EV;
    constexpr int ROWS = GS_THREADS / 16;                // 16-lane rows in the workgroup
    __shared__ float part[ROWS][NTOK * E];
    __shared__ float zs[GS_TOK * 16];
    __shared__ int32_t r_idx[GS_TOK * E], r_cnt[E], r_off[E];
    const int tid = threadIdx.x;
    const bool mine = 8 * tid < d;                       // d <= 8 * GS_THREADS (checked by the host)
    const int r0 = mine ? 8 * tid : 0;                   // idle threads read rows 0..7 and add nothing
    const float b = (bias && tid < NTOK * E) ? bias[tid % E] : 0.f;  // needed last, requested first
    gs_bf16x8 xv[NTOK], wv[8][EV];
#pragma unroll
    for (int t = 0; t < NTOK; ++t) xv[t] = *reinterpret_cast<const gs_bf16x8 *>(x + (size_t)(t < T ? t : 0) * d + r0);
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int v = 0; v < EV; ++v) wv[j][v] = *reinterpret_cast<const gs_bf16x8 *>(w + (size_t)(r0 + j) * E + 8 * v);
    float acc[NTOK][E];
#pragma unroll
    for (int t = 0; t < NTOK; ++t)
#pragma unroll
        for (int e = 0; e < E; ++e) {
            float a = 0.f;
#pragma unroll
            for (int j = 0; j < 8; ++j) a = fmaf((float)xv[t][j], (float)wv[j][e >> 3][e & 7], a);
            a = mine ? a : 0.f;
            acc[t][e] = group_sum(a);
        }
    if ((tid & 15) == 0) {
#pragma unroll
        for (int t = 0; t < NTOK; ++t)
#pragma unroll
            for (int e = 0; e < E; ++e) part[tid >> 4][t * E + e] = acc[t][e];
    }
    __syncthreads();
    if (tid < NTOK * E) {
        const int e = tid % E;
        float sum = part[0][tid];
#pragma unroll
        for (int r = 1; r < ROWS; ++r) sum += part[r][tid];
        zs[(tid / E) * 16 + e] = sum + b;
    }
    __syncthreads();
    const bool route = row_of != nullptr;
    softmax_topk_n<1>(zs, 16, 0, T, E, k, idx_out, prob_out, probs_out, flags, route ? r_idx : nullptr);
    if (!route) return;
    group_in_workgroup(r_idx, r_cnt, r_off, T * k, E, k, GS_THREADS, row_of, offsets, src_row);
}

// Runs the smallest gate for (E, T) in the calling workgroup of GS_THREADS threads (uniform call).
__device__ inline void gate_small_dispatch(int E, const __bf16 *x, const __bf16 *w, const float *bias, int T, int d, int k,
                                           int32_t *idx_out, float *prob_out, float *probs_out, uint32_t *flags,
                                           int32_t *row_of, int32_t *offsets, int32_t *src_row) {
#define PG_GS(EV_, NTOK_) gate_small_body<EV_, NTOK_>(x, w, bias, T, d, k, idx_out, prob_out, probs_out, flags, row_of, offsets, src_row)
    if (E == 8) {
        if (T == 1) PG_GS(1, 1);
        else if (T == 2) PG_GS(1, 2);
        else PG_GS(1, 4);
    } else {
        if (T == 1) PG_GS(2, 1);
        else if (T == 2) PG_GS(2, 2);
        else PG_GS(2, 4);
    }
#undef PG_GS
}

// Host side: is (T tokens, this configuration) a gate the smallest-gate code serves?
inline bool gate_small_applies(const pgmoe_config &c, int T) {
    return c.dtype == PGMOE_BF16 && T >= 1 && T <= GS_TOK && (c.n_experts == 8 || c.n_experts == 16) && c.d_model <= 8 * GS_THREADS;
}

}  // namespace pgmoe
#endif  // PGMOE_GATE_SMALL_H
