// Group tokens by expert (Sec. II-B: each activated expert processes the tokens routed to it):
// histogram of the selected expert ids, exclusive prefix sum, stable rank of every entry
// inside its expert's group, and the row gather x_perm[row_of[n]] = x[n / k].  The whole-stack
// step skips the gather: route_kernel also writes the inverse map (grouped row -> token) and the
// expert kernels read their rows through it.
//
// route_kernel: one workgroup of 1024 threads; each of its 16 wavefronts owns one contiguous
// range of the entries.  Pass 1 counts every range into a histogram of its own (LDS atomics:
// integer, so order does not matter).  One thread per expert then turns the 16 histograms into
// the start of every (wavefront, expert) run, and one wavefront scans the expert totals.  Pass 2
// needs no further workgroup barrier: a wavefront walks its range in order, 64 entries at a time;
// equal keys find each other with one ballot per key bit, which gives the stable rank inside the
// 64, and the run's start moves on by the number of matches.  Everything is integer work and
// bit-reproducible.
// gather_rows_kernel: one wavefront per entry, 16-byte copies.
#include "pgmoe_internal.h"

namespace pgmoe {

constexpr int ROUTE_THREADS = 1024;
constexpr int ROUTE_WAVES = ROUTE_THREADS / 64;

__global__ __launch_bounds__(ROUTE_THREADS) void route_kernel(const int32_t *__restrict__ idx, int n, int E, int k,
                                                               int32_t *__restrict__ row_of,
                                                               int32_t *__restrict__ offsets,
                                                               int32_t *__restrict__ src_row, uint32_t *flags) {
    __shared__ int run_start[ROUTE_WAVES][PGMOE_MAX_EXPERTS];  // pass 1: counts; then: next free row of the (wavefront, expert) run
    __shared__ int total[PGMOE_MAX_EXPERTS];                    // entries per expert, then the expert's first row
    static_assert(PGMOE_MAX_EXPERTS == 256, "four experts per lane in the scan below");

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int per = ((n + ROUTE_WAVES - 1) / ROUTE_WAVES + 63) & ~63;  // entries per wavefront, whole rounds of 64
    const int lo = min(n, wave * per), hi = min(n, lo + per);
    for (int i = tid; i < ROUTE_WAVES * PGMOE_MAX_EXPERTS; i += ROUTE_THREADS) (&run_start[0][0])[i] = 0;
    __syncthreads();

    // the first ROUTE_KEEP rounds of a wavefront's range stay in registers for pass 2 (all of them up to
    // 8192 entries), and their loads are in flight together
    constexpr int ROUTE_KEEP = 8;
    int kept[ROUTE_KEEP];
#pragma unroll
    for (int c = 0; c < ROUTE_KEEP; ++c) {
        const int i = lo + c * 64 + lane;
        kept[c] = i < hi ? idx[i] : 0;
    }
    bool bad = false;
#pragma unroll
    for (int c = 0; c < ROUTE_KEEP; ++c) {
        const int i = lo + c * 64 + lane;
        if (kept[c] < 0 || kept[c] >= E) {
            bad = true;
            kept[c] = kept[c] < 0 ? 0 : E - 1;
        }
        if (i < hi) atomicAdd(&run_start[wave][kept[c]], 1);
    }
    for (int i = lo + ROUTE_KEEP * 64 + lane; i < hi; i += 64) {
        int e = idx[i];
        if (e < 0 || e >= E) {
            bad = true;
            e = e < 0 ? 0 : E - 1;
        }
        atomicAdd(&run_start[wave][e], 1);
    }
    if (__any(bad) && lane == 0) atomicOr(flags, kFlagBadIndex);
    __syncthreads();

    // per expert: counts of the wavefronts -> offsets of their runs inside the expert's group
    if (tid < PGMOE_MAX_EXPERTS) {
        int run = 0;
        if (tid < E)
            for (int w = 0; w < ROUTE_WAVES; ++w) {
                const int c = run_start[w][tid];
                run_start[w][tid] = run;
                run += c;
            }
        total[tid] = run;
    }
    __syncthreads();
    // exclusive scan of the expert totals by the first wavefront, four experts per lane
    if (wave == 0) {
        const int t0 = total[4 * lane], t1 = total[4 * lane + 1], t2 = total[4 * lane + 2], t3 = total[4 * lane + 3];
        int incl = t0 + t1 + t2 + t3;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int o = __shfl_up(incl, off);
            if (lane >= off) incl += o;
        }
        const int first[4] = {incl - (t0 + t1 + t2 + t3), incl - (t1 + t2 + t3), incl - (t2 + t3), incl - t3};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int e = 4 * lane + j;
            total[e] = first[j];
            if (e < E) offsets[e] = first[j];
        }
        if (lane == 0) offsets[E] = n;
    }
    __syncthreads();

    int nbits = 0;
    while ((1 << nbits) < E) ++nbits;
    volatile int *my_run = run_start[wave];  // shared by the lanes of this wavefront only, which run in lockstep
    auto place = [&](int i, bool valid, int e) {
        unsigned long long peers = __ballot(valid);
        for (int b = 0; b < nbits; ++b) {
            const bool bit = (e >> b) & 1;
            const unsigned long long m = __ballot(bit);
            peers &= bit ? m : ~m;
        }
        const unsigned long long below = (1ull << lane) - 1ull;
        const int rank_in_round = __popcll(peers & below);
        const int start = my_run[e];       // every lane reads before the leaders write
        __builtin_amdgcn_wave_barrier();
        if (valid && rank_in_round == 0) my_run[e] = start + __popcll(peers);
        __builtin_amdgcn_wave_barrier();
        if (valid) {
            const int r = total[e] + start + rank_in_round;
            row_of[i] = r;
            if (src_row) src_row[r] = i / k;  // the inverse map: which token's row sits in grouped row r
        }
    };
#pragma unroll
    for (int c = 0; c < ROUTE_KEEP; ++c) {
        const int i = lo + c * 64 + lane;
        if (lo + c * 64 < hi) place(i, i < hi, kept[c]);  // uniform over the wavefront
    }
    for (int c0 = lo + ROUTE_KEEP * 64; c0 < hi; c0 += 64) {
        const int i = c0 + lane;
        const bool valid = i < hi;
        int e = 0;
        if (valid) {
            e = idx[i];
            e = e < 0 ? 0 : (e >= E ? E - 1 : e);
        }
        place(i, valid, e);
    }
}

// x_perm[row_of[n]] = x[n / k]; `vec` bytes per lane access (16 or 4), row_bytes % vec == 0.
template <typename V>
__global__ __launch_bounds__(256) void gather_rows_kernel(const char *__restrict__ x, const int32_t *__restrict__ row_of,
                                                           int n, int k, int row_bytes, char *__restrict__ x_perm) {
    const int entry = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (entry >= n) return;
    const int lane = threadIdx.x & 63;
    const V *src = reinterpret_cast<const V *>(x + (size_t)(entry / k) * row_bytes);
    V *dst = reinterpret_cast<V *>(x_perm + (size_t)row_of[entry] * row_bytes);
    const int nv = row_bytes / (int)sizeof(V);
    for (int i = lane; i < nv; i += 64) dst[i] = src[i];
}

int launch_route(pgmoe_ctx *ctx, const int32_t *idx, int T, int32_t *row_of, int32_t *offsets, int32_t *src_row,
                 hipStream_t s) {
    const pgmoe_config &c = ctx->cfg;
    hipLaunchKernelGGL(route_kernel, dim3(1), dim3(ROUTE_THREADS), 0, s, idx, T * c.top_k, c.n_experts, c.top_k, row_of,
                       offsets, src_row, ctx->dev_flags);
    PG_HIP(ctx, hipGetLastError());
    return PGMOE_OK;
}

int launch_permute(pgmoe_ctx *ctx, const void *x, const int32_t *idx, int T, void *x_perm, int32_t *row_of,
                   int32_t *offsets, hipStream_t s) {
    const pgmoe_config &c = ctx->cfg;
    const int n = T * c.top_k;
    const int rc = launch_route(ctx, idx, T, row_of, offsets, nullptr, s);
    if (rc) return rc;
    if (n == 0) return PGMOE_OK;
    const int row_bytes = c.d_model * (int)ctx->elem;
    const int grid = (n + 3) / 4;
    if (row_bytes % 16 == 0)
        hipLaunchKernelGGL(gather_rows_kernel<uint4>, dim3(grid), dim3(256), 0, s, (const char *)x, row_of, n, c.top_k,
                           row_bytes, (char *)x_perm);
    else
        hipLaunchKernelGGL(gather_rows_kernel<uint32_t>, dim3(grid), dim3(256), 0, s, (const char *)x, row_of, n,
                           c.top_k, row_bytes, (char *)x_perm);
    PG_HIP(ctx, hipGetLastError());
    return PGMOE_OK;
}

}  // namespace pgmoe
