// Group tokens by expert (Sec. II-B: each activated expert processes the tokens routed to it):
// histogram of the selected expert ids, exclusive prefix sum, stable rank of every entry
// inside its expert's group, and the row gather x_perm[row_of[n]] = x[n / k].  The whole-stack
// step skips the gather: route_kernel also writes the inverse map (grouped row -> token) and the
// expert kernels read their rows through it.
//
// route_kernel: one workgroup of 1024 threads (16 wavefronts).  Pass 1 counts with LDS
// atomics (integer, so order does not matter).  Pass 2 walks the entries in order, 1024 at
// a time; inside a wavefront equal keys find each other with one ballot per key bit, and a
// per-wavefront count table turns that into a stable rank.  Everything is integer work and
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
    __shared__ int cnt[PGMOE_MAX_EXPERTS];
    __shared__ int scan[PGMOE_MAX_EXPERTS];
    __shared__ int base[PGMOE_MAX_EXPERTS];
    __shared__ int whist[ROUTE_WAVES][PGMOE_MAX_EXPERTS];
    __shared__ int wbase[ROUTE_WAVES][PGMOE_MAX_EXPERTS];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int i = tid; i < PGMOE_MAX_EXPERTS; i += ROUTE_THREADS) cnt[i] = 0;
    for (int i = tid; i < ROUTE_WAVES * PGMOE_MAX_EXPERTS; i += ROUTE_THREADS) (&whist[0][0])[i] = 0;
    __syncthreads();

    bool bad = false;
    for (int i = tid; i < n; i += ROUTE_THREADS) {
        int e = idx[i];
        if (e < 0 || e >= E) {
            bad = true;
            e = e < 0 ? 0 : E - 1;
        }
        atomicAdd(&cnt[e], 1);
    }
    if (__any(bad) && lane == 0) atomicOr(flags, kFlagBadIndex);
    __syncthreads();

    // exclusive scan of cnt[0..E) (E <= 256): Hillis-Steele on the first 256 threads
    if (tid < PGMOE_MAX_EXPERTS) scan[tid] = tid < E ? cnt[tid] : 0;
    __syncthreads();
    for (int off = 1; off < PGMOE_MAX_EXPERTS; off <<= 1) {
        int v = 0;
        if (tid < PGMOE_MAX_EXPERTS && tid >= off) v = scan[tid - off];
        __syncthreads();
        if (tid < PGMOE_MAX_EXPERTS) scan[tid] += v;
        __syncthreads();
    }
    if (tid < E) {
        const int excl = scan[tid] - cnt[tid];
        base[tid] = excl;
        offsets[tid] = excl;
    }
    if (tid == 0) offsets[E] = n;
    __syncthreads();

    int nbits = 0;
    while ((1 << nbits) < E) ++nbits;

    for (int c0 = 0; c0 < n; c0 += ROUTE_THREADS) {
        const int i = c0 + tid;
        const bool valid = i < n;
        int e = 0;
        if (valid) {
            e = idx[i];
            e = e < 0 ? 0 : (e >= E ? E - 1 : e);
        }
        unsigned long long peers = __ballot(valid);
        for (int b = 0; b < nbits; ++b) {
            const bool bit = (e >> b) & 1;
            const unsigned long long m = __ballot(bit);
            peers &= bit ? m : ~m;
        }
        const unsigned long long below = (1ull << lane) - 1ull;
        const int rank_in_wave = __popcll(peers & below);
        const bool leader = valid && rank_in_wave == 0;
        if (leader) whist[wave][e] = __popcll(peers);
        __syncthreads();
        if (tid < E) {
            int run = base[tid];
            for (int w = 0; w < ROUTE_WAVES; ++w) {
                wbase[w][tid] = run;
                run += whist[w][tid];
            }
            base[tid] = run;
        }
        __syncthreads();
        if (valid) {
            const int r = wbase[wave][e] + rank_in_wave;
            row_of[i] = r;
            if (src_row) src_row[r] = i / k;  // the inverse map: which token's row sits in grouped row r
        }
        if (leader) whist[wave][e] = 0;
        __syncthreads();
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
