// Device-side expert migration (Sec. IV-C: once the pre-gate has picked the next block's
// experts, only those are moved from host memory to the GPU, while the current block runs).
//
// One small grid on the copy stream does the whole job without the host: every workgroup
// scans the routing indices into an LDS presence table, derives the ascending list of
// distinct experts (slot j <- j-th of them, the same rule the FFN uses to find its weights)
// and then pulls its share of the selected blobs straight out of the pinned host store with
// 16-byte loads over the host link.  Host-link reads in flight slow down every concurrent HBM
// access on this chip (a 9.4 MB read kernel goes from 2.9 us to 7/9/12/30 us with 64/96/128/512
// KiB of pull loads outstanding), so the grid keeps just enough in flight to saturate the link:
// 24 workgroups x 4 wavefronts x one 1 KiB load each (96 KiB: 56.3 of 57 GB/s).
#include "pgmoe_internal.h"

namespace pgmoe {

constexpr int FETCH_THREADS = 256;
constexpr int FETCH_GRID = 24;
constexpr int FETCH_UNROLL = 1;

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

template <typename V>
__global__ __launch_bounds__(FETCH_THREADS) void fetch_pull_kernel(
    const int32_t *__restrict__ idx, int n, int E, const char *__restrict__ src_block, size_t expert_stride,
    char *__restrict__ gen_base, size_t expert_bytes, int slots, int all, int32_t *__restrict__ unique_out,
    uint32_t *flags) {
    __shared__ int present[PGMOE_MAX_EXPERTS];
    __shared__ int list[PGMOE_MAX_EXPERTS];
    __shared__ int s_u;
    const int tid = threadIdx.x;
    for (int e = tid; e < PGMOE_MAX_EXPERTS; e += FETCH_THREADS) present[e] = (all && e < E) ? 1 : 0;  // all: slot = expert id
    __syncthreads();
    bool bad = false;
    for (int i = tid; i < n; i += FETCH_THREADS) {
        const int e = idx[i];
        if (e >= 0 && e < E) present[e] = 1;  // all writers store the same value
        else bad = true;
    }
    if (__any(bad) && (tid & 63) == 0 && blockIdx.x == 0) atomicOr(flags, kFlagBadIndex);
    __syncthreads();
    if (tid == 0) {
        int u = 0;
        for (int e = 0; e < E; ++e)
            if (present[e]) list[u++] = e;
        s_u = u;
    }
    __syncthreads();
    int U = s_u;
    if (blockIdx.x == 0 && tid == 0) {
        *unique_out = U;
        if (U > slots) atomicOr(flags, kFlagNoSlot);
    }
    if (U > slots) U = slots;

    // all selected blobs form one range of U * upe vector units, dealt out grid-stride
    const unsigned upe = (unsigned)(expert_bytes / sizeof(V));
    const unsigned total = (unsigned)U * upe;
    const unsigned stride = gridDim.x * FETCH_THREADS;
    unsigned i = blockIdx.x * FETCH_THREADS + tid;
    for (; (unsigned long long)i + (unsigned long long)(FETCH_UNROLL - 1) * stride < total; i += FETCH_UNROLL * stride) {
        V v[FETCH_UNROLL];
        unsigned slot[FETCH_UNROLL], off[FETCH_UNROLL];
#pragma unroll
        for (int u = 0; u < FETCH_UNROLL; ++u) {
            const unsigned g = i + u * stride;
            slot[u] = g / upe;
            off[u] = g - slot[u] * upe;
            v[u] = __builtin_nontemporal_load(reinterpret_cast<const V *>(src_block + (size_t)list[slot[u]] * expert_stride) + off[u]);
        }
#pragma unroll
        for (int u = 0; u < FETCH_UNROLL; ++u)
            reinterpret_cast<V *>(gen_base + (size_t)slot[u] * expert_bytes)[off[u]] = v[u];
    }
    for (; i < total; i += stride) {
        const unsigned sl = i / upe, of = i - sl * upe;
        reinterpret_cast<V *>(gen_base + (size_t)sl * expert_bytes)[of] =
            reinterpret_cast<const V *>(src_block + (size_t)list[sl] * expert_stride)[of];
    }
}

int launch_fetch_pull(pgmoe_ctx *ctx, int block, bool all, const int32_t *idx, int n, hipStream_t s) {
    const int gen = block & 1;
    char *gen_base = ctx->slot_pool + (size_t)gen * ctx->slots * ctx->expert_bytes;
    const char *src = ctx->store_dev + (size_t)block * ctx->block_stride;
    if (ctx->expert_bytes % 16 == 0)
        hipLaunchKernelGGL(fetch_pull_kernel<u32x4>, dim3(FETCH_GRID), dim3(FETCH_THREADS), 0, s, idx, n, ctx->cfg.n_experts,
                           src, ctx->expert_stride, gen_base, ctx->expert_bytes, ctx->slots, all ? 1 : 0, ctx->dev_unique + block,
                           ctx->dev_flags);
    else
        hipLaunchKernelGGL(fetch_pull_kernel<unsigned int>, dim3(FETCH_GRID), dim3(FETCH_THREADS), 0, s, idx, n,
                           ctx->cfg.n_experts, src, ctx->expert_stride, gen_base, ctx->expert_bytes, ctx->slots, all ? 1 : 0,
                           ctx->dev_unique + block, ctx->dev_flags);
    PG_HIP(ctx, hipGetLastError());
    return PGMOE_OK;
}

}  // namespace pgmoe
