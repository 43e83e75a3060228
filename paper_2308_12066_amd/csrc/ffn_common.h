// Shared by the expert-FFN translation units (ffn.hip: fused, decode and float32 kernels, launch
// planning; ffn_gemm.hip: the two tiled GEMMs for launches with hundreds of rows per expert).
#ifndef PGMOE_FFN_COMMON_H
#define PGMOE_FFN_COMMON_H
#include <algorithm>
#include <cstdlib>

#include "pgmoe_internal.h"

namespace pgmoe {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(1))) bf16x8 global_bf16x8;  // a load through this is a global_load, never flat

// ------------------------------------------------------------------------------------------
// Which (expert, row range, slot) does chunk number `chunk` cover?  Chunks are numbered expert
// by expert, ceil(n_e / rows_per_chunk) per expert.  Every wavefront computes this on its own
// from the E+1 offsets (E <= 256: four experts per lane), so no LDS or barrier is needed.
struct ChunkInfo {
    int expert, slot, row0, nrows;  // nrows == 0: chunk does not exist
};

// Inclusive prefix sum over the 64 lanes of a wavefront (all of them active) with data-parallel
// primitives: four shifts inside each row of 16 lanes, then lane 15 of row 0 / 2 into row 1 / 3
// and lane 31 into rows 2 and 3.  Six VALU operations instead of six trips through the LDS crossbar.
template <int CTRL, int ROW_MASK>
__device__ inline int dpp_or_zero(int v) {
    return __builtin_amdgcn_update_dpp(0, v, CTRL, ROW_MASK, 0xf, false);  // lanes without a source get 0
}
__device__ inline int wave_incl_scan(int v) {
    v += dpp_or_zero<0x111, 0xf>(v);  // row_shr:1
    v += dpp_or_zero<0x112, 0xf>(v);  // row_shr:2
    v += dpp_or_zero<0x114, 0xf>(v);  // row_shr:4
    v += dpp_or_zero<0x118, 0xf>(v);  // row_shr:8
    v += dpp_or_zero<0x142, 0xa>(v);  // row_bcast:15 -> rows 1 and 3
    v += dpp_or_zero<0x143, 0xc>(v);  // row_bcast:31 -> rows 2 and 3
    return v;
}

__device__ inline ChunkInfo find_chunk(const int32_t *__restrict__ offsets, int E, int rows_per_chunk, int chunk) {
    const int lane = threadIdx.x & 63;
    ChunkInfo ci = {0, 0, 0, 0};
    int chunk_base = 0, slot_base = 0;
    for (int q = 0; q * 64 < E; ++q) {
        const int e = q * 64 + lane;
        int lo = 0, n = 0;
        if (e < E) {
            lo = offsets[e];
            n = offsets[e + 1] - lo;
        }
        const int c = (n + rows_per_chunk - 1) / rows_per_chunk;
        const int nz = n > 0 ? 1 : 0;
        const int c_incl = wave_incl_scan(c), nz_incl = wave_incl_scan(nz);
        const int c_excl = chunk_base + c_incl - c;
        const bool mine = chunk >= c_excl && chunk < c_excl + c;
        const unsigned long long hit = __ballot(mine);
        if (hit) {
            const int src = __ffsll((long long)hit) - 1;  // uniform: read that lane's values directly
            const int first = (chunk - __builtin_amdgcn_readlane(c_excl, src)) * rows_per_chunk;
            ci.expert = q * 64 + src;
            ci.slot = slot_base + __builtin_amdgcn_readlane(nz_incl, src) - 1;
            ci.row0 = __builtin_amdgcn_readlane(lo, src) + first;
            ci.nrows = min(rows_per_chunk, __builtin_amdgcn_readlane(n, src) - first);
            return ci;
        }
        chunk_base += __builtin_amdgcn_readlane(c_incl, 63);
        slot_base += __builtin_amdgcn_readlane(nz_incl, 63);
    }
    return ci;
}

// Number of chunks of rows_per_chunk rows over all experts (the same count on every lane).
__device__ inline int count_chunks(const int32_t *__restrict__ offsets, int E, int rows_per_chunk) {
    const int lane = threadIdx.x & 63;
    int total = 0;
    for (int q = 0; q * 64 < E; ++q) {
        const int e = q * 64 + lane;
        const int n = e < E ? offsets[e + 1] - offsets[e] : 0;
        total += __builtin_amdgcn_readlane(wave_incl_scan((n + rows_per_chunk - 1) / rows_per_chunk), 63);
    }
    return total;
}

// ------------------------------------------------------------------------------------------
// Workgroup barrier that orders LDS traffic only: global loads already in flight (the weight
// prefetch ring) stay in flight across it.
__device__ inline void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// ---- host side, defined in ffn.hip
// Next free event pair when FFN timing is on, else -1.
int ffn_timing_slot(pgmoe_ctx *ctx);
// y_perm = bf16(sum of the P float32 partials [P][n_rows, d]), added in a fixed order.
int launch_ffn_reduce(pgmoe_ctx *ctx, const float *partial, int P, int n_rows, void *y_perm, hipStream_t s);

// ---- host side, defined in ffn_gemm.hip
// Does a launch of n_rows rows take the two-GEMM path?
bool uses_gemm_kernels(const pgmoe_config &c, int n_rows);
// Workspace the two-GEMM path needs for max_tokens * top_k rows.
size_t ffn_gemm_workspace_bytes(const pgmoe_config &c);
// Workspace bytes one two-GEMM launch of n_rows rows uses.
size_t ffn_gemm_launch_bytes(const pgmoe_config &c, int n_rows);
// The two-GEMM path of launch_ffn (same arguments).
int launch_ffn_gemm(pgmoe_ctx *ctx, const char *w_base, size_t w_stride, bool slot_by_rank, int n_slots, const void *x_rows,
                    const int32_t *offsets, int n_rows, void *y_perm, void *workspace, hipStream_t s, int *keep_partials,
                    const unsigned long long *table, const int32_t *src_row);

}  // namespace pgmoe
#endif  // PGMOE_FFN_COMMON_H
