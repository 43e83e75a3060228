// Expert execution for launches with hundreds of rows per expert (Sec. II-B: every activated
// expert, a dense FFN, processes the tokens routed to it): the two products as two tiled GEMMs.
#include "ffn_common.h"

namespace pgmoe {

// ------------------------------------------------------------------------------------------
// Many rows per expert (hundreds): the weights must be reused across many rows, so the two
// products run as two tiled GEMMs with the hidden activation (bf16) parked in the workspace
// between them, after a small kernel that gathers the rows and packs them as operand tiles:
//   ffn_gemm_pack_rows_kernel   Xp = rows of x, chunk by chunk, as 1 KiB operand tiles
//   ffn_gemm_tile_kernel<UP>    H[rows, f] = ReLU(Xp . W1)                           K = d
//   ffn_gemm_tile_kernel<DOWN>  partial[s][rows, d] = H[rows, K-slice s] . W2        K = f / n_split
// Both products work on chunks of 128 rows of one expert and 128 output columns, four wavefronts
// as 2 x 2 with 4 x 4 accumulator tiles each, and load BOTH operands straight from memory into
// LDS in operand order (every operand tile is 1 KiB contiguous: the packed rows, the packed
// hidden activation the up-projection writes, and the pre-tiled weights).
//
// Measured on the 4096-row, 8-expert shape (d 768, f 3072; 19.3 GFLOP per product): pack 5 us,
// up 32 us, down 35 us (the vendor GEMM library: 27 + 41 us for the two products, no gather, no
// ReLU).  What was learnt on the way, in the order it mattered:
//  * matrix-core accumulators must be ordinary vector registers (build flag): with the
//    accumulator-register form the register allocator copies accumulators about inside the k
//    loop and every copy waits for the product before it (6 us per product);
//  * a product's time is that of its load stream alone (down-projection: loads and barriers
//    without any arithmetic 33 us; arithmetic and LDS reads without loads 25 us): about 300 MB
//    cross from L2 to the CUs per product and L2 misses on a quarter to a third of it (per XCD
//    one expert's weights and rows against 4 MB of L2); a workgroup advances only when the
//    slowest of a stage's sixteen tiles is there.  Neither a deeper ring (3 to 8 stages), nor
//    more workgroups per CU, nor reading fragments a stage ahead, nor K slices, nor k orders
//    rotated per expert / per column block (memory channels), nor the items of several chunks
//    ordered column block by column block, nor v_mfma_f32_32x32x16_bf16 on the same tiles move
//    it by more than a tenth; a fifth wavefront that touches the lines 16 stages ahead (to have
//    them in L2) makes it slower (50 us: its touches are as many L2 requests as the loads);
//  * 256 x 256 tiles with eight wavefronts halve that traffic and reach 32 us for the down
//    product; not kept.  The same tile with four wavefronts of 128 x 128 (sixteen 32x32x16
//    accumulators each, pinned to the accumulation registers from inline assembly) is correct
//    but slower still, 40 us: with one wavefront per SIMD every wait is exposed;
//  * the up-projection first staged row-major x through registers into LDS (41 us; direct loads
//    of row-major x are slower still, 44 us: an operand tile takes 16 bytes from each of 16 rows
//    per lane group and the address unit, not the data, paces the load).  Packing the rows once
//    (5 us) and loading them like every other operand is 3 us faster in all and leaves one
//    kernel for both products.
constexpr int GEMM_ROWS = 128, GEMM_COLS = 128;

// XCD-aware dealing of the (chunk, column block) items of a GEMM launch.  Workgroups go to the 8
// XCDs round-robin in launch order and every XCD has its own L2; the items that exist are dealt
// out so that each XCD works through one contiguous run of them, chunk-major: the workgroups
// that share a chunk's rows, and the chunks that share an expert's weights, meet in one L2.
// False: this workgroup has no item (uniform over the workgroup).
__device__ inline bool gemm_item(const int32_t *__restrict__ offsets, int E, int &chunk_id, int &col_id) {
    const int gy = gridDim.y;
    const int n_items = count_chunks(offsets, E, GEMM_ROWS) * gy;
    const int lin = blockIdx.y * gridDim.x + blockIdx.x;
    const int xcd = lin & 7, turn = lin >> 3;
    if (turn >= (n_items >> 3) + (xcd < (n_items & 7) ? 1 : 0)) return false;
    const int item = xcd * (n_items >> 3) + min(xcd, n_items & 7) + turn;
    chunk_id = item / gy;
    col_id = item - chunk_id * gy;
    return true;
}

// The rows of every 128-row chunk, gathered through the row -> token map and stored as the 1 KiB
// operand tiles the tile kernel below loads straight into LDS: per chunk [d/32 k-tiles][8 row
// tiles][1 KiB], a tile holding 16 rows x 32 features in matrix-core operand order (cell row%16 +
// 16*((feature%32)/8), 8 features per cell): the layout of the packed hidden activation.  Rows
// past the chunk's end are zero.  One workgroup packs PACK_KT k-tiles of one chunk: wavefront w
// packs row tiles w and w + 4, a lane reads 16 bytes of two rows per k-tile (64 contiguous bytes
// per row and wavefront) and consecutive lanes write consecutive cells, so whole tiles go out as
// contiguous kilobytes; every load is requested before the first store.
constexpr int PACK_KT = 2;
__global__ __launch_bounds__(256) void ffn_gemm_pack_rows_kernel(
    const __bf16 *__restrict__ x_rows, const int32_t *__restrict__ offsets, int E, int d,
    const int32_t *__restrict__ src_row,  // nullable: grouped row r is row src_row[r] of x_rows
    __bf16 *__restrict__ x_packed) {
    const ChunkInfo ci = find_chunk(offsets, E, GEMM_ROWS, blockIdx.x);
    if (ci.nrows == 0) return;  // uniform over the workgroup
    constexpr int RT = GEMM_ROWS / 16;
    const int kt0 = blockIdx.y * PACK_KT;
    const int cell = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint4 *src = reinterpret_cast<const uint4 *>(x_rows);
    uint4 *dst = reinterpret_cast<uint4 *>(x_packed) + (size_t)blockIdx.x * GEMM_ROWS * (d >> 3);
    const int cells_per_row = d >> 3;
    size_t from[RT / 4];
    bool live[RT / 4];
#pragma unroll
    for (int j = 0; j < RT / 4; ++j) {
        const int row = (wave + 4 * j) * 16 + (cell & 15);
        live[j] = row < ci.nrows;
        const int r = ci.row0 + (live[j] ? row : 0);
        from[j] = (size_t)(src_row ? src_row[r] : r) * cells_per_row + (cell >> 4);
    }
    uint4 v[RT / 4][PACK_KT];
#pragma unroll
    for (int j = 0; j < RT / 4; ++j)
#pragma unroll
        for (int k = 0; k < PACK_KT; ++k) v[j][k] = src[from[j] + (size_t)(kt0 + k) * 4];
#pragma unroll
    for (int j = 0; j < RT / 4; ++j)
#pragma unroll
        for (int k = 0; k < PACK_KT; ++k)
            dst[((size_t)(kt0 + k) * RT + wave + 4 * j) * 64 + cell] = live[j] ? v[j][k] : make_uint4(0, 0, 0, 0);
}

// One product with both operands loaded straight into LDS (global_load_lds_dwordx4: each
// lane's 16 bytes land at LDS base + 16 * lane, so a 1 KiB operand tile that is contiguous in
// memory arrives in operand order with no register round trip and no staging writes).  A stage
// is one 32-k tile of both operands (8 + 8 KiB); NS stages of LDS form a ring.
//
// The loads are issued from inline assembly rather than through the compiler's builtin: the
// compiler cannot tell which stage a later LDS read belongs to and would wait for every load in
// flight before it, which is exactly the prefetch.  Here the kernel counts its own loads (they
// complete in order) and waits with explicit s_waitcnt vmcnt.  M0 (the LDS base of such a load)
// is written inside the statement; nothing else in this kernel keeps a value in M0.
__device__ inline unsigned lds_address(const void *p) {
    return (unsigned)(size_t)(__attribute__((address_space(3))) const char *)p;
}
__device__ inline void load_tile_to_lds(const char *src_lane, unsigned lds_tile) {  // src_lane: this lane's 16 bytes
    asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(src_lane), "s"(lds_tile) : "memory", "m0");
}

// UP = false: the down-projection, partial[s][rows, N] = A[rows, K-slice s] . W2 with K = f, N = d.
// UP = true : the up-projection, H = ReLU(A . W1) with K = d, N = f, A the packed rows, W1's tiles
//             n-tile major (the k-tiles of one 16-column slab are contiguous), the result rounded
//             to bf16 and stored packed for the down-projection.
template <int NS, bool UP>
__global__ __launch_bounds__(256) void ffn_gemm_tile_kernel(
    const char *__restrict__ a_packed, const int32_t *__restrict__ offsets, int E, int K, int N, int n_split,
    const char *__restrict__ w_base, size_t w_stride, int slot_by_rank, int n_slots,
    const unsigned long long *__restrict__ table, void *__restrict__ out, int n_rows) {
    constexpr int NT = GEMM_ROWS / 16;     // 1 KiB tiles per operand and stage (GEMM_COLS / 16 is the same)
    constexpr int TPW = 2 * NT / 4;        // tiles a wavefront brings per stage: TPW/2 row tiles, TPW/2 column tiles
    constexpr int STAGE = 2 * NT * 1024;   // per stage: NT row tiles, then NT column tiles
    static_assert(GEMM_ROWS == GEMM_COLS && NS >= 3 && TPW * (NS - 2) < 64, "NS - 1 stages of TPW loads per wavefront in flight");
    extern __shared__ __attribute__((aligned(1024))) char ring[];  // NS stages
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wn = wave & 1, wm = wave >> 1;
    int chunk_id, col_id;
    if (!gemm_item(offsets, E, chunk_id, col_id)) return;
    const ChunkInfo ci = find_chunk(offsets, E, GEMM_ROWS, chunk_id);
    if (ci.nrows == 0) return;  // uniform over the workgroup
    const char *wexp = table ? reinterpret_cast<const char *>(table[ci.expert])
                             : w_base + (size_t)(slot_by_rank ? ci.slot : ci.expert) * w_stride;
    const bool no_weights = table ? wexp == nullptr : (slot_by_rank && ci.slot >= n_slots);
    const char *wsafe = no_weights ? w_base : wexp;  // a valid address; the rows are written as zeros below

    const int n_blocks = N / GEMM_COLS;
    const int nb = col_id % n_blocks, split = col_id / n_blocks;
    const int n0 = nb * GEMM_COLS;
    const int n_kt = K / n_split / 32, kt0 = split * n_kt;
    const int w_nt = N / 16;  // W2 is stored k-tile major, W1 n-tile major
    // This wavefront brings row tiles and column tiles (TPW/2)*wave .. of every stage;
    // src[i]: this lane's 16 bytes of its i-th tile for the k-tile to request next.
    const char *src[TPW];
    size_t step[TPW];  // to the same tile of the next k-tile
#pragma unroll
    for (int i = 0; i < TPW / 2; ++i) {
        const int t = (TPW / 2) * wave + i;
        src[i] = a_packed + (size_t)chunk_id * GEMM_ROWS * K * 2 + ((size_t)kt0 * NT + t) * 1024 + lane * 16;
        step[i] = NT * 1024;
        if (UP) {
            src[TPW / 2 + i] = wsafe + ((size_t)((n0 >> 4) + t) * (K / 32) + kt0) * 1024 + lane * 16;
            step[TPW / 2 + i] = 1024;
        } else {
            src[TPW / 2 + i] = wsafe + (size_t)K * N * 2 + ((size_t)kt0 * w_nt + (n0 >> 4) + t) * 1024 + lane * 16;
            step[TPW / 2 + i] = (size_t)w_nt * 1024;
        }
    }
    const unsigned ring_lds = lds_address(ring) + __builtin_amdgcn_readfirstlane((TPW / 2) * wave * 1024);
    auto issue = [&](unsigned stage_off) {  // the next k-tile of this wavefront's tiles, into the stage at stage_off
#pragma unroll
        for (int i = 0; i < TPW / 2; ++i) {
            load_tile_to_lds(src[i], ring_lds + stage_off + i * 1024);
            load_tile_to_lds(src[TPW / 2 + i], ring_lds + stage_off + NT * 1024 + i * 1024);
        }
    };
    auto advance = [&](int requested) {  // a request past the last k-tile re-reads the last one
        if (requested < n_kt) {
#pragma unroll
            for (int i = 0; i < TPW; ++i) src[i] += step[i];
        }
    };

    floatx4 acc[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int m = 0; m < 4; ++m) acc[a][m] = floatx4{0.f, 0.f, 0.f, 0.f};

    // NS - 1 stages are requested ahead.  The surplus requests at the end go into a stage nobody
    // needs and keep the count of outstanding loads uniform.
    int ahead = 0;  // k-tiles requested so far
    for (; ahead < NS - 1; ++ahead) {
        issue(ahead * STAGE);
        advance(ahead + 1);
    }
    const bf16x8 *A = reinterpret_cast<const bf16x8 *>(ring) + (wm * 4) * 64 + lane;
    const bf16x8 *W = reinterpret_cast<const bf16x8 *>(ring + NT * 1024) + (wn * 4) * 64 + lane;
    auto read_frags = [&](unsigned stage_off, bf16x8 (&wf)[4], bf16x8 (&af)[4]) {
        const bf16x8 *Ac = A + (stage_off >> 4), *Wc = W + (stage_off >> 4);
#pragma unroll
        for (int a = 0; a < 4; ++a) wf[a] = Wc[a * 64];
#pragma unroll
        for (int m = 0; m < 4; ++m) af[m] = Ac[m * 64];
    };
    auto multiply = [&](const bf16x8 (&wf)[4], const bf16x8 (&af)[4]) {
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
            for (int m = 0; m < 4; ++m)
                acc[a][m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[a], af[m], acc[a][m], 0, 0, 0);
    };
    // The operand fragments of stage kt+1 are read from LDS while stage kt is multiplied (two
    // register sets, the loop runs two stages per turn; n_kt is even, the launcher checks).  In
    // turn kt: stage kt+1 has landed for this wavefront (at most the NS-3 stages after it are
    // outstanding) and, after the barrier, for everyone; everyone's reads of stage kt-1 were
    // consumed by matrix-core instructions issued before the barrier, so its buffer takes the
    // request for stage kt+NS-1; the wait on the LDS counter makes that hold wherever the compiler
    // puts the matrix-core instructions (it costs nothing: those fragments are needed right after).
    // A fence here would make the compiler wait for every load in flight.
    bf16x8 wf0[4], af0[4], wf1[4], af1[4];
    asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(TPW * (NS - 2)) : "memory");
    read_frags(0, wf0, af0);
    unsigned nxt = STAGE, refill = (NS - 1) * STAGE;  // byte offsets: the stage to read next, the one to request into
    auto turn = [&](const bf16x8 (&wf)[4], const bf16x8 (&af)[4], bf16x8 (&wf_next)[4], bf16x8 (&af_next)[4]) {
        asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(TPW * (NS - 3)) : "memory");
        issue(refill);
        ++ahead;
        advance(ahead);
        read_frags(nxt, wf_next, af_next);
        multiply(wf, af);
        refill = refill + STAGE == NS * STAGE ? 0 : refill + STAGE;
        nxt = nxt + STAGE == NS * STAGE ? 0 : nxt + STAGE;
    };
    for (int kt = 0; kt < n_kt; kt += 2) {
        turn(wf0, af0, wf1, af1);
        turn(wf1, af1, wf0, af0);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the surplus requests must not outlive the workgroup's LDS

    // lane holds row wm*64 + m*16 + tok, output columns n0 + wn*64 + a*16 + 4*g + {0..3}
    const int tok = lane & 15, g = lane >> 4;
#pragma unroll
    for (int m = 0; m < 4; ++m) {
        const int r = (wm * 4 + m) * 16 + tok;
        if (r >= ci.nrows) continue;
        if (UP) {
            // Packed layout of H: per chunk [N/32 k-tiles][NT row tiles][1 KiB]; a tile holds 16 rows x 32
            // features in matrix-core operand order: cell row%16 + 16*((feature%32)/8), 8 features per
            // cell.  Rows past the chunk's end are left unwritten (the down-projection never stores
            // what it computes from them).
            __bf16 *dst = reinterpret_cast<__bf16 *>(out) + (size_t)chunk_id * GEMM_ROWS * N + (size_t)(r >> 4) * 512 +
                          (tok + 16 * (g >> 1)) * 8 + 4 * (g & 1);
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                bf16x4 o;
                o.x = (__bf16)fmaxf(acc[a][m].x, 0.f);
                o.y = (__bf16)fmaxf(acc[a][m].y, 0.f);
                o.z = (__bf16)fmaxf(acc[a][m].z, 0.f);
                o.w = (__bf16)fmaxf(acc[a][m].w, 0.f);
                if (no_weights) o = bf16x4{0, 0, 0, 0};
                const int kt = (n0 >> 5) + wn * 2 + (a >> 1);  // k-tile of the down-projection these 16 features fall in
                *reinterpret_cast<bf16x4 *>(dst + (size_t)kt * NT * 512 + (a & 1) * 32 * 8) = o;
            }
        } else {
            float *dst = reinterpret_cast<float *>(out) + ((size_t)split * n_rows + (size_t)ci.row0 + r) * N + n0 + wn * 64 + 4 * g;
#pragma unroll
            for (int a = 0; a < 4; ++a)
                *reinterpret_cast<floatx4 *>(dst + a * 16) = no_weights ? floatx4{0.f, 0.f, 0.f, 0.f} : acc[a][m];
        }
    }
}

// The two-GEMM path pays off once an expert sees enough rows for its weights to be reused out
// of LDS many times: at least 192 rows per expert on average.
constexpr int GEMM_SPLIT = 4;  // most K slices of the down-projection (float32 partials)
bool uses_gemm_kernels(const pgmoe_config &c, int n_rows) {
    if (c.dtype != PGMOE_BF16) return false;
    // the k loop takes two 32-k tiles per turn (in every K slice of the down-projection); the pack kernel PACK_KT k-tiles per workgroup
    if (c.d_model % GEMM_COLS || c.d_ff % GEMM_COLS || c.d_model % (32 * PACK_KT) || c.d_ff % (GEMM_SPLIT * 64)) return false;
    const int active = std::max(1, std::min(c.n_experts, n_rows));
    return n_rows / active >= 192;
}

// float32 partials of the down-projection (most K slices), then the bf16 hidden activation and
// the packed rows in 128-row chunks, at most one partly filled chunk per expert
size_t ffn_gemm_workspace_bytes(const pgmoe_config &c) {
    const int64_t max_rows = (int64_t)c.max_tokens * c.top_k;
    return (size_t)GEMM_SPLIT * max_rows * c.d_model * 4 +
           (size_t)(max_rows / GEMM_ROWS + std::min<int64_t>(c.n_experts, max_rows)) * GEMM_ROWS * (c.d_ff + c.d_model) * 2 + 256;
}

// K slices of the down-projection: as few as still give every CU a workgroup (fewer float32
// partials to write and to add up); one slice runs one workgroup per CU with a deeper ring, more
// slices two per CU
static int gemm_split(const pgmoe_config &c, int n_rows) {
    const int tiles = (n_rows / GEMM_ROWS) * (c.d_model / GEMM_COLS);
    return tiles >= 160 ? 1 : (tiles >= 80 ? 2 : GEMM_SPLIT);
}

// Workspace one launch of n_rows rows uses: the float32 partials, the packed hidden activation, the packed rows.
size_t ffn_gemm_launch_bytes(const pgmoe_config &c, int n_rows) {
    const int active = std::max(1, std::min(c.n_experts, n_rows));
    const int max_chunks = active + n_rows / GEMM_ROWS;
    return (size_t)gemm_split(c, n_rows) * n_rows * c.d_model * 4 + (size_t)max_chunks * GEMM_ROWS * (c.d_ff + c.d_model) * 2;
}

int launch_ffn_gemm(pgmoe_ctx *ctx, const char *w_base, size_t w_stride, bool slot_by_rank, int n_slots, const void *x_perm,
                    const int32_t *offsets, int n_rows, void *y_perm, void *workspace, hipStream_t s, int *keep_partials,
                    const unsigned long long *table, const int32_t *src_row) {
    const pgmoe_config &c = ctx->cfg;
    // float32 partials [split][n_rows, d] first (the combine reads them at the workspace's start),
    // then the packed hidden activation, 128-row chunk by chunk (at most one partly filled chunk per expert)
    const int active = std::max(1, std::min(c.n_experts, n_rows));
    const int max_chunks = active + n_rows / GEMM_ROWS;
    const int split = gemm_split(c, n_rows);
    const size_t p_bytes = (size_t)split * n_rows * c.d_model * 4;
    const size_t h_bytes = (size_t)max_chunks * GEMM_ROWS * c.d_ff * 2;
    const size_t xp_bytes = (size_t)max_chunks * GEMM_ROWS * c.d_model * 2;
    if (h_bytes + p_bytes + xp_bytes > ffn_workspace_bytes(c))
        return fail(ctx, PGMOE_EINVAL, "pgmoe_expert_ffn: hidden activation, packed rows and partial sums of %d rows do not fit the workspace", n_rows);
    float *partial = (float *)workspace;
    __bf16 *h = (__bf16 *)((char *)workspace + p_bytes);
    __bf16 *xp = (__bf16 *)((char *)workspace + p_bytes + h_bytes);
    const int tslot = ffn_timing_slot(ctx);
    if (tslot >= 0) PG_HIP(ctx, hipEventRecord(ctx->tim_begin[tslot], s));
    hipLaunchKernelGGL(ffn_gemm_pack_rows_kernel, dim3(max_chunks, c.d_model / 32 / PACK_KT), dim3(256), 0, s, (const __bf16 *)x_perm,
                       offsets, c.n_experts, c.d_model, src_row, xp);
    PG_HIP(ctx, hipGetLastError());
#define PG_TILE(NS_, UP_, GRID_, A_, K_, N_, SPLIT_, OUT_)                                                                       \
do {                                                                                                                         \
    constexpr int lds = NS_ * 2 * (GEMM_ROWS / 16) * 1024;                                                                   \
    auto kern_ = ffn_gemm_tile_kernel<NS_, UP_>;                                                                             \
    if (int rc_ = allow_dynamic_lds(ctx, reinterpret_cast<const void *>(kern_), lds)) return rc_;                            \
    hipLaunchKernelGGL(kern_, GRID_, dim3(256), lds, s, (const char *)(A_), offsets, c.n_experts, K_, N_, SPLIT_, w_base,    \
                       w_stride, slot_by_rank ? 1 : 0, n_slots, table, (void *)(OUT_), n_rows);                              \
} while (0)
    // up-projection: a ring of four stages leaves room for two workgroups per CU (its k loop is short)
    const dim3 grid_up(max_chunks, c.d_ff / GEMM_COLS);
    PG_TILE(4, true, grid_up, xp, c.d_model, c.d_ff, 1, h);
    PG_HIP(ctx, hipGetLastError());
    const dim3 grid_down(max_chunks, (c.d_model / GEMM_COLS) * split);
    if (split == 1) PG_TILE(6, false, grid_down, h, c.d_ff, c.d_model, split, partial);
    else PG_TILE(4, false, grid_down, h, c.d_ff, c.d_model, split, partial);
#undef PG_TILE
    PG_HIP(ctx, hipGetLastError());
    if (tslot >= 0) PG_HIP(ctx, hipEventRecord(ctx->tim_end[tslot], s));
    if (keep_partials) {
        *keep_partials = split;
        return PGMOE_OK;
    }
    return launch_ffn_reduce(ctx, partial, split, n_rows, y_perm, s);
}

}  // namespace pgmoe
