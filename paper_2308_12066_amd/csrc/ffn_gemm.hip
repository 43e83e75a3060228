// Expert execution for launches with hundreds of rows per expert (Sec. II-B: every activated
// expert, a dense FFN, processes the tokens routed to it): the two products as two tiled GEMMs.
#include "ffn_common.h"

namespace pgmoe {

// ------------------------------------------------------------------------------------------
// Many rows per expert (hundreds): the weights must be reused across many rows, so the two
// products run as two tiled GEMMs with the hidden activation (bf16) parked in the workspace
// between them:
//   ffn_gemm_up_kernel    H[rows, f] = ReLU(X[rows, d] . W1)                       K = d
//   ffn_gemm_down_kernel  partial[s][rows, d] = H[rows, K-slice s] . W2            K = f / n_split
// Both work on chunks of 128 rows of one expert and 128 output columns, four wavefronts as 2 x 2
// with 4 x 4 accumulator tiles each, operands in LDS in operand order.  H is stored PACKED, chunk
// by chunk, as the 1 KiB operand tiles the down-projection needs (see the up kernel's last
// lines), so that the down kernel can load both its operands straight into LDS.
//
// Measured on the 4096-row, 8-expert shape (d 768, f 3072; 19.3 GFLOP per product): up 41 us,
// down 35 us.  What was learnt on the way, in the order it mattered:
//  * matrix-core accumulators must be ordinary vector registers (build flag): with the
//    accumulator-register form the register allocator copies accumulators about inside the k
//    loop and every copy waits for the product before it (6 us per product);
//  * the down kernel's time is that of its load stream alone (loads and barriers without any
//    arithmetic: 33 us; arithmetic and LDS reads without loads: 25 us): 302 MB cross from L2 to
//    the CUs per product and L2 misses on about a quarter of it (per XCD one expert's weights
//    and rows, 7.8 MB, against 4 MB of L2).  Neither a deeper ring (3 to 8 stages), nor more
//    workgroups per CU, nor reading fragments a stage ahead, nor K slices, nor k orders rotated
//    per expert / per column block (memory channels) move it by more than a tenth; a fifth
//    wavefront that touches the lines 8 to 24 stages ahead (to have them in L2) makes it slower
//    (55 us: it has to join every barrier, and the workgroup then waits for its loads too);
//  * 256 x 256 tiles with eight wavefronts halve that traffic and reach 32 us for the down
//    product, but need 256-row chunks, with which the up product is slower; not kept.  The same
//    tile with four wavefronts of 128 x 128 (sixteen 32x32x16 accumulators each, pinned to the
//    accumulation registers from inline assembly, whose last product per accumulator must carry
//    its own wait states because the compiler reads "finished" accumulators at once) is correct
//    but slower still, 40 us: with one wavefront per SIMD every wait is exposed;
//  * for the up product the same direct loads are slower (44 us) than staging through registers:
//    x is row-major, an operand tile then takes 16 bytes from each of 16 rows per lane group
//    and the address unit, not the data, paces the load.  Variants of the register-staged kernel
//    measured earlier and not kept: 192-column tiles, unswizzled cells with 16-row loads (40 %
//    slower), two LDS buffers with one barrier per stage, 256 x 256 tiles with the weights
//    loaded straight into registers.
constexpr int GEMM_ROWS = 128, GEMM_COLS = 128, GEMM_KSTEP = 64, GEMM_RING = 2;

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

__global__ __launch_bounds__(256) void ffn_gemm_up_kernel(
    const __bf16 *__restrict__ x_rows, const int32_t *__restrict__ offsets, int E, int d, int f,
    const char *__restrict__ w_base, size_t w_stride, int slot_by_rank, int n_slots,
    const unsigned long long *__restrict__ table, __bf16 *__restrict__ h_packed,
    const int32_t *__restrict__ src_row) {  // nullable: grouped row r is row src_row[r] of x_rows
    constexpr int WMT = GEMM_ROWS / 32, RT = 2 * WMT, NA = GEMM_ROWS / 32;  // row tiles per wavefront / workgroup, A loads per wavefront and stage
    __shared__ __attribute__((aligned(16))) bf16x8 a_lds[2 * RT * 64];  // [k-tile][row-tile][cell]
    __shared__ __attribute__((aligned(16))) bf16x8 w_lds[2 * 8 * 64];   // [k-tile][n-tile][cell]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wn = wave & 1, wm = wave >> 1;  // 64-column half, 64-row half
    int chunk_id, nb;
    if (!gemm_item(offsets, E, chunk_id, nb)) return;
    const ChunkInfo ci = find_chunk(offsets, E, GEMM_ROWS, chunk_id);
    if (ci.nrows == 0) return;  // uniform over the workgroup
    const char *wexp = table ? reinterpret_cast<const char *>(table[ci.expert])
                             : w_base + (size_t)(slot_by_rank ? ci.slot : ci.expert) * w_stride;
    const bool no_weights = table ? wexp == nullptr : (slot_by_rank && ci.slot >= n_slots);  // no slot: rows are zeroed
    const int n0 = nb * GEMM_COLS;
    // an expert without a slot reads the first blob of the pool instead (a valid address) and
    // its rows are written as zeros below
    const global_bf16x8 *wmat = (const global_bf16x8 *)(no_weights ? w_base : wexp) + lane;
    const int w_kt = d / 32;  // k-tiles of W1, which is stored n-tile major

    // staging: this wavefront's NA row fragments and 4 weight fragments of a 64-k stage, held in a
    // ring of GEMM_RING stages of registers: stage s + GEMM_RING is requested when stage s has been
    // handed to LDS, so a request has GEMM_RING stages of matrix-core work to arrive in
    const int tok = lane & 15, g = lane >> 4;
    bf16x8 sa[GEMM_RING][NA], sw[GEMM_RING][4];
    // Rows are fetched as whole 128-byte lines (8 lanes per row, 8 rows per load), so inside
    // LDS the 16-byte cells of a fragment are placed by a swizzle that keeps both the row-major
    // writes and the operand-order reads (lane = token + 16 * k-group) free of bank conflicts.
    auto cell_of = [](int t, int kg, int kt) { return 16 * (t >> 2) + 4 * ((t & 3) ^ ((kt & 1) << 1)) + (kg ^ (t >> 2)); };
    const int ld_row = lane >> 3, ld_kt = (lane >> 2) & 1, ld_kg = lane & 3;
    // where this lane's NA rows start in x_rows (rows past the chunk's end read the chunk's last
    // row, a valid address; what is computed for them is never stored)
    size_t a_off[NA];
#pragma unroll
    for (int i = 0; i < NA; ++i) {
        const int row = ci.row0 + min((wave * NA + i) * 8 + ld_row, ci.nrows - 1);
        a_off[i] = (size_t)(src_row ? src_row[row] : row) * d + 8 * (lane & 7);
    }
    auto request = [&](int k0, bf16x8 (&ra)[NA], bf16x8 (&rw)[4]) {
        // nothing may touch a loaded value before it goes to LDS, or the wait for it would move
        // up to here and undo the prefetch
#pragma unroll
        for (int i = 0; i < NA; ++i) ra[i] = *(const global_bf16x8 *)(x_rows + a_off[i] + k0);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int idx = wave * 4 + i, kt = idx >> 3, nt = idx & 7;
            rw[i] = wmat[((size_t)((n0 >> 4) + nt) * w_kt + (k0 >> 5) + kt) << 6];
        }
    };
    // where this lane's staged row cells go, and where its operand cells are read from
    int st_cell[NA];
#pragma unroll
    for (int i = 0; i < NA; ++i) {
        const int r = (wave * NA + i) * 8 + ld_row;
        st_cell[i] = (ld_kt * RT + (r >> 4)) * 64 + cell_of(r & 15, ld_kg, ld_kt);
    }
    const int rd_cell0 = cell_of(tok, g, 0), rd_cell1 = cell_of(tok, g, 1);

    floatx4 acc[4][WMT];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int m = 0; m < WMT; ++m) acc[a][m] = floatx4{0.f, 0.f, 0.f, 0.f};

    // n_stage is a multiple of GEMM_RING (the launcher checks), and a request past the last stage
    // re-reads the last one instead of being skipped: the loop body has no conditional around the
    // ring registers, so the compiler never has to merge (and thereby wait for) loaded values.
    const int n_stage = d / GEMM_KSTEP;
    const int k_last = d - GEMM_KSTEP;
#pragma unroll
    for (int r = 0; r < GEMM_RING; ++r) request(min(r * GEMM_KSTEP, k_last), sa[r], sw[r]);
    for (int s0 = 0; s0 < n_stage; s0 += GEMM_RING) {
#pragma unroll
        for (int r = 0; r < GEMM_RING; ++r) {
            const int st = s0 + r;
            __syncthreads();  // everyone is done reading the previous stage
#pragma unroll
            for (int i = 0; i < NA; ++i) a_lds[st_cell[i]] = sa[r][i];
#pragma unroll
            for (int i = 0; i < 4; ++i) w_lds[(wave * 4 + i) * 64 + lane] = sw[r][i];
            __syncthreads();
            request(min((st + GEMM_RING) * GEMM_KSTEP, k_last), sa[r], sw[r]);
#pragma unroll
            for (int kt = 0; kt < 2; ++kt) {
                bf16x8 wf[4], af[WMT];
#pragma unroll
                for (int a = 0; a < 4; ++a) wf[a] = w_lds[(kt * 8 + wn * 4 + a) * 64 + lane];
#pragma unroll
                for (int m = 0; m < WMT; ++m) af[m] = a_lds[(kt * RT + wm * WMT + m) * 64 + (kt ? rd_cell1 : rd_cell0)];
#pragma unroll
                for (int a = 0; a < 4; ++a)
#pragma unroll
                    for (int m = 0; m < WMT; ++m)
                        acc[a][m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[a], af[m], acc[a][m], 0, 0, 0);
            }
        }
    }

    // Lane holds row r = wm*64 + m*16 + tok, hidden features n0 + wn*64 + a*16 + 4*g + {0..3}.
    // Packed layout of H: per chunk [f/32 k-tiles][RT row tiles][1 KiB]; a tile holds 16 rows x 32
    // features in matrix-core operand order: cell row%16 + 16*((feature%32)/8), 8 features per
    // cell.  Rows past the chunk's end are left unwritten (the down kernel never stores what it
    // computes from them).
#pragma unroll
    for (int m = 0; m < WMT; ++m) {
        const int r = wm * 16 * WMT + m * 16 + tok;
        if (r >= ci.nrows) continue;
        __bf16 *dst = h_packed + (size_t)chunk_id * GEMM_ROWS * f + (size_t)(r >> 4) * 512 + (tok + 16 * (g >> 1)) * 8 + 4 * (g & 1);
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            bf16x4 o;
            o.x = (__bf16)fmaxf(acc[a][m].x, 0.f);
            o.y = (__bf16)fmaxf(acc[a][m].y, 0.f);
            o.z = (__bf16)fmaxf(acc[a][m].z, 0.f);
            o.w = (__bf16)fmaxf(acc[a][m].w, 0.f);
            if (no_weights) o = bf16x4{0, 0, 0, 0};
            const int kt = (n0 >> 5) + wn * 2 + (a >> 1);  // k-tile of the down-projection these 16 features fall in
            *reinterpret_cast<bf16x4 *>(dst + (size_t)kt * RT * 512 + (a & 1) * 32 * 8) = o;
        }
    }
}

// Down-projection with both operands loaded straight into LDS (global_load_lds_dwordx4: each
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

template <int NS>
__global__ __launch_bounds__(256) void ffn_gemm_down_kernel(
    const char *__restrict__ h_packed, const int32_t *__restrict__ offsets, int E, int d, int f, int n_split,
    const char *__restrict__ w_base, size_t w_stride, int slot_by_rank, int n_slots,
    const unsigned long long *__restrict__ table, float *__restrict__ partial, int n_rows) {
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

    const int n_blocks = d / GEMM_COLS;
    const int nb = col_id % n_blocks, split = col_id / n_blocks;
    const int n0 = nb * GEMM_COLS;
    const int n_kt = f / n_split / 32, kt0 = split * n_kt;
    const int w_nt = d / 16;  // W2 is stored k-tile major
    // This wavefront brings row tiles and column tiles (TPW/2)*wave .. of every stage;
    // src[i]: this lane's 16 bytes of its i-th tile for the k-tile to request next.
    const char *src[TPW];
    size_t step[TPW];  // to the same tile of the next k-tile
#pragma unroll
    for (int i = 0; i < TPW / 2; ++i) {
        const int t = (TPW / 2) * wave + i;
        src[i] = h_packed + (size_t)chunk_id * GEMM_ROWS * f * 2 + ((size_t)kt0 * NT + t) * 1024 + lane * 16;
        step[i] = NT * 1024;
        src[TPW / 2 + i] = wsafe + (size_t)d * f * 2 + ((size_t)kt0 * w_nt + (n0 >> 4) + t) * 1024 + lane * 16;
        step[TPW / 2 + i] = (size_t)w_nt * 1024;
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
        float *dst = partial + ((size_t)split * n_rows + (size_t)ci.row0 + r) * d + n0 + wn * 64 + 4 * g;
#pragma unroll
        for (int a = 0; a < 4; ++a)
            *reinterpret_cast<floatx4 *>(dst + a * 16) = no_weights ? floatx4{0.f, 0.f, 0.f, 0.f} : acc[a][m];
    }
}

// The two-GEMM path pays off once an expert sees enough rows for its weights to be reused out
// of LDS many times: at least 192 rows per expert on average.
constexpr int GEMM_SPLIT = 4;  // most K slices of the down-projection (float32 partials)
bool uses_gemm_kernels(const pgmoe_config &c, int n_rows) {
    if (c.dtype != PGMOE_BF16) return false;
    // the up kernel's k loop runs in whole rings of 64-k stages, the down kernel's two 32-k tiles per turn in every K slice
    if (c.d_model % GEMM_COLS || c.d_ff % GEMM_COLS || c.d_model % (GEMM_KSTEP * GEMM_RING) || c.d_ff % (GEMM_SPLIT * 64)) return false;
    const int active = std::max(1, std::min(c.n_experts, n_rows));
    return n_rows / active >= 192;
}

// float32 partials of the down-projection (most K slices), then the bf16 hidden activation in
// 128-row chunks, at most one partly filled chunk per expert
size_t ffn_gemm_workspace_bytes(const pgmoe_config &c) {
    const int64_t max_rows = (int64_t)c.max_tokens * c.top_k;
    return (size_t)GEMM_SPLIT * max_rows * c.d_model * 4 +
           (size_t)(max_rows / GEMM_ROWS + std::min<int64_t>(c.n_experts, max_rows)) * GEMM_ROWS * c.d_ff * 2 + 256;
}

// K slices of the down-projection: as few as still give every CU a workgroup (fewer float32
// partials to write and to add up); one slice runs one workgroup per CU with a deeper ring, more
// slices two per CU
static int gemm_split(const pgmoe_config &c, int n_rows) {
    const int tiles = (n_rows / GEMM_ROWS) * (c.d_model / GEMM_COLS);
    return tiles >= 160 ? 1 : (tiles >= 80 ? 2 : GEMM_SPLIT);
}

// Workspace one launch of n_rows rows uses: the float32 partials, then the packed hidden activation.
size_t ffn_gemm_launch_bytes(const pgmoe_config &c, int n_rows) {
    const int active = std::max(1, std::min(c.n_experts, n_rows));
    const int max_chunks = active + n_rows / GEMM_ROWS;
    return (size_t)gemm_split(c, n_rows) * n_rows * c.d_model * 4 + (size_t)max_chunks * GEMM_ROWS * c.d_ff * 2;
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
    if (h_bytes + p_bytes > ffn_workspace_bytes(c))
        return fail(ctx, PGMOE_EINVAL, "pgmoe_expert_ffn: hidden activation and partial sums of %d rows do not fit the workspace", n_rows);
    float *partial = (float *)workspace;
    __bf16 *h = (__bf16 *)((char *)workspace + p_bytes);
    const int tslot = ffn_timing_slot(ctx);
    if (tslot >= 0) PG_HIP(ctx, hipEventRecord(ctx->tim_begin[tslot], s));
    hipLaunchKernelGGL(ffn_gemm_up_kernel, dim3(max_chunks, c.d_ff / GEMM_COLS), dim3(256), 0, s, (const __bf16 *)x_perm, offsets,
                       c.n_experts, c.d_model, c.d_ff, w_base, w_stride, slot_by_rank ? 1 : 0, n_slots, table, h, src_row);
    PG_HIP(ctx, hipGetLastError());
    const dim3 grid_down(max_chunks, (c.d_model / GEMM_COLS) * split);
#define PG_DOWN(NS_)                                                                                                             \
do {                                                                                                                         \
    constexpr int lds = NS_ * 2 * (GEMM_ROWS / 16) * 1024;                                                                   \
    if (int rc_ = allow_dynamic_lds(ctx, reinterpret_cast<const void *>(ffn_gemm_down_kernel<NS_>), lds)) return rc_;       \
    hipLaunchKernelGGL(ffn_gemm_down_kernel<NS_>, grid_down, dim3(256), lds, s, (const char *)h, offsets, c.n_experts,       \
                       c.d_model, c.d_ff, split, w_base, w_stride, slot_by_rank ? 1 : 0, n_slots, table, partial, n_rows);   \
} while (0)
    if (split == 1) PG_DOWN(6);
    else PG_DOWN(4);
#undef PG_DOWN
    PG_HIP(ctx, hipGetLastError());
    if (tslot >= 0) PG_HIP(ctx, hipEventRecord(ctx->tim_end[tslot], s));
    if (keep_partials) {
        *keep_partials = split;
        return PGMOE_OK;
    }
    return launch_ffn_reduce(ctx, partial, split, n_rows, y_perm, s);
}

}  // namespace pgmoe
