// Expert execution (Sec. II-B: every activated expert, a dense FFN, processes the tokens
// routed to it):  y_perm[rows of e] = ReLU(x_perm[rows of e] . W1_e) . W2_e.
//
// bf16 path - three kernels, picked from the shape of the launch alone (plan_ffn and friends):
//   ffn_fused_kernel   the general, HBM-bound case (described next);
//   ffn_decode_kernel  a handful of active experts with <= 16 rows each (batch-1 decode);
//   ffn_gemm_up_kernel + ffn_gemm_down_kernel  hundreds of rows per expert: two tiled GEMMs.
// The fused kernel streams the weights from HBM exactly once per 16*MT-row chunk:
//   workgroup = (chunk of <= 16*MT rows of one expert) x (a range of d_ff columns)
//   = (blockIdx.x, blockIdx.y).
//   It keeps the chunk's activations in LDS, already in matrix-core operand order, and walks
//   its d_ff range in sub-slabs of SUB = 16*NW columns (NW wavefronts per workgroup):
//     phase A  wave w computes the 16 hidden features of n-tile w over the full d_model
//              reduction (W1 tiles are contiguous in memory along k), applies ReLU, rounds to
//              bf16 and drops the result into LDS in operand order for phase B;
//     phase B  every wave multiplies that sub-slab of hidden features into its own d_model/NW
//              output columns (W2 tiles of one k-tile are contiguous along n) and keeps the
//              running output in registers across all sub-slabs.
//   The hidden activation never leaves the CU.  With P > 1 d_ff ranges per chunk the partial
//   outputs go to a float32 scratch [P][rows][d] and ffn_reduce_kernel adds them in fixed
//   order (no atomics: results are bit-reproducible); with P == 1 the kernel writes y_perm.
//   The weights are the A operand (v_mfma_f32_16x16x32_bf16, 16 features x 32 k) and the
//   tokens the B operand, so each lane ends up with 4 consecutive features of one token.
//
// f32 path - plain float32 kernels (correctness configuration; no matrix cores).
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

__device__ inline int wave_incl_scan(int v, int lane) {
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int o = __shfl_up(v, off);
        if (lane >= off) v += o;
    }
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
        const int c_incl = wave_incl_scan(c, lane), nz_incl = wave_incl_scan(nz, lane);
        const int c_excl = chunk_base + c_incl - c;
        const bool mine = chunk >= c_excl && chunk < c_excl + c;
        const unsigned long long hit = __ballot(mine);
        if (hit) {
            const int src = __ffsll((long long)hit) - 1;
            const int first = (chunk - __shfl(c_excl, src)) * rows_per_chunk;
            ci.expert = q * 64 + src;
            ci.slot = slot_base + __shfl(nz_incl, src) - 1;
            ci.row0 = __shfl(lo, src) + first;
            ci.nrows = min(rows_per_chunk, __shfl(n, src) - first);
            return ci;
        }
        chunk_base += __shfl(c_incl, 63);
        slot_base += __shfl(nz_incl, 63);
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
        total += __shfl(wave_incl_scan((n + rows_per_chunk - 1) / rows_per_chunk, lane), 63);
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

// MT: 16-row tiles per chunk; KT = d_model/32; NW: wavefronts per workgroup (sub-slab = 16*NW
// d_ff columns); D: weight tiles (1 KiB each) a wavefront keeps in flight.
//
// Per sub-slab a wavefront consumes NT = KT + KTB*NTB weight tiles in a fixed order: first the
// KT tiles of its own W1 n-tile (phase A), then, for each of the KTB k-tiles of the sub-slab,
// its NTB W2 tiles (phase B).  The tiles form one linear stream over all sub-slabs; tile g+D is
// requested when tile g is consumed, so loads run ahead of the matrix cores across both phases
// and across the LDS barrier between them.
template <int MT, int KT, int NW, int D>
__global__ __launch_bounds__(NW * 64) void ffn_fused_kernel(
    const __bf16 *__restrict__ x_perm, const int32_t *__restrict__ offsets, int E, int f, int f_range,
    const char *__restrict__ w_base, size_t w_stride, int slot_by_rank, int n_slots,
    const unsigned long long *__restrict__ table, float *__restrict__ partial, __bf16 *__restrict__ y_perm, int n_rows,
    const int32_t *__restrict__ src_row) {  // nullable: grouped row r is row src_row[r] of x_perm (rows not gathered yet)
    constexpr int SUB = 16 * NW;      // d_ff columns per sub-slab
    constexpr int KTB = SUB / 32;     // k-tiles of phase B per sub-slab
    constexpr int NTD = KT * 2;       // n-tiles of the output (d_model / 16)
    constexpr int NTB = NTD / NW;     // output n-tiles per wavefront
    constexpr int NT_A = KT, NT_B = KTB * NTB, NT = NT_A + NT_B;
    constexpr int d = KT * 32;
    static_assert(NTD % NW == 0 && SUB % 32 == 0, "tile split");
    extern __shared__ __attribute__((aligned(16))) char smem[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    const ChunkInfo ci = find_chunk(offsets, E, 16 * MT, blockIdx.x);
    if (ci.nrows == 0) return;  // uniform over the workgroup
    // where the expert's blob is: through the cache's pointer table, by slot rank, or by expert id
    const char *wexp = table ? reinterpret_cast<const char *>(table[ci.expert])
                             : w_base + (size_t)(slot_by_rank ? ci.slot : ci.expert) * w_stride;
    const bool no_weights = table ? wexp == nullptr : (slot_by_rank && ci.slot >= n_slots);  // no slot: rows are zeroed

    // weights are addressed as global memory explicitly: the blob's address may come out of the
    // cache's pointer table, and a load the compiler cannot prove global becomes a flat load, which
    // also counts on the LDS wait counter and would drain the prefetch ring at every LDS read
    const global_bf16x8 *w1 = (const global_bf16x8 *)wexp + lane;
    const global_bf16x8 *w2 = (const global_bf16x8 *)(wexp + (size_t)d * f * 2) + lane;
    const int n_sub = no_weights ? 0 : f_range / SUB;
    const int fs0 = blockIdx.y * f_range;

    // tile i (0 <= i < NT, compile-time after unrolling) of sub-slab s
    auto tile_ptr = [&](int s, int i) -> const global_bf16x8 * {
        const int fs = fs0 + s * SUB;
        if (i < NT_A) return w1 + (((size_t)((fs >> 4) + wave) * KT + i) << 6);
        const int j = i - NT_A, kb = j / NTB, a = j - kb * NTB;
        return w2 + (((size_t)((fs >> 5) + kb) * NTD + wave * NTB + a) << 6);
    };

    bf16x8 ring[D];
#pragma unroll
    for (int g = 0; g < D; ++g) {
        if (g / NT < n_sub) ring[g] = *tile_ptr(g / NT, g % NT);
    }

    bf16x8 *xs = reinterpret_cast<bf16x8 *>(smem);   // [MT][KT][64] operand cells
    bf16x8 *hs = xs + (size_t)MT * KT * 64;          // [2][MT][KTB][64]

    // stage the chunk's rows (zero-filling rows beyond nrows) while the first weight tiles fly
    {
        constexpr int cells_per_row = d >> 3;
        const uint4 *src = reinterpret_cast<const uint4 *>(x_perm);
        uint4 *dst = reinterpret_cast<uint4 *>(xs);
        for (int i = tid; i < 16 * MT * cells_per_row; i += NW * 64) {
            const int m = i / cells_per_row, k8 = i - m * cells_per_row;
            uint4 v = make_uint4(0, 0, 0, 0);
            if (m < ci.nrows) {
                const int row = ci.row0 + m;
                v = src[(size_t)(src_row ? src_row[row] : row) * cells_per_row + k8];
            }
            dst[(((m >> 4) * KT + (k8 >> 2)) << 6) + (m & 15) + 16 * (k8 & 3)] = v;
        }
    }
    lds_barrier();

    floatx4 yacc[NTB][MT];
#pragma unroll
    for (int a = 0; a < NTB; ++a)
#pragma unroll
        for (int m = 0; m < MT; ++m) yacc[a][m] = floatx4{0.f, 0.f, 0.f, 0.f};

    const int q = lane >> 4;
    for (int s = 0; s < n_sub; ++s) {
        floatx4 hacc[MT];
#pragma unroll
        for (int m = 0; m < MT; ++m) hacc[m] = floatx4{0.f, 0.f, 0.f, 0.f};
        bf16x8 hfrag[MT];
        const bf16x8 *hb = hs + (size_t)(s & 1) * MT * KTB * 64;
#pragma unroll
        for (int i = 0; i < NT; ++i) {
            const bf16x8 v = ring[i % D];
            {   // request tile g + D of the stream
                const int ds = (i + D) / NT, ii = (i + D) % NT;
                if (s + ds < n_sub) ring[i % D] = *tile_ptr(s + ds, ii);
            }
            if (i < NT_A) {
                // ---- phase A: hidden features [fs + 16*wave, +16) over the full d_model reduction
#pragma unroll
                for (int m = 0; m < MT; ++m)
                    hacc[m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(v, xs[((m * KT + i) << 6) + lane], hacc[m], 0, 0, 0);
                if (i == NT_A - 1) {
                    // ReLU, round to bf16, store as phase-B operand: feature 16*wave + 4*q + r is
                    // k-tile wave/2, k-group 2*(wave%2) + q/2, position 4*(q%2) + r of token lane%16
                    char *hbase = reinterpret_cast<char *>(hs + (size_t)(s & 1) * MT * KTB * 64);
#pragma unroll
                    for (int m = 0; m < MT; ++m) {
                        bf16x4 h;
                        h.x = (__bf16)fmaxf(hacc[m].x, 0.f);
                        h.y = (__bf16)fmaxf(hacc[m].y, 0.f);
                        h.z = (__bf16)fmaxf(hacc[m].z, 0.f);
                        h.w = (__bf16)fmaxf(hacc[m].w, 0.f);
                        const int cell = ((m * KTB + (wave >> 1)) << 6) + (lane & 15) + 16 * (2 * (wave & 1) + (q >> 1));
                        *reinterpret_cast<bf16x4 *>(hbase + (size_t)cell * 16 + 8 * (q & 1)) = h;
                    }
                    // one barrier per sub-slab is enough: the next sub-slab writes the other half of hs
                    lds_barrier();
                }
            } else {
                // ---- phase B: y[:, wave's columns] += H_sub . W2[fs .. fs+SUB, wave's columns]
                const int j = i - NT_A, kb = j / NTB, a = j - kb * NTB;
                if (a == 0) {
#pragma unroll
                    for (int m = 0; m < MT; ++m) hfrag[m] = hb[((m * KTB + kb) << 6) + lane];
                }
#pragma unroll
                for (int m = 0; m < MT; ++m)
                    yacc[a][m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(v, hfrag[m], yacc[a][m], 0, 0, 0);
            }
        }
    }

    // ---- epilogue: lane holds token (lane%16) of tile m, output columns 16*(wave*NTB+a) + 4*q + {0..3}
    const int tok = lane & 15;
#pragma unroll
    for (int m = 0; m < MT; ++m) {
        const int r = m * 16 + tok;
        if (r >= ci.nrows) continue;
        const size_t row = (size_t)ci.row0 + r;
        if (partial) {
            float *dst = partial + ((size_t)blockIdx.y * n_rows + row) * d + (wave * NTB) * 16 + 4 * q;
#pragma unroll
            for (int a = 0; a < NTB; ++a) *reinterpret_cast<floatx4 *>(dst + a * 16) = yacc[a][m];
        } else {
            __bf16 *dst = y_perm + row * d + (wave * NTB) * 16 + 4 * q;
#pragma unroll
            for (int a = 0; a < NTB; ++a) {
                bf16x4 o;
                o.x = (__bf16)yacc[a][m].x;
                o.y = (__bf16)yacc[a][m].y;
                o.z = (__bf16)yacc[a][m].z;
                o.w = (__bf16)yacc[a][m].w;
                *reinterpret_cast<bf16x4 *>(dst + a * 16) = o;
            }
        }
    }
}

// Decode-sized variant (at most a few experts active, <= 16 rows each): one workgroup of four
// wavefronts per (chunk, 32-column sub-slab of d_ff), every weight tile it needs requested before
// anything else happens, so the kernel is one round of memory latency deep instead of a ring of
// dependent rounds.  Phase A splits the d_model reduction over wavefront pairs (wave = n-tile
// + 2 * k-half; the two halves are added in LDS, k-half 0 first), phase B gives each wavefront a
// quarter of the output columns.  Always writes float32 partials (one per sub-slab).
template <int KT>
__global__ __launch_bounds__(256) void ffn_decode_kernel(
    const __bf16 *__restrict__ x_perm, const int32_t *__restrict__ offsets, int E, int f,
    const char *__restrict__ w_base, size_t w_stride, int slot_by_rank, int n_slots,
    const unsigned long long *__restrict__ table, float *__restrict__ partial, int n_rows,
    const int32_t *__restrict__ src_row) {  // nullable: grouped row r is row src_row[r] of x_perm
    constexpr int d = KT * 32;
    constexpr int NTD = KT * 2;   // output n-tiles
    constexpr int NA = KT / 2;    // phase-A tiles per wavefront
    constexpr int NB = NTD / 4;   // phase-B tiles per wavefront
    static_assert(KT % 2 == 0, "k split");
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int cw = wave & 1, ks = wave >> 1;

    const ChunkInfo ci = find_chunk(offsets, E, 16, blockIdx.x);
    if (ci.nrows == 0) return;  // uniform over the workgroup
    const char *wexp = table ? reinterpret_cast<const char *>(table[ci.expert])
                             : w_base + (size_t)(slot_by_rank ? ci.slot : ci.expert) * w_stride;
    const bool no_weights = table ? wexp == nullptr : (slot_by_rank && ci.slot >= n_slots);  // no slot: rows are zeroed
    const int fs = blockIdx.y * 32;

    bf16x8 ta[NA], tb[NB];
    if (!no_weights) {
        const global_bf16x8 *w1 = (const global_bf16x8 *)wexp + (((size_t)((fs >> 4) + cw) * KT) << 6) + lane;
        const global_bf16x8 *w2 = (const global_bf16x8 *)(wexp + (size_t)d * f * 2) +
                           (((size_t)(fs >> 5) * NTD + wave * NB) << 6) + lane;
#pragma unroll
        for (int i = 0; i < NA; ++i) ta[i] = w1[(size_t)(ks + 2 * i) << 6];
#pragma unroll
        for (int a = 0; a < NB; ++a) tb[a] = w2[(size_t)a << 6];
    } else {
#pragma unroll
        for (int i = 0; i < NA; ++i) ta[i] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int a = 0; a < NB; ++a) tb[a] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
    }

    bf16x8 *xs = reinterpret_cast<bf16x8 *>(smem);                       // [KT][64] operand cells
    floatx4 *hsum = reinterpret_cast<floatx4 *>(xs + (size_t)KT * 64);   // [2 k-halves][2 n-tiles][64]
    {
        constexpr int cells_per_row = d >> 3;
        const uint4 *src = reinterpret_cast<const uint4 *>(x_perm);
        uint4 *dst = reinterpret_cast<uint4 *>(xs);
        for (int i = tid; i < 16 * cells_per_row; i += 256) {
            const int m = i / cells_per_row, k8 = i - m * cells_per_row;
            uint4 v = make_uint4(0, 0, 0, 0);
            if (m < ci.nrows) {
                const int row = ci.row0 + m;
                v = src[(size_t)(src_row ? src_row[row] : row) * cells_per_row + k8];
            }
            dst[((k8 >> 2) << 6) + m + 16 * (k8 & 3)] = v;
        }
    }
    lds_barrier();

    // ---- phase A: 16 hidden features (n-tile cw of the sub-slab) over this wavefront's k-tiles
    floatx4 hacc = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < NA; ++i)
        hacc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ta[i], xs[((ks + 2 * i) << 6) + lane], hacc, 0, 0, 0);
    hsum[(ks * 2 + cw) * 64 + lane] = hacc;
    lds_barrier();

    // ---- hidden activation as phase-B operand: lane (token lane%16, k-group g = lane/16) needs
    // features 8g .. 8g+7 of the 32, i.e. n-tile g/2, accumulator rows 4*q' + r for q' = 2*(g%2), +1
    const int tok = lane & 15, g = lane >> 4;
    bf16x8 hfrag;
    {
        const int src = (g >> 1) * 64 + (2 * (g & 1)) * 16 + tok;
        const floatx4 lo = hsum[src] + hsum[128 + src];
        const floatx4 hi = hsum[src + 16] + hsum[128 + src + 16];
        hfrag[0] = (__bf16)fmaxf(lo.x, 0.f);
        hfrag[1] = (__bf16)fmaxf(lo.y, 0.f);
        hfrag[2] = (__bf16)fmaxf(lo.z, 0.f);
        hfrag[3] = (__bf16)fmaxf(lo.w, 0.f);
        hfrag[4] = (__bf16)fmaxf(hi.x, 0.f);
        hfrag[5] = (__bf16)fmaxf(hi.y, 0.f);
        hfrag[6] = (__bf16)fmaxf(hi.z, 0.f);
        hfrag[7] = (__bf16)fmaxf(hi.w, 0.f);
    }

    // ---- phase B: this wavefront's NB output n-tiles; lane holds token tok, columns 16*tile + 4*g + {0..3}
    float *dst = partial + ((size_t)blockIdx.y * n_rows + (size_t)ci.row0 + tok) * d + (wave * NB) * 16 + 4 * g;
#pragma unroll
    for (int a = 0; a < NB; ++a) {
        const floatx4 y = __builtin_amdgcn_mfma_f32_16x16x32_bf16(tb[a], hfrag, floatx4{0.f, 0.f, 0.f, 0.f}, 0, 0, 0);
        if (tok < ci.nrows) *reinterpret_cast<floatx4 *>(dst + a * 16) = y;
    }
}

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
    asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(src_lane), "s"(lds_tile) : "memory");
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

// y_perm[row][c] = bf16( sum_p partial[p][row][c] ).  A workgroup of 256 threads covers 256/PL
// float4 columns; its PL "p-lanes" each add every PL-th partial (p = pl, pl+PL, ...) and the PL
// sub-sums are added in ascending order, so the result does not depend on scheduling.  PL is
// picked from P alone (1 for P <= 2, 4 for P <= 8, else 16).
template <int PL>
__global__ __launch_bounds__(256) void ffn_reduce_kernel(const float *__restrict__ partial, int P, int n_rows, int d,
                                                          __bf16 *__restrict__ y_perm) {
    constexpr int COLS = 256 / PL;
    __shared__ floatx4 sub[PL][COLS + 1];
    const size_t total4 = (size_t)n_rows * d / 4;
    const int col = threadIdx.x % COLS, pl = threadIdx.x / COLS;
    const size_t i = (size_t)blockIdx.x * COLS + col;
    floatx4 s = floatx4{0.f, 0.f, 0.f, 0.f};
    if (i < total4) {
        const floatx4 *src = reinterpret_cast<const floatx4 *>(partial) + i;
        for (int p = pl; p < P; p += PL) s += src[(size_t)p * total4];
    }
    static_assert(PL == 1 || PL == 4 || PL == 16, "keep in step with reduce_lanes()");
    if (PL > 1) {
        sub[pl][col] = s;
        __syncthreads();
        if (pl != 0) return;
        s = sub[0][col];
#pragma unroll
        for (int k = 1; k < PL; ++k) s += sub[k][col];
    }
    if (i < total4) {
        bf16x4 o;
        o.x = (__bf16)s.x;
        o.y = (__bf16)s.y;
        o.z = (__bf16)s.z;
        o.w = (__bf16)s.w;
        reinterpret_cast<bf16x4 *>(y_perm)[i] = o;
    }
}

// ------------------------------------------------------------------------------------------
// float32 path.  One workgroup per (row = blockIdx.x, 256 output columns = blockIdx.y); the row's expert and slot are
// found once per workgroup.
__device__ inline void find_row_expert(const int32_t *offsets, int E, int row, int *expert, int *slot) {
    int e = 0, s = -1;
    for (int i = 0; i < E; ++i) {
        const int lo = offsets[i], hi = offsets[i + 1];
        if (hi > lo) ++s;
        if (row >= lo && row < hi) {
            e = i;
            break;
        }
    }
    *expert = e;
    *slot = s < 0 ? 0 : s;
}

__global__ __launch_bounds__(256) void ffn_f32_hidden_kernel(const float *__restrict__ x_perm,
                                                              const int32_t *__restrict__ offsets, int E, int d, int f,
                                                              const char *__restrict__ w_base, size_t w_stride,
                                                              int slot_by_rank, int n_slots,
                                                              const unsigned long long *__restrict__ table,
                                                              float *__restrict__ h) {
    __shared__ int s_e, s_s;
    const int row = blockIdx.x;
    if (threadIdx.x == 0) find_row_expert(offsets, E, row, &s_e, &s_s);
    __syncthreads();
    const float *w1 = table ? reinterpret_cast<const float *>(table[s_e])
                            : reinterpret_cast<const float *>(w_base + (size_t)(slot_by_rank ? s_s : s_e) * w_stride);
    const int j = blockIdx.y * 256 + threadIdx.x;
    if (j >= f) return;
    if (table ? w1 == nullptr : (slot_by_rank && s_s >= n_slots)) {  // expert did not get a slot
        h[(size_t)row * f + j] = 0.f;
        return;
    }
    const float *xr = x_perm + (size_t)row * d;
    float acc = 0.f;
    for (int i = 0; i < d; ++i) acc = fmaf(xr[i], w1[(size_t)i * f + j], acc);
    h[(size_t)row * f + j] = fmaxf(acc, 0.f);
}

__global__ __launch_bounds__(256) void ffn_f32_out_kernel(const float *__restrict__ h, const int32_t *__restrict__ offsets,
                                                           int E, int d, int f, const char *__restrict__ w_base,
                                                           size_t w_stride, int slot_by_rank, int n_slots,
                                                           const unsigned long long *__restrict__ table,
                                                           float *__restrict__ y_perm) {
    __shared__ int s_e, s_s;
    const int row = blockIdx.x;
    if (threadIdx.x == 0) find_row_expert(offsets, E, row, &s_e, &s_s);
    __syncthreads();
    const float *wb = table ? reinterpret_cast<const float *>(table[s_e])
                            : reinterpret_cast<const float *>(w_base + (size_t)(slot_by_rank ? s_s : s_e) * w_stride);
    const float *w2 = wb + (size_t)d * f;
    const int c = blockIdx.y * 256 + threadIdx.x;
    if (c >= d) return;
    if (table ? wb == nullptr : (slot_by_rank && s_s >= n_slots)) {
        y_perm[(size_t)row * d + c] = 0.f;
        return;
    }
    const float *hr = h + (size_t)row * f;
    float acc = 0.f;
    for (int j = 0; j < f; ++j) acc = fmaf(hr[j], w2[(size_t)j * d + c], acc);
    y_perm[(size_t)row * d + c] = acc;
}

// ------------------------------------------------------------------------------------------
static int smallest_divisor_at_least(int n, int want) {
    for (int p = std::max(1, want); p <= n; ++p)
        if (n % p == 0) return p;
    return n;
}

// Geometry of the fused kernel for n_rows rows, from the shape of the launch alone.
FfnPlan plan_ffn(const pgmoe_config &c, int n_rows) {
    FfnPlan p;
    const int E = c.n_experts;
    const int kt = c.d_model / 32;
    const int active = std::max(1, std::min(E, n_rows));  // upper bound of the distinct experts
    const int mean_rows = (n_rows + E - 1) / E;
    // rows per chunk: 16 for decode-sized batches, up to 64 when experts see tens of rows
    int mt = mean_rows <= 4 ? 1 : (mean_rows <= 20 ? 2 : 4);
    // wavefronts per workgroup: 2 (32-column sub-slabs) when there are too few experts to fill
    // the chip otherwise, 8 for the 64-row chunks (halves the accumulators per wavefront)
    int nw = 4;
    if (mt == 1 && active * (c.d_ff / 64) < 256 && (kt == 24 || kt == 32)) nw = 2;
    if (mt == 4 && (kt == 24 || kt == 32)) nw = 8;
    if (mt == 4 && nw == 4 && kt > 24) mt = 2;
    if (mt == 2 && kt > 32) mt = 1;
    p.mt = mt;
    p.nw = nw;
    p.max_chunks = active + n_rows / (16 * mt);
    const int sub = 16 * nw;
    const int nsub = c.d_ff / sub;
    // partial sums: aim at >= 768 workgroups, but keep the float32 partial traffic
    // (write + read = 8 bytes per element per partial) below ~6 % of the weight bytes
    int want = (768 + active - 1) / active;
    const double traffic_cap = 0.06 * (double)active * c.d_ff / (2.0 * n_rows);
    want = std::max(1, std::min(want, (int)traffic_cap));
    p.n_partial = smallest_divisor_at_least(nsub, std::min(want, nsub));
    p.f_range = c.d_ff / p.n_partial;
    return p;
}

// The decode-sized kernel serves launches of 16-row chunks split into one partial per
// 32-column sub-slab (what plan_ffn picks when only a few experts are active).
static bool uses_decode_kernel(const pgmoe_config &c, const FfnPlan &p) {
    const int kt = c.d_model / 32;
    return p.mt == 1 && p.nw == 2 && p.n_partial == c.d_ff / 32 && (kt == 24 || kt == 32) && !getenv("PGMOE_FFN_NO_DECODE");
}

// The two-GEMM path pays off once an expert sees enough rows for its weights to be reused out
// of LDS many times: at least 192 rows per expert on average.
constexpr int GEMM_SPLIT = 4;  // most K slices of the down-projection (float32 partials)
static bool uses_gemm_kernels(const pgmoe_config &c, int n_rows) {
    if (c.dtype != PGMOE_BF16 || getenv("PGMOE_FFN_NO_GEMM")) return false;
    // the up kernel's k loop runs in whole rings of 64-k stages, the down kernel's two 32-k tiles per turn in every K slice
    if (c.d_model % GEMM_COLS || c.d_ff % GEMM_COLS || c.d_model % (GEMM_KSTEP * GEMM_RING) || c.d_ff % (GEMM_SPLIT * 64)) return false;
    const int active = std::max(1, std::min(c.n_experts, n_rows));
    return n_rows / active >= 192;
}

const char *ffn_kernel_name(const pgmoe_config &c, int n_rows) {
    if (c.dtype == PGMOE_F32) return "ffn_f32_hidden_kernel+ffn_f32_out_kernel";
    if (uses_gemm_kernels(c, n_rows)) return "ffn_gemm_up_kernel+ffn_gemm_down_kernel";
    return uses_decode_kernel(c, plan_ffn(c, n_rows)) ? "ffn_decode_kernel" : "ffn_fused_kernel";
}

size_t ffn_workspace_bytes(const pgmoe_config &c) {
    const int64_t max_rows = (int64_t)c.max_tokens * c.top_k;
    if (c.dtype == PGMOE_F32) return (size_t)max_rows * c.d_ff * 4;
    // worst case over every geometry plan_ffn can pick: one partial per 32-column sub-slab
    const size_t worst = (size_t)(c.d_ff / 32) * std::min<int64_t>(max_rows, 4096) * c.d_model * 4;
    const size_t big = (size_t)16 * max_rows * c.d_model * 4;
    // two-GEMM path: the partials of the down-projection, then the bf16 hidden activation in
    // 128-row chunks, at most one partly filled chunk per expert
    const size_t gemm = (size_t)GEMM_SPLIT * max_rows * c.d_model * 4 +
                        (size_t)(max_rows / GEMM_ROWS + std::min<int64_t>(c.n_experts, max_rows)) * GEMM_ROWS * c.d_ff * 2 + 256;
    return ((std::max(std::max(worst, big), gemm) + 255) & ~(size_t)255);
}

// Next free event pair when FFN timing is on, else -1.
static int timing_slot(pgmoe_ctx *ctx) {
    if (!ctx->tim_on || ctx->tim_n >= ctx->tim_cap) return -1;
    return ctx->tim_n++;
}

template <int MT, int KT, int NW, int D>
static int launch_fused(pgmoe_ctx *ctx, const FfnPlan &p, const char *w_base, size_t w_stride, bool slot_by_rank, int n_slots,
                        const void *x_perm, const int32_t *offsets, int n_rows, void *y_perm, void *workspace,
                        hipStream_t s, int *keep_partials, const unsigned long long *table, const int32_t *src_row) {
    const pgmoe_config &c = ctx->cfg;
    const size_t lds = (size_t)MT * KT * 1024 + 2u * MT * (16 * NW / 32) * 1024;
    auto kern = ffn_fused_kernel<MT, KT, NW, D>;
    static thread_local bool attr_set = false;  // per instantiation
    if (lds > 48 * 1024 && !attr_set) {
        PG_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        attr_set = true;
    }
    float *partial = p.n_partial > 1 ? (float *)workspace : nullptr;
    if (partial && (size_t)p.n_partial * n_rows * c.d_model * 4 > ffn_workspace_bytes(c))
        return fail(ctx, PGMOE_EINVAL, "pgmoe_expert_ffn: %d partial sums of %d rows do not fit the workspace", p.n_partial, n_rows);
    const int tslot = timing_slot(ctx);
    if (tslot >= 0) PG_HIP(ctx, hipEventRecord(ctx->tim_begin[tslot], s));
    hipLaunchKernelGGL(kern, dim3(p.max_chunks, p.n_partial), dim3(NW * 64), lds, s, (const __bf16 *)x_perm, offsets,
                       c.n_experts, c.d_ff, p.f_range, w_base, w_stride, slot_by_rank ? 1 : 0, n_slots, table, partial, (__bf16 *)y_perm,
                       n_rows, src_row);
    PG_HIP(ctx, hipGetLastError());
    if (tslot >= 0) PG_HIP(ctx, hipEventRecord(ctx->tim_end[tslot], s));
    if (keep_partials) {
        *keep_partials = partial ? p.n_partial : 0;
        return PGMOE_OK;
    }
    if (partial) {
        const size_t total4 = (size_t)n_rows * c.d_model / 4;
        const int pl = reduce_lanes(p.n_partial);
        if (pl == 1)
            hipLaunchKernelGGL(ffn_reduce_kernel<1>, dim3((unsigned)((total4 + 255) / 256)), dim3(256), 0, s, partial,
                               p.n_partial, n_rows, c.d_model, (__bf16 *)y_perm);
        else if (pl == 4)
            hipLaunchKernelGGL(ffn_reduce_kernel<4>, dim3((unsigned)((total4 + 63) / 64)), dim3(256), 0, s, partial,
                               p.n_partial, n_rows, c.d_model, (__bf16 *)y_perm);
        else
            hipLaunchKernelGGL(ffn_reduce_kernel<16>, dim3((unsigned)((total4 + 15) / 16)), dim3(256), 0, s, partial,
                               p.n_partial, n_rows, c.d_model, (__bf16 *)y_perm);
        PG_HIP(ctx, hipGetLastError());
    }
    return PGMOE_OK;
}

int launch_ffn(pgmoe_ctx *ctx, const char *w_base, size_t w_stride, bool slot_by_rank, int n_slots, const void *x_perm,
               const int32_t *offsets, int n_rows, void *y_perm, void *workspace, hipStream_t s, int *keep_partials,
               const unsigned long long *table, const int32_t *src_row) {
    const pgmoe_config &c = ctx->cfg;
    if (keep_partials) *keep_partials = 0;
    if (n_rows == 0) return PGMOE_OK;
    if (c.dtype == PGMOE_F32) {
        float *h = (float *)workspace;
        const int tslot = timing_slot(ctx);
        if (tslot >= 0) PG_HIP(ctx, hipEventRecord(ctx->tim_begin[tslot], s));
        hipLaunchKernelGGL(ffn_f32_hidden_kernel, dim3(n_rows, (c.d_ff + 255) / 256), dim3(256), 0, s,
                           (const float *)x_perm, offsets, c.n_experts, c.d_model, c.d_ff, w_base, w_stride,
                           slot_by_rank ? 1 : 0, n_slots, table, h);
        PG_HIP(ctx, hipGetLastError());
        hipLaunchKernelGGL(ffn_f32_out_kernel, dim3(n_rows, (c.d_model + 255) / 256), dim3(256), 0, s, h, offsets,
                           c.n_experts, c.d_model, c.d_ff, w_base, w_stride, slot_by_rank ? 1 : 0, n_slots, table, (float *)y_perm);
        PG_HIP(ctx, hipGetLastError());
        if (tslot >= 0) PG_HIP(ctx, hipEventRecord(ctx->tim_end[tslot], s));
        return PGMOE_OK;
    }
    if (uses_gemm_kernels(c, n_rows)) {
        // float32 partials [split][n_rows, d] first (the combine reads them at the workspace's start),
        // then the packed hidden activation, 128-row chunk by chunk (at most one partly filled chunk per expert)
        const int active = std::max(1, std::min(c.n_experts, n_rows));
        const int max_chunks = active + n_rows / GEMM_ROWS;
        // K slices of the down-projection: as few as still give every CU a workgroup (fewer
        // float32 partials to write and to add up); one slice runs one workgroup per CU with a
        // deeper ring, more slices two per CU
        const int tiles = (n_rows / GEMM_ROWS) * (c.d_model / GEMM_COLS);
        const int split = tiles >= 160 ? 1 : (tiles >= 80 ? 2 : GEMM_SPLIT);
        const size_t p_bytes = (size_t)split * n_rows * c.d_model * 4;
        const size_t h_bytes = (size_t)max_chunks * GEMM_ROWS * c.d_ff * 2;
        if (h_bytes + p_bytes > ffn_workspace_bytes(c))
            return fail(ctx, PGMOE_EINVAL, "pgmoe_expert_ffn: hidden activation and partial sums of %d rows do not fit the workspace", n_rows);
        float *partial = (float *)workspace;
        __bf16 *h = (__bf16 *)((char *)workspace + p_bytes);
        const int tslot = timing_slot(ctx);
        if (tslot >= 0) PG_HIP(ctx, hipEventRecord(ctx->tim_begin[tslot], s));
        hipLaunchKernelGGL(ffn_gemm_up_kernel, dim3(max_chunks, c.d_ff / GEMM_COLS), dim3(256), 0, s, (const __bf16 *)x_perm, offsets,
                           c.n_experts, c.d_model, c.d_ff, w_base, w_stride, slot_by_rank ? 1 : 0, n_slots, table, h, src_row);
        PG_HIP(ctx, hipGetLastError());
        const dim3 grid_down(max_chunks, (c.d_model / GEMM_COLS) * split);
#define PG_DOWN(NS_)                                                                                                             \
    do {                                                                                                                         \
        constexpr int lds = NS_ * 2 * (GEMM_ROWS / 16) * 1024;                                                                   \
        static thread_local bool attr_set = false;                                                                               \
        if (!attr_set) {                                                                                                         \
            PG_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(ffn_gemm_down_kernel<NS_>),                           \
                                            hipFuncAttributeMaxDynamicSharedMemorySize, lds));                                   \
            attr_set = true;                                                                                                     \
        }                                                                                                                        \
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
        const size_t total4 = (size_t)n_rows * c.d_model / 4;
        static_assert(GEMM_SPLIT <= 8, "reduce_lanes() gives 1 or 4 lanes for this many partials");
        if (reduce_lanes(split) == 1)
            hipLaunchKernelGGL(ffn_reduce_kernel<1>, dim3((unsigned)((total4 + 255) / 256)), dim3(256), 0, s, partial, split, n_rows,
                               c.d_model, (__bf16 *)y_perm);
        else
            hipLaunchKernelGGL(ffn_reduce_kernel<4>, dim3((unsigned)((total4 + 63) / 64)), dim3(256), 0, s, partial, split, n_rows,
                               c.d_model, (__bf16 *)y_perm);
        PG_HIP(ctx, hipGetLastError());
        return PGMOE_OK;
    }
    const FfnPlan p = plan_ffn(c, n_rows);
    const int kt = c.d_model / 32;
    if (uses_decode_kernel(c, p)) {
        // a few experts with at most 16 rows each, one partial per 32-column sub-slab
        float *partial = (float *)workspace;
        if ((size_t)p.n_partial * n_rows * c.d_model * 4 > ffn_workspace_bytes(c))
            return fail(ctx, PGMOE_EINVAL, "pgmoe_expert_ffn: %d partial sums of %d rows do not fit the workspace", p.n_partial, n_rows);
        const int tslot = timing_slot(ctx);
        if (tslot >= 0) PG_HIP(ctx, hipEventRecord(ctx->tim_begin[tslot], s));
        const dim3 grid(p.max_chunks, p.n_partial);
        const size_t lds = (size_t)kt * 1024 + 4096;
        if (kt == 24)
            hipLaunchKernelGGL(ffn_decode_kernel<24>, grid, dim3(256), lds, s, (const __bf16 *)x_perm, offsets, c.n_experts, c.d_ff,
                               w_base, w_stride, slot_by_rank ? 1 : 0, n_slots, table, partial, n_rows, src_row);
        else
            hipLaunchKernelGGL(ffn_decode_kernel<32>, grid, dim3(256), lds, s, (const __bf16 *)x_perm, offsets, c.n_experts, c.d_ff,
                               w_base, w_stride, slot_by_rank ? 1 : 0, n_slots, table, partial, n_rows, src_row);
        PG_HIP(ctx, hipGetLastError());
        if (tslot >= 0) PG_HIP(ctx, hipEventRecord(ctx->tim_end[tslot], s));
        if (keep_partials) {
            *keep_partials = p.n_partial;
            return PGMOE_OK;
        }
        const size_t total4 = (size_t)n_rows * c.d_model / 4;
        hipLaunchKernelGGL(ffn_reduce_kernel<16>, dim3((unsigned)((total4 + 15) / 16)), dim3(256), 0, s, partial, p.n_partial, n_rows,
                           c.d_model, (__bf16 *)y_perm);
        PG_HIP(ctx, hipGetLastError());
        return PGMOE_OK;
    }
    if (c.d_ff % (16 * p.nw)) return fail(ctx, PGMOE_EINVAL, "pgmoe_expert_ffn: d_ff=%d is not a multiple of the %d-column sub-slab", c.d_ff, 16 * p.nw);
#define PG_CASE(MT_, KT_, NW_, D_) \
    if (p.mt == MT_ && kt == KT_ && p.nw == NW_) return launch_fused<MT_, KT_, NW_, D_>(ctx, p, w_base, w_stride, slot_by_rank, n_slots, x_perm, offsets, n_rows, y_perm, workspace, s, keep_partials, table, src_row)
    PG_CASE(1, 2, 4, 4); PG_CASE(1, 4, 4, 8); PG_CASE(1, 8, 4, 16); PG_CASE(1, 16, 4, 16); PG_CASE(1, 24, 4, 16);
    PG_CASE(1, 32, 4, 16); PG_CASE(1, 64, 4, 16); PG_CASE(1, 24, 2, 24); PG_CASE(1, 32, 2, 24);
    PG_CASE(2, 2, 4, 4); PG_CASE(2, 4, 4, 8); PG_CASE(2, 8, 4, 16); PG_CASE(2, 16, 4, 16); PG_CASE(2, 24, 4, 16);
    PG_CASE(2, 32, 4, 16);
    PG_CASE(4, 2, 4, 4); PG_CASE(4, 4, 4, 8); PG_CASE(4, 8, 4, 16); PG_CASE(4, 16, 4, 16); PG_CASE(4, 24, 4, 16);
    PG_CASE(4, 24, 8, 8); PG_CASE(4, 32, 8, 8);
#undef PG_CASE
    return fail(ctx, PGMOE_EINVAL, "pgmoe_expert_ffn: no bf16 kernel built for d_model=%d with %d-row chunks and %d wavefronts", c.d_model, 16 * p.mt, p.nw);
}

}  // namespace pgmoe
