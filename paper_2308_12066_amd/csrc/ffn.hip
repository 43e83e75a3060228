// Expert execution (Sec. II-B: every activated expert, a dense FFN, processes the tokens
// routed to it):  y_perm[rows of e] = ReLU(x_perm[rows of e] . W1_e) . W2_e.
//
// bf16 path - three kernels, picked from the shape of the launch alone (plan_ffn and friends):
//   ffn_fused_kernel   the general, HBM-bound case (described next);
//   ffn_decode_kernel  a handful of active experts with <= 16 rows each (batch-1 decode);
//   ffn_gemm_pack_rows_kernel + ffn_gemm_tile_kernel (twice)  hundreds of rows per expert: two tiled GEMMs (ffn_gemm.hip).
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
#include <mutex>

#include "ffn_common.h"
#include "gate_small.h"

namespace pgmoe {

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

// The pre-gate a decode-sized launch carries (FusedGate with the types the kernel needs).
struct DecodeGate {
    const __bf16 *x, *w;
    const float *bias;
    int T, k, E;
    int32_t *idx;
    float *prob;
    uint32_t *flags;
    int32_t *row_of, *offsets, *src_row;
};

// Decode-sized variant (at most a few experts active, <= 16 rows each): one workgroup of four
// wavefronts per (chunk, 32-column sub-slab of d_ff), every weight tile it needs requested before
// anything else happens, so the kernel is one round of memory latency deep instead of a ring of
// dependent rounds.  Phase A splits the d_model reduction over wavefront pairs (wave = n-tile
// + 2 * k-half; the two halves are added in LDS, k-half 0 first), phase B gives each wavefront a
// quarter of the output columns.  Always writes float32 partials (one per sub-slab).
// The chunk's rows of x are fetched after the weights have been requested, through the row ->
// token map: asking for the map at kernel start and for x ahead of the weights, or right behind
// them, was measured 0.5 and 0.3 us slower per launch (same box, alternating builds): whatever
// delays the first weight request costs more than the late x saves.
template <int KT>
__global__ __launch_bounds__(256) void ffn_decode_kernel(
    const __bf16 *__restrict__ x_perm, const int32_t *__restrict__ offsets, int E, int f,
    const char *__restrict__ w_base, size_t w_stride, int slot_by_rank, int n_slots,
    const unsigned long long *__restrict__ table, float *__restrict__ partial, int n_rows,
    const int32_t *__restrict__ src_row,  // nullable: grouped row r is row src_row[r] of x_perm
    DecodeGate gate) {            // gate.x != nullptr: workgroup (0, gridDim.y - 1) runs that gate instead of a sub-slab
    constexpr int d = KT * 32;
    if (gate.x != nullptr && blockIdx.y == gridDim.y - 1) {  // uniform over the workgroup
        if (blockIdx.x == 0)
            gate_small_dispatch(gate.E, gate.x, gate.w, gate.bias, gate.T, d, gate.k, gate.idx, gate.prob, nullptr, gate.flags,
                                gate.row_of, gate.offsets, gate.src_row);
        return;
    }
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
    if (mt == 4 && (kt == 24 || kt == 32) && c.d_ff % 128 == 0) nw = 8;
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
    if (n_rows > 4096 && p.n_partial > 16) {  // what ffn_workspace_bytes sets aside for launches this large
        p.n_partial = 16;
        while (nsub % p.n_partial) --p.n_partial;
    }
    p.f_range = c.d_ff / p.n_partial;
    return p;
}

// Instantiations of ffn_fused_kernel that are built: X(MT, KT, NW, D) = 16*MT rows per chunk,
// d_model = 32*KT, NW wavefronts, prefetch ring of D tiles.  plan_ffn only ever picks from this
// list for a d_model that appears in it (pgmoe_create refuses any other d_model for bf16).
#define PG_FUSED_CASES(X)                                                                                   \
    X(1, 2, 4, 4) X(1, 4, 4, 8) X(1, 8, 4, 16) X(1, 16, 4, 16) X(1, 24, 4, 16) X(1, 32, 4, 16) X(1, 64, 4, 16) \
    X(1, 24, 2, 24) X(1, 32, 2, 24)                                                                         \
    X(2, 2, 4, 4) X(2, 4, 4, 8) X(2, 8, 4, 16) X(2, 16, 4, 16) X(2, 24, 4, 16) X(2, 32, 4, 16)              \
    X(4, 2, 4, 4) X(4, 4, 4, 8) X(4, 8, 4, 16) X(4, 16, 4, 16) X(4, 24, 4, 16) X(4, 24, 8, 8) X(4, 32, 8, 8)

static bool fused_case_built(int mt, int kt, int nw) {
#define X(MT_, KT_, NW_, D_) \
    if (mt == MT_ && kt == KT_ && nw == NW_) return true;
    PG_FUSED_CASES(X)
#undef X
    return false;
}

// Every d_model of the list has the 16-row, four-wavefront instantiation; what else plan_ffn may
// pick for it is in the list too (checked shape by shape by the host-side tests).
bool ffn_supports_d_model(int d_model) { return d_model % 32 == 0 && fused_case_built(1, d_model / 32, 4); }

// The decode-sized kernel serves launches of 16-row chunks split into one partial per
// 32-column sub-slab (what plan_ffn picks when only a few experts are active).
static bool uses_decode_kernel(const pgmoe_config &c, const FfnPlan &p) {
    const int kt = c.d_model / 32;
    return p.mt == 1 && p.nw == 2 && p.n_partial == c.d_ff / 32 && (kt == 24 || kt == 32);
}

const char *ffn_kernel_name(const pgmoe_config &c, int n_rows) {
    if (c.dtype == PGMOE_F32) return "ffn_f32_hidden_kernel+ffn_f32_out_kernel";
    if (uses_gemm_kernels(c, n_rows)) return "ffn_gemm_pack_rows_kernel+ffn_gemm_tile_kernel";
    const FfnPlan p = plan_ffn(c, n_rows);
    if (uses_decode_kernel(c, p)) return "ffn_decode_kernel";
    return fused_case_built(p.mt, c.d_model / 32, p.nw) && c.d_ff % (16 * p.nw) == 0 ? "ffn_fused_kernel" : nullptr;
}

size_t ffn_workspace_bytes(const pgmoe_config &c) {
    const int64_t max_rows = (int64_t)c.max_tokens * c.top_k;
    if (c.dtype == PGMOE_F32) return (size_t)max_rows * c.d_ff * 4;
    // worst case over every geometry plan_ffn can pick: one partial per 32-column sub-slab
    const size_t worst = (size_t)(c.d_ff / 32) * std::min<int64_t>(max_rows, 4096) * c.d_model * 4;
    const size_t big = (size_t)16 * max_rows * c.d_model * 4;
    const size_t gemm = ffn_gemm_workspace_bytes(c);  // two-GEMM path
    return ((std::max(std::max(worst, big), gemm) + 255) & ~(size_t)255);
}

// Workspace bytes the launch of n_rows rows uses (what launch_ffn below writes and reads).
size_t ffn_launch_workspace_bytes(const pgmoe_config &c, int n_rows) {
    if (n_rows <= 0) return 0;
    if (c.dtype == PGMOE_F32) return (size_t)n_rows * c.d_ff * 4;
    if (uses_gemm_kernels(c, n_rows)) return ffn_gemm_launch_bytes(c, n_rows);
    const FfnPlan p = plan_ffn(c, n_rows);
    if (uses_decode_kernel(c, p) || p.n_partial > 1) return (size_t)p.n_partial * n_rows * c.d_model * 4;
    return 0;
}

// Scratch of pgmoe_expert_ffn_static(): part of the library's device image, so no call ever
// allocates it; every GPU the library runs on holds its own copy at its own address.  In host
// code the array's name is only a handle for hipGetSymbolAddress: the address kernels and
// copies take is resolved once per device, here, and kept.
static __device__ __align__(256) unsigned char scratch[PGMOE_STATIC_SCRATCH_BYTES];
static void *g_scratch_ptr[64] = {};
static std::mutex g_scratch_mutex;  // contexts may be created from several host threads

int resolve_static_scratch(pgmoe_ctx *ctx) {  // the context's device is current (pgmoe_create)
    const int dev = ctx->device;
    if (dev < 0 || dev >= (int)(sizeof g_scratch_ptr / sizeof g_scratch_ptr[0]))
        return fail(ctx, PGMOE_EINVAL, "pgmoe_create: device ordinal %d outside 0..63", dev);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        PG_HIP(ctx, hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr || !aligned(ptr, 256)) return fail(ctx, PGMOE_EHIP, "pgmoe_create: the static scratch buffer resolved to %p", ptr);
        g_scratch_ptr[dev] = ptr;
    }
    ctx->static_scratch = g_scratch_ptr[dev];
    return PGMOE_OK;
}

int ffn_timing_slot(pgmoe_ctx *ctx) {
    if (!ctx->tim_on || ctx->tim_n >= ctx->tim_cap) return -1;
    return ctx->tim_n++;
}

int launch_ffn_reduce(pgmoe_ctx *ctx, const float *partial, int P, int n_rows, void *y_perm, hipStream_t s) {
    const int d = ctx->cfg.d_model;
    const size_t total4 = (size_t)n_rows * d / 4;
    const int pl = reduce_lanes(P);  // p-lanes per column: 256 / pl float4 columns per workgroup
    const dim3 grid((unsigned)((total4 + 256 / pl - 1) / (256 / pl)));
    if (pl == 1) hipLaunchKernelGGL(ffn_reduce_kernel<1>, grid, dim3(256), 0, s, partial, P, n_rows, d, (__bf16 *)y_perm);
    else if (pl == 4) hipLaunchKernelGGL(ffn_reduce_kernel<4>, grid, dim3(256), 0, s, partial, P, n_rows, d, (__bf16 *)y_perm);
    else hipLaunchKernelGGL(ffn_reduce_kernel<16>, grid, dim3(256), 0, s, partial, P, n_rows, d, (__bf16 *)y_perm);
    PG_HIP(ctx, hipGetLastError());
    return PGMOE_OK;
}

template <int MT, int KT, int NW, int D>
static int launch_fused(pgmoe_ctx *ctx, const FfnPlan &p, const char *w_base, size_t w_stride, bool slot_by_rank, int n_slots,
                        const void *x_perm, const int32_t *offsets, int n_rows, void *y_perm, void *workspace,
                        hipStream_t s, int *keep_partials, const unsigned long long *table, const int32_t *src_row) {
    const pgmoe_config &c = ctx->cfg;
    const size_t lds = (size_t)MT * KT * 1024 + 2u * MT * (16 * NW / 32) * 1024;
    auto kern = ffn_fused_kernel<MT, KT, NW, D>;
    if (int rc = allow_dynamic_lds(ctx, reinterpret_cast<const void *>(kern), lds)) return rc;
    float *partial = p.n_partial > 1 ? (float *)workspace : nullptr;
    if (partial && (size_t)p.n_partial * n_rows * c.d_model * 4 > ffn_workspace_bytes(c))
        return fail(ctx, PGMOE_EINVAL, "pgmoe_expert_ffn: %d partial sums of %d rows do not fit the workspace", p.n_partial, n_rows);
    const int tslot = ffn_timing_slot(ctx);
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
    if (partial) return launch_ffn_reduce(ctx, partial, p.n_partial, n_rows, y_perm, s);
    return PGMOE_OK;
}

int launch_ffn(pgmoe_ctx *ctx, const char *w_base, size_t w_stride, bool slot_by_rank, int n_slots, const void *x_perm,
               const int32_t *offsets, int n_rows, void *y_perm, void *workspace, hipStream_t s, int *keep_partials,
               const unsigned long long *table, const int32_t *src_row, const FusedGate *gate, bool *gate_done) {
    const pgmoe_config &c = ctx->cfg;
    if (keep_partials) *keep_partials = 0;
    if (gate_done) *gate_done = false;
    if (n_rows == 0) return PGMOE_OK;
    if (c.dtype == PGMOE_F32) {
        float *h = (float *)workspace;
        const int tslot = ffn_timing_slot(ctx);
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
    if (uses_gemm_kernels(c, n_rows))
        return launch_ffn_gemm(ctx, w_base, w_stride, slot_by_rank, n_slots, x_perm, offsets, n_rows, y_perm, workspace, s,
                               keep_partials, table, src_row);
    const FfnPlan p = plan_ffn(c, n_rows);
    const int kt = c.d_model / 32;
    if (uses_decode_kernel(c, p)) {
        // a few experts with at most 16 rows each, one partial per 32-column sub-slab
        float *partial = (float *)workspace;
        if ((size_t)p.n_partial * n_rows * c.d_model * 4 > ffn_workspace_bytes(c))
            return fail(ctx, PGMOE_EINVAL, "pgmoe_expert_ffn: %d partial sums of %d rows do not fit the workspace", p.n_partial, n_rows);
        const int tslot = ffn_timing_slot(ctx);
        if (tslot >= 0) PG_HIP(ctx, hipEventRecord(ctx->tim_begin[tslot], s));
        // one more row of workgroups for the pre-gate this launch carries, if it is one the smallest-gate code serves
        DecodeGate dg = {};
        if (gate && gate_done && gate_small_applies(c, gate->T)) {
            dg = DecodeGate{(const __bf16 *)gate->x, (const __bf16 *)gate->w, gate->bias, gate->T, c.top_k, c.n_experts, gate->idx,
                            gate->prob, ctx->dev_flags, gate->row_of, gate->offsets, gate->src_row};
            *gate_done = true;
        }
        const dim3 grid(p.max_chunks, p.n_partial + (dg.x ? 1 : 0));
        const size_t lds = (size_t)kt * 1024 + 4096;
        if (kt == 24)
            hipLaunchKernelGGL(ffn_decode_kernel<24>, grid, dim3(256), lds, s, (const __bf16 *)x_perm, offsets, c.n_experts, c.d_ff,
                               w_base, w_stride, slot_by_rank ? 1 : 0, n_slots, table, partial, n_rows, src_row, dg);
        else
            hipLaunchKernelGGL(ffn_decode_kernel<32>, grid, dim3(256), lds, s, (const __bf16 *)x_perm, offsets, c.n_experts, c.d_ff,
                               w_base, w_stride, slot_by_rank ? 1 : 0, n_slots, table, partial, n_rows, src_row, dg);
        PG_HIP(ctx, hipGetLastError());
        if (tslot >= 0) PG_HIP(ctx, hipEventRecord(ctx->tim_end[tslot], s));
        if (keep_partials) {
            *keep_partials = p.n_partial;
            return PGMOE_OK;
        }
        return launch_ffn_reduce(ctx, partial, p.n_partial, n_rows, y_perm, s);
    }
    if (c.d_ff % (16 * p.nw)) return fail(ctx, PGMOE_EINVAL, "pgmoe_expert_ffn: d_ff=%d is not a multiple of the %d-column sub-slab", c.d_ff, 16 * p.nw);
#define X(MT_, KT_, NW_, D_)                                                                                                  \
    if (p.mt == MT_ && kt == KT_ && p.nw == NW_)                                                                              \
        return launch_fused<MT_, KT_, NW_, D_>(ctx, p, w_base, w_stride, slot_by_rank, n_slots, x_perm, offsets, n_rows, y_perm, \
                                               workspace, s, keep_partials, table, src_row);
    PG_FUSED_CASES(X)
#undef X
    return fail(ctx, PGMOE_EINVAL, "pgmoe_expert_ffn: no bf16 kernel built for d_model=%d with %d-row chunks and %d wavefronts", c.d_model, 16 * p.mt, p.nw);
}

}  // namespace pgmoe
