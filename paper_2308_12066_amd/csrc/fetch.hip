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
// 24 workgroups x 4 wavefronts x one 1 KiB load each (96 KiB: 56.3 of 57 GB/s).  The slowdown is
// not confined to the XCD the loads come from: with all 24 workgroups placed on one XCD the
// concurrent FFN is slower still (14.6 instead of 11.6 us) and so is the link (50 instead of 52 GB/s).
#include "pgmoe_internal.h"

namespace pgmoe {

constexpr int FETCH_THREADS = 256;
constexpr int FETCH_GRID = 24;
constexpr int FETCH_UNROLL = 1;

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// Turn-taking on the host link.  Consecutive migrations of a stack step run on two alternating
// streams, so that the next one is already resident when the current one ends and the link never
// idles at the hand-over; left alone, the two kernels would share the link while they overlap,
// which delays the EARLIER one: its block starts later, the pre-gate behind that block issues
// the fetch after next later, and the link idles there instead (17-23 us per pair of blocks on
// the Switch-Base-8 decode stack).  So the kernels of a step take turns: kernel number seq does
// its planning at once but starts copying only when turn[0] (how many of this step's migrations
// have passed the turn on) has reached seq.  This orders link traffic only, no data depends on
// it: the wait is bounded by the clock (half a second) and a kernel that gives up just copies
// alongside its predecessor as before.  The turn passes on as soon as the FIRST workgroup of a
// kernel is done (all have the same amount to copy, so the others are within their last loads:
// the successor's first loads fill the link while those drain); only the step's last kernel
// counts its workgroups (turn[1]) and its last one sets the turn back to 0, so that a captured
// step replays with the same arguments; the step's first kernel clears it as well, which limits
// what a late straggler of the previous step (or a step that ended early) can leave behind to one
// pair of kernels copying side by side.
constexpr unsigned long long TURN_TIMEOUT_TICKS = 50000000ull;  // of the 100 MHz wall clock: the bound inside a stack step

__device__ inline void wait_for_turn(uint32_t *turn, int seq, unsigned long long timeout_ticks) {
    if (seq == 0 && blockIdx.x == 0 && threadIdx.x == 0) __hip_atomic_store(turn, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (seq <= 0) return;  // uniform over the kernel
    if (threadIdx.x == 0) {
        const unsigned long long t0 = wall_clock64();
        while (__hip_atomic_load(turn, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < (uint32_t)seq &&
               wall_clock64() - t0 < timeout_ticks)
            __builtin_amdgcn_s_sleep(32);
    }
    __syncthreads();
}

__device__ inline void end_of_turn(uint32_t *turn, int seq, int last) {
    if (seq < 0) return;  // uniform over the kernel
    __syncthreads();      // every load of this workgroup has returned (its value went into a store)
    if (threadIdx.x == 0) {
        if (!last) {
            atomicMax(turn, (uint32_t)seq + 1u);
        } else if (atomicAdd(turn + 1, 1u) == gridDim.x - 1) {
            __hip_atomic_store(turn + 1, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(turn, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

// With tracing on, a migration kernel leaves the 100 MHz clock of the moment it starts copying
// (first workgroup, after its wait for the turn) in clk[0] and of the moment its last workgroup
// has its last load back in clk[1] (a maximum: the clock only grows, so an earlier migration's
// value never wins): the copy itself, without the wait that the kernel's duration includes.
__device__ inline void copy_clock_begin(unsigned long long *clk) {
    if (clk && blockIdx.x == 0 && threadIdx.x == 0) __hip_atomic_store(clk, wall_clock64(), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline void copy_clock_end(unsigned long long *clk) {
    if (!clk) return;  // uniform over the kernel
    __syncthreads();   // every load of this workgroup has returned (its value went into a store)
    if (threadIdx.x == 0) atomicMax(clk + 1, wall_clock64());
}

template <typename V>
__global__ __launch_bounds__(FETCH_THREADS) void fetch_pull_kernel(
    const int32_t *__restrict__ idx, int n, int E, const char *__restrict__ src_block, size_t expert_stride,
    char *__restrict__ gen_base, size_t expert_bytes, int slots, int all, int32_t *__restrict__ unique_out,
    uint32_t *flags, uint32_t *turn, int seq, int last, unsigned long long turn_timeout, unsigned long long *clk) {
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
    wait_for_turn(turn, seq, turn_timeout);
    copy_clock_begin(clk);

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
    copy_clock_end(clk);
    end_of_turn(turn, seq, last);
}

// ------------------------------------------------------------------------------------------
// Pull with an expert cache (the paper evaluates LIFO, LFU and LRU caches on top of the
// migration; Sec. VI, "Caching experts").  Per block the device keeps, in two alternating
// copies, which expert each cache slot holds and the bookkeeping the policy needs.  Every
// workgroup reads the same (old) copy and derives the same plan in its first wavefront, one
// lane per cache slot: selected experts that are cached are hits; each missing expert, in
// ascending order, replaces the policy's victim among the slots not used by this fetch (empty
// slots first) and is copied straight into that cache slot, or goes to the generation's slots
// when no victim is left.  Workgroup 0 writes the new copy of the state, the per-expert pointer
// table the FFN reads, and the counters.
constexpr int CACHE_STATE_INTS = 4 * PGMOE_MAX_CACHE_SLOTS + 4;  // cexp, cuse, ccnt, cins, then tick, ins_seq

__device__ inline void wave_argmin_u64(unsigned long long &key, int &lane_id) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const unsigned long long ok = __shfl_xor(key, off);
        const int ol = __shfl_xor(lane_id, off);
        if (ok < key || (ok == key && ol < lane_id)) {
            key = ok;
            lane_id = ol;
        }
    }
}

template <typename V>
__global__ __launch_bounds__(FETCH_THREADS) void fetch_pull_cache_kernel(
    const int32_t *__restrict__ idx, int n, int E, const char *__restrict__ src_block, size_t expert_stride,
    char *__restrict__ gen_base, size_t expert_bytes, int slots, char *__restrict__ cache_base, int C, int policy,
    const int32_t *__restrict__ state_in, int32_t *__restrict__ state_out, unsigned long long *__restrict__ table,
    int32_t *__restrict__ stats_out, uint32_t *flags, uint32_t *turn, int seq, int last, unsigned long long turn_timeout,
    unsigned long long *clk) {
    __shared__ int present[PGMOE_MAX_EXPERTS];               // 0 not selected, 1 selected
    __shared__ int cp_src[PGMOE_MAX_EXPERTS];                // copies: source expert
    __shared__ unsigned long long cp_dst[PGMOE_MAX_EXPERTS]; // copies: destination address
    __shared__ unsigned long long tbl[PGMOE_MAX_EXPERTS];    // address of every selected expert
    __shared__ int s_counts[4];                              // copies, unique, hits, overflow
    const int tid = threadIdx.x, lane = tid & 63;
    for (int e = tid; e < PGMOE_MAX_EXPERTS; e += FETCH_THREADS) {
        present[e] = 0;
        tbl[e] = 0ull;
    }
    __syncthreads();
    bool bad = false;
    for (int i = tid; i < n; i += FETCH_THREADS) {
        const int e = idx[i];
        if (e >= 0 && e < E) present[e] = 1;
        else bad = true;
    }
    if (__any(bad) && lane == 0 && blockIdx.x == 0) atomicOr(flags, kFlagBadIndex);
    __syncthreads();

    if (tid < 64) {  // wavefront 0 plans; lane = cache slot
        const bool slot = lane < C;
        int cexp = slot ? state_in[lane] : -1;
        int cuse = slot ? state_in[PGMOE_MAX_CACHE_SLOTS + lane] : 0;
        int ccnt = slot ? state_in[2 * PGMOE_MAX_CACHE_SLOTS + lane] : 0;
        int cins = slot ? state_in[3 * PGMOE_MAX_CACHE_SLOTS + lane] : 0;
        const int tick = state_in[4 * PGMOE_MAX_CACHE_SLOTS] + 1;
        int ins_seq = state_in[4 * PGMOE_MAX_CACHE_SLOTS + 1];
        bool pinned = false;
        if (slot && cexp >= 0 && present[cexp] == 1) {  // hit: distinct lanes hold distinct experts
            pinned = true;
            tbl[cexp] = (unsigned long long)(cache_base + (size_t)lane * expert_bytes);
            present[cexp] = 2;
            cuse = tick;
            ccnt += 1;
        }
        const int hits = __popcll(__ballot(pinned));
        int n_copy = 0, n_gen = 0, uniq = hits, overflow = 0;
        for (int e = 0; e < E; ++e) {
            if (present[e] != 1) continue;  // LDS value is uniform over the wavefront
            ++uniq;
            unsigned long long key = ~0ull;
            if (slot && !pinned) {
                if (cexp < 0) key = 0ull;  // empty slots first
                else if (policy == PGMOE_CACHE_LRU) key = 1ull + (unsigned)cuse;
                else if (policy == PGMOE_CACHE_LFU) key = 1ull + (((unsigned long long)(unsigned)ccnt << 32) | (unsigned)cuse);
                else key = 1ull + (0xffffffffull - (unsigned)cins);  // LIFO: most recently inserted first
            }
            int v = lane;
            wave_argmin_u64(key, v);
            unsigned long long dst = 0ull;
            if (key != ~0ull) {
                if (lane == v) {
                    cexp = e;
                    cuse = tick;
                    ccnt = 1;
                    cins = ins_seq + 1;
                    pinned = true;
                }
                ++ins_seq;
                dst = (unsigned long long)(cache_base + (size_t)v * expert_bytes);
            } else if (n_gen < slots) {
                dst = (unsigned long long)(gen_base + (size_t)n_gen * expert_bytes);
                ++n_gen;
            } else {
                overflow = 1;  // nowhere to put it: the FFN zeroes its rows (table entry stays 0)
            }
            if (lane == 0) {
                tbl[e] = dst;
                if (dst) {
                    cp_src[n_copy] = e;
                    cp_dst[n_copy] = dst;
                }
            }
            if (dst) ++n_copy;
        }
        if (lane == 0) {
            s_counts[0] = n_copy;
            s_counts[1] = uniq;
            s_counts[2] = hits;
            s_counts[3] = overflow;
        }
        if (blockIdx.x == 0) {
            if (slot) {
                state_out[lane] = cexp;
                state_out[PGMOE_MAX_CACHE_SLOTS + lane] = cuse;
                state_out[2 * PGMOE_MAX_CACHE_SLOTS + lane] = ccnt;
                state_out[3 * PGMOE_MAX_CACHE_SLOTS + lane] = cins;
            }
            if (lane == 0) {
                state_out[4 * PGMOE_MAX_CACHE_SLOTS] = tick;
                state_out[4 * PGMOE_MAX_CACHE_SLOTS + 1] = ins_seq;
                stats_out[0] = uniq;
                stats_out[1] = n_copy;
                stats_out[2] = hits;
                if (overflow) atomicOr(flags, kFlagNoSlot);
            }
        }
    }
    __syncthreads();
    if (blockIdx.x == 0)
        for (int e = tid; e < E; e += FETCH_THREADS) table[e] = tbl[e];
    wait_for_turn(turn, seq, turn_timeout);
    copy_clock_begin(clk);

    const unsigned upe = (unsigned)(expert_bytes / sizeof(V));
    const unsigned total = (unsigned)s_counts[0] * upe;
    const unsigned stride = gridDim.x * FETCH_THREADS;
    for (unsigned i = blockIdx.x * FETCH_THREADS + tid; i < total; i += stride) {
        const unsigned j = i / upe, of = i - j * upe;
        reinterpret_cast<V *>(cp_dst[j])[of] =
            __builtin_nontemporal_load(reinterpret_cast<const V *>(src_block + (size_t)cp_src[j] * expert_stride) + of);
    }
    copy_clock_end(clk);
    end_of_turn(turn, seq, last);
}

size_t cache_state_bytes(const pgmoe_config &c) { return (size_t)c.n_blocks * 2 * CACHE_STATE_INTS * sizeof(int32_t); }

int launch_fetch_pull(pgmoe_ctx *ctx, int block, bool all, const int32_t *idx, int n, hipStream_t s, int seq, bool last,
                      unsigned long long turn_timeout_ticks) {
    const int gen = block % ctx->n_gen;
    const unsigned long long tmo = turn_timeout_ticks ? turn_timeout_ticks : TURN_TIMEOUT_TICKS;
    unsigned long long *clk = ctx->trace ? ctx->dev_copy_clock + 2 * (size_t)block : nullptr;
    uint32_t *turn = ctx->dev_flags + 4;  // two counters in the flag block's first 64 bytes
    const int is_last = last ? 1 : 0;
    char *gen_base = ctx->slot_pool + (size_t)gen * ctx->slots * ctx->expert_bytes;
    const char *src = ctx->store_dev + (size_t)block * ctx->block_stride;
    if (ctx->cfg.cache_slots > 0 && !all) {
        const int C = ctx->cfg.cache_slots, par = ctx->cache_parity[block];
        char *cache_base = ctx->cache_pool + (size_t)block * C * ctx->expert_bytes;
        const int32_t *st_in = ctx->cache_state + ((size_t)block * 2 + par) * CACHE_STATE_INTS;
        int32_t *st_out = ctx->cache_state + ((size_t)block * 2 + (par ^ 1)) * CACHE_STATE_INTS;
        unsigned long long *table = ctx->dev_table + (size_t)block * PGMOE_MAX_EXPERTS;
        int32_t *stats = ctx->cache_stats + (size_t)block * 4;
        if (ctx->expert_bytes % 16 == 0)
            hipLaunchKernelGGL(fetch_pull_cache_kernel<u32x4>, dim3(FETCH_GRID), dim3(FETCH_THREADS), 0, s, idx, n,
                               ctx->cfg.n_experts, src, ctx->expert_stride, gen_base, ctx->expert_bytes, ctx->slots, cache_base,
                               C, ctx->cfg.cache_policy, st_in, st_out, table, stats, ctx->dev_flags, turn, seq, is_last, tmo, clk);
        else
            hipLaunchKernelGGL(fetch_pull_cache_kernel<unsigned int>, dim3(FETCH_GRID), dim3(FETCH_THREADS), 0, s, idx, n,
                               ctx->cfg.n_experts, src, ctx->expert_stride, gen_base, ctx->expert_bytes, ctx->slots, cache_base,
                               C, ctx->cfg.cache_policy, st_in, st_out, table, stats, ctx->dev_flags, turn, seq, is_last, tmo, clk);
        PG_HIP(ctx, hipGetLastError());
        ctx->cache_parity[block] = par ^ 1;
        return PGMOE_OK;
    }
    if (ctx->expert_bytes % 16 == 0)
        hipLaunchKernelGGL(fetch_pull_kernel<u32x4>, dim3(FETCH_GRID), dim3(FETCH_THREADS), 0, s, idx, n, ctx->cfg.n_experts,
                           src, ctx->expert_stride, gen_base, ctx->expert_bytes, ctx->slots, all ? 1 : 0, ctx->dev_unique + block,
                           ctx->dev_flags, turn, seq, is_last, tmo, clk);
    else
        hipLaunchKernelGGL(fetch_pull_kernel<unsigned int>, dim3(FETCH_GRID), dim3(FETCH_THREADS), 0, s, idx, n,
                           ctx->cfg.n_experts, src, ctx->expert_stride, gen_base, ctx->expert_bytes, ctx->slots, all ? 1 : 0,
                           ctx->dev_unique + block, ctx->dev_flags, turn, seq, is_last, tmo, clk);
    PG_HIP(ctx, hipGetLastError());
    return PGMOE_OK;
}

}  // namespace pgmoe
