// Internal declarations shared by the translation units of libpgmoe (not installed).
#pragma once

#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <cstring>

#include "pgmoe.h"

namespace pgmoe {

enum StoreMode { STORE_NONE = 0, STORE_HOST = 1, STORE_RESIDENT = 2 };

constexpr int kGen = PGMOE_MAX_PREGATE_DISTANCE + 1;  // most block generations resident at once
constexpr int kSpareStreams = 6;  // most replacements of the context's own copy stream (pgmoe_check_streams)

// Device-side sticky condition bits (see pgmoe_device_flags).
constexpr uint32_t kFlagNaN = 1u;
constexpr uint32_t kFlagBadIndex = 2u;
constexpr uint32_t kFlagNoSlot = 4u;

// Rows of one expert that a single FFN workgroup handles at once (bf16 path): 16 * MT.
constexpr int kTileRows = 16;

struct BlockStats {
    pgmoe_fetch_stats s;
    bool timed;   // fetch_begin/fetch_end were recorded for this block
    bool pulled;  // fetched by the pull kernel: counts live on the device
    bool cached;  // ... through the expert cache: counts in cache_stats
    bool in_line; // the fetch ran on the compute stream itself: the stream stood still for all of it
};

}  // namespace pgmoe

struct pgmoe_ctx {
    pgmoe_config cfg;
    bool host_only;
    int device;
    size_t elem;          // bytes per activation / weight element
    size_t expert_bytes;  // 2*d*f*elem
    int slots;            // slots per generation
    int distance;         // pre-gate distance N (>= 1)
    int n_gen;            // N + 1 block generations: block b lives in generation b % n_gen

    // expert store
    int store_mode;
    const char *store_base;
    size_t expert_stride, block_stride;

    // device resources
    char *slot_pool;       // [n_gen][slots][expert_bytes]
    uint32_t *dev_flags;   // [0] sticky condition bits; [4], [5] turn counters of the migration kernels (fetch.hip)
    int32_t *dev_unique;   // [n_blocks] distinct experts found by the pull kernel (dev_flags + 64 bytes)
    unsigned long long *dev_copy_clock;  // [n_blocks][2] copy start / end of the block's last traced pull kernel (100 MHz ticks)
    int32_t *dev_src_row;  // [n_blocks][max_tokens * k] grouped row -> token, written by each block's routing
    bool *routed;          // [n_blocks] host: this step's gate kernel already grouped the block's tokens
    // turn-taking of a stack step's migration kernels on the host link (see fetch.hip): position of
    // the next one in the step (-1: not inside a step), and the position of the step's last one
    int pull_seq = -1, pull_last = -1;
    unsigned long long turn_timeout_ticks = 0;  // bound of the wait for the turn (0 = default); set by the test hook only
    // set by pgmoe_stack_step around one fetch: the routing was computed on the copy stream the
    // fetch will use (stream order covers it), so no event from the compute stream is needed
    bool routed_on_copy_stream = false;
    hipEvent_t step_start = nullptr;  // compute stream -> the context's own copy stream at the start of a step
    const char *store_dev; // device-visible address of the pinned host store
    bool pull;             // fetch with the device-side pull kernel
    int32_t *idx_staging;  // pinned host [max_tokens * k]
    hipEvent_t idx_ready;
    hipEvent_t fetch_done[pgmoe::kGen];
    hipEvent_t ffn_done[pgmoe::kGen];
    hipEvent_t fork[pgmoe::kGen], join[pgmoe::kGen];  // memcpy mode: a block's copies go out on two streams
    hipEvent_t *fetch_begin;  // [n_blocks] timing
    hipEvent_t *fetch_end;    // [n_blocks]
    int fetched_block[pgmoe::kGen];  // block whose experts the generation holds (-1: none)
    int live_slots[pgmoe::kGen];
    bool ffn_recorded[pgmoe::kGen];
    hipStream_t ffn_stream[pgmoe::kGen];    // stream the generation's last FFN ran on
    hipStream_t fetch_stream[pgmoe::kGen];  // stream the generation's last fetch ran on
    hipStream_t copy2;                      // internal second copy stream
    hipStream_t spare_streams[pgmoe::kSpareStreams] = {};  // earlier ones that shared a hardware queue with a caller's stream
    bool gen_all[pgmoe::kGen];              // generation holds every expert of its block (slot = expert id)
    bool gen_table[pgmoe::kGen];            // generation was filled through the expert cache: FFN reads dev_table

    // expert cache (cfg.cache_slots > 0)
    char *cache_pool;                 // [n_blocks][cache_slots][expert_bytes]
    int32_t *cache_state;             // [n_blocks][2][state] device
    unsigned long long *dev_table;    // [n_blocks][PGMOE_MAX_EXPERTS] device address of every selected expert
    int32_t *cache_stats;             // [n_blocks][4] device: unique, copies, hits
    unsigned char *cache_parity;      // [n_blocks] host: which state copy is current
    int schedule;                           // PGMOE_SCHED_*
    float standin_us;                       // non-MoE stand-in per block (0 = none)
    bool fetch_timing;               // record fetch_begin / fetch_end
    bool trace;                      // record the per-block compute-stream events below
    hipEvent_t *ev_c0, *ev_ready, *ev_waited, *ev_c1;  // [n_blocks] each
    bool *traced;                    // [n_blocks] events of the last step are valid
    pgmoe::BlockStats *stats;  // [n_blocks]

    // optional timing of the FFN kernel (pgmoe_ffn_timing_begin/end)
    hipEvent_t *tim_begin, *tim_end;
    int tim_cap, tim_n;
    bool tim_on;
    float tim_overhead_ms;  // what one event pair adds around a kernel

    void *static_scratch = nullptr;  // this device's copy of the library's static scratch buffer (pgmoe_expert_ffn_static)

    // kernels whose dynamic-LDS limit has been raised for this context's device (allow_dynamic_lds)
    const void *lds_ready[48] = {};
    int n_lds_ready = 0;

    char err[512];
};

namespace pgmoe {

int fail(pgmoe_ctx *ctx, int code, const char *fmt, ...) __attribute__((format(printf, 3, 4)));
int hip_fail(pgmoe_ctx *ctx, hipError_t e, const char *what);
// Validates cfg; on failure writes the reason to buf and returns PGMOE_EINVAL.
int check_config(const pgmoe_config *cfg, char *buf, size_t n);

#define PG_HIP(ctx, call)                                               \
    do {                                                                \
        hipError_t e_ = (call);                                         \
        if (e_ != hipSuccess) return ::pgmoe::hip_fail(ctx, e_, #call); \
    } while (0)

inline bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

// A launch with more than 48 KiB of dynamic LDS needs the kernel's limit raised first, once per
// kernel and device; the context remembers which of its kernels have had that done.
inline int allow_dynamic_lds(pgmoe_ctx *ctx, const void *kernel, size_t bytes) {
    if (bytes <= 48 * 1024) return PGMOE_OK;
    for (int i = 0; i < ctx->n_lds_ready; ++i)
        if (ctx->lds_ready[i] == kernel) return PGMOE_OK;
    PG_HIP(ctx, hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes));
    if (ctx->n_lds_ready < (int)(sizeof ctx->lds_ready / sizeof ctx->lds_ready[0])) ctx->lds_ready[ctx->n_lds_ready++] = kernel;
    return PGMOE_OK;
}

// Geometry of the bf16 FFN launch for n_rows permuted rows (host side, deterministic):
// rows per workgroup chunk, number of d_ff ranges (partial sums) and the chunk-count bound.
struct FfnPlan {
    int mt;          // 16-row tiles per chunk (1, 2 or 4)
    int nw;          // wavefronts per workgroup (2, 4 or 8); sub-slab = 16*nw d_ff columns
    int f_range;     // d_ff columns per workgroup (multiple of the sub-slab)
    int n_partial;   // d_ff / f_range
    int max_chunks;  // upper bound of sum_e ceil(n_e / (16*mt))
};
FfnPlan plan_ffn(const pgmoe_config &cfg, int n_rows);
size_t ffn_workspace_bytes(const pgmoe_config &cfg);
size_t ffn_launch_workspace_bytes(const pgmoe_config &cfg, int n_rows);  // what one launch of n_rows rows uses of it
// Device address of the library's static scratch buffer on the context's device (which must be
// current) into ctx->static_scratch; resolved once per device and process.
int resolve_static_scratch(pgmoe_ctx *ctx);
const char *ffn_kernel_name(const pgmoe_config &cfg, int n_rows);  // nullptr: no kernel is built for this launch
bool ffn_supports_d_model(int d_model);                          // bf16: expert kernels are built for this d_model

// Kernel launchers (each validates nothing: callers did).  All asynchronous on `s`.
// row_of / offsets / src_row / routed (all or none): if the launch can also group the tokens by
// expert (decode-sized batch, bf16 matrix-core gate), it writes what launch_route would and sets
// *routed; otherwise *routed = false and the three arrays are left alone.
int launch_gate(pgmoe_ctx *ctx, const void *x, const void *w, const float *bias, int T, int32_t *idx,
                float *prob, float *probs, hipStream_t s, int32_t *row_of = nullptr, int32_t *offsets = nullptr,
                int32_t *src_row = nullptr, bool *routed = nullptr);
int launch_permute(pgmoe_ctx *ctx, const void *x, const int32_t *idx, int T, void *x_perm,
                   int32_t *row_of, int32_t *offsets, hipStream_t s);
// The integer half of launch_permute; src_row (nullable) receives the inverse map grouped row -> token.
int launch_route(pgmoe_ctx *ctx, const int32_t *idx, int T, int32_t *row_of, int32_t *offsets, int32_t *src_row,
                 hipStream_t s);
// A pre-gate that an expert-FFN launch may carry as one extra workgroup (Sec. IV-B: the pre-gate
// of block i is evaluated on the same hidden state as block i's experts and needs nothing from
// them, so the two can run side by side in one launch).  Only decode-sized launches do it.
struct FusedGate {
    const void *x;                  // [T, d] hidden state the gate is evaluated on
    const void *w;                  // [d, E] gate weight
    const float *bias;              // [E] | nullptr
    int T;
    int32_t *idx;                   // [T, k] out
    float *prob;                    // [T, k] out
    int32_t *row_of, *offsets, *src_row;  // grouping of the routed block, out
};
// keep_partials != nullptr: if the launch produces float32 partial sums, leave them in the
// workspace unreduced and report their number there (0 = y_perm was written directly).
// gate != nullptr: carry that gate if this launch can (then *gate_done = true), else leave it to the caller.
int launch_ffn(pgmoe_ctx *ctx, const char *w_base, size_t w_stride, bool slot_by_rank, int n_slots, const void *x_perm,
               const int32_t *offsets, int n_rows, void *y_perm, void *workspace, hipStream_t s, int *keep_partials = nullptr,
               const unsigned long long *table = nullptr,  // table: per-expert weight addresses (0 = none), overrides w_base
               const int32_t *src_row = nullptr,  // bf16 only: x_perm is the un-grouped x [T,d], grouped row r reads x[src_row[r]]
               const FusedGate *gate = nullptr, bool *gate_done = nullptr);
// p-lanes of the partial-sum reduction for P partials (fixes the order of the additions)
inline int reduce_lanes(int P) { return P <= 2 ? 1 : (P <= 8 ? 4 : 16); }
// Combine straight from P unreduced float32 partials [P][n_rows][d] (bf16 contexts only): same
// arithmetic, in the same order, as ffn_reduce_kernel followed by launch_combine.
int launch_combine_partials(pgmoe_ctx *ctx, const float *partial, int P, int n_rows, const int32_t *row_of,
                            const float *prob, int T, void *y, const void *x_res, void *x_next, hipStream_t s);
// seq: position among the migration kernels of the running stack step (they take turns on the
// host link in that order), -1 for a kernel that is not part of one; last: the step's last one
// turn_timeout_ticks: bound of that wait in ticks of the 100 MHz clock (0 = the default of half a second)
int launch_fetch_pull(pgmoe_ctx *ctx, int block, bool all, const int32_t *idx, int n, hipStream_t s, int seq = -1,
                      bool last = false, unsigned long long turn_timeout_ticks = 0);
size_t cache_state_bytes(const pgmoe_config &c);
int launch_combine(pgmoe_ctx *ctx, const void *y_perm, const int32_t *row_of, const float *prob, int T,
                   void *y, const void *x_res, void *x_next, hipStream_t s);

}  // namespace pgmoe
