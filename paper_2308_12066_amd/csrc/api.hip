// libpgmoe: context, argument validation, host-side helpers and the exported entry points of
// the single operations.  Kernels live in gate.hip, permute.hip, ffn.hip, ffn_gemm.hip, combine.hip; the
// migration engine and the whole-stack step in engine.hip.
#include <algorithm>
#include <new>

#include "pgmoe_internal.h"

namespace pgmoe {

static thread_local char g_err[512] = "";

int fail(pgmoe_ctx *ctx, int code, const char *fmt, ...) {
    char *dst = ctx ? ctx->err : g_err;
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(dst, 512, fmt, ap);
    va_end(ap);
    return code;
}

int hip_fail(pgmoe_ctx *ctx, hipError_t e, const char *what) {
    return fail(ctx, PGMOE_EHIP, "%s failed: %s", what, hipGetErrorString(e));
}

static int default_slots(const pgmoe_config &c) {
    int64_t n = (int64_t)c.max_tokens * c.top_k;
    return (int)std::min<int64_t>(c.n_experts, n);
}

int check_config(const pgmoe_config *c, char *buf, size_t n) {
#define BAD(...)                    \
    do {                            \
        snprintf(buf, n, __VA_ARGS__); \
        return PGMOE_EINVAL;        \
    } while (0)
    if (!c) BAD("config is NULL");
    if (c->dtype != PGMOE_F32 && c->dtype != PGMOE_BF16) BAD("dtype %d is neither f32 nor bf16", c->dtype);
    if (c->d_model < 1 || c->d_ff < 1) BAD("d_model=%d, d_ff=%d must be >= 1", c->d_model, c->d_ff);
    if (c->d_model > 65536 || c->d_ff > 262144) BAD("d_model=%d / d_ff=%d too large", c->d_model, c->d_ff);
    if (c->dtype == PGMOE_BF16 && (c->d_model % 64 || c->d_ff % 64))
        BAD("bf16 needs d_model and d_ff to be multiples of 64 (got %d, %d)", c->d_model, c->d_ff);
    if (c->dtype == PGMOE_BF16 && c->d_model > 2048)
        BAD("bf16 path keeps a 16-row activation tile in LDS: d_model <= 2048 (got %d)", c->d_model);
    if (c->n_experts < 1 || c->n_experts > PGMOE_MAX_EXPERTS)
        BAD("n_experts=%d outside 1..%d", c->n_experts, PGMOE_MAX_EXPERTS);
    if (c->top_k < 1 || c->top_k > c->n_experts) BAD("top_k=%d outside 1..n_experts=%d", c->top_k, c->n_experts);
    if (c->n_blocks < 1 || c->n_blocks > 4096) BAD("n_blocks=%d outside 1..4096", c->n_blocks);
    if (c->max_tokens < 1 || (int64_t)c->max_tokens * c->top_k > (1 << 24))
        BAD("max_tokens=%d (x top_k=%d) outside 1..2^24", c->max_tokens, c->top_k);
    if (c->slots_per_gen < 0 || c->slots_per_gen > c->n_experts)
        BAD("slots_per_gen=%d outside 0..n_experts", c->slots_per_gen);
    if (c->flags & ~(PGMOE_FLAG_HOST_ONLY | PGMOE_FLAG_FETCH_MEMCPY | PGMOE_FLAG_FETCH_AUTO)) BAD("unknown flag bits 0x%x", c->flags);
    if ((c->flags & PGMOE_FLAG_FETCH_MEMCPY) && (c->flags & PGMOE_FLAG_FETCH_AUTO))
        BAD("PGMOE_FLAG_FETCH_MEMCPY and PGMOE_FLAG_FETCH_AUTO exclude each other");
    if (c->cache_slots < 0 || c->cache_slots > PGMOE_MAX_CACHE_SLOTS || c->cache_slots > c->n_experts)
        BAD("cache_slots=%d outside 0..min(%d, n_experts)", c->cache_slots, PGMOE_MAX_CACHE_SLOTS);
    if (c->cache_policy < PGMOE_CACHE_LRU || c->cache_policy > PGMOE_CACHE_LIFO) BAD("cache_policy=%d unknown", c->cache_policy);
    if (c->pregate_distance < 0 || c->pregate_distance > PGMOE_MAX_PREGATE_DISTANCE)
        BAD("pregate_distance=%d outside 0..%d", c->pregate_distance, PGMOE_MAX_PREGATE_DISTANCE);
    if (c->cache_slots > 0 && (c->flags & PGMOE_FLAG_FETCH_MEMCPY))
        BAD("the expert cache is kept by the device-side pull engine: not available with PGMOE_FLAG_FETCH_MEMCPY");
    const uint64_t eb = (uint64_t)2 * c->d_model * c->d_ff * (c->dtype == PGMOE_F32 ? 4 : 2);
    const uint64_t slots = c->slots_per_gen > 0 ? c->slots_per_gen : default_slots(*c);
    // (the same rule pgmoe_create applies)
    const bool auto_copy_engines = (c->flags & PGMOE_FLAG_FETCH_AUTO) && c->cache_slots == 0 && slots * eb >= PGMOE_AUTO_COPY_ENGINE_BYTES;
    if (!(c->flags & PGMOE_FLAG_FETCH_MEMCPY) && !auto_copy_engines) {
        // the pull kernels number the 16-byte (4-byte if the blob is no multiple of 16) units of
        // everything one migration may copy with 32 bits
        if ((slots + c->cache_slots) * (eb / (eb % 16 ? 4 : 16)) >= (1ull << 32) - (1ull << 20))
            BAD("%llu slots of %llu-byte experts are more than one device-side migration can address: fewer slots_per_gen, "
                "or PGMOE_FLAG_FETCH_MEMCPY", (unsigned long long)(slots + c->cache_slots), (unsigned long long)eb);
    }
    return PGMOE_OK;
#undef BAD
}

}  // namespace pgmoe

// ---------------------------------------------------------------- weight layout (host)
// Element (k, n) of a [K, N] bf16 matrix sits in tile (k/32, n/16) at ((n%16) + 16*((k%32)/8))*8 + k%8
// (the layout described in pgmoe.h); tiles are ordered n-major or k-major.
template <bool PACK>
static void tile_copy(uint16_t *tiled, uint16_t *plain, int K, int N, bool nt_major) {
    for (int kt = 0; kt < K / 32; ++kt)
        for (int nt = 0; nt < N / 16; ++nt) {
            const size_t tile = nt_major ? (size_t)nt * (K / 32) + kt : (size_t)kt * (N / 16) + nt;
            uint16_t *t = tiled + tile * 512;
            for (int g = 0; g < 4; ++g)
                for (int nn = 0; nn < 16; ++nn) {
                    uint16_t *cell = t + (size_t)(nn + 16 * g) * 8;
                    uint16_t *src = plain + (size_t)(kt * 32 + g * 8) * N + nt * 16 + nn;
                    for (int j = 0; j < 8; ++j) {
                        if (PACK) cell[j] = src[(size_t)j * N];
                        else src[(size_t)j * N] = cell[j];
                    }
                }
        }
}

using namespace pgmoe;

__global__ void noop_kernel() {}

// Median event-to-event time around an empty kernel minus the period of back-to-back empty
// kernels: the share of an event pair's reading that is not kernel time.
static int measure_pair_overhead(pgmoe_ctx *ctx, float *out_ms) {
    constexpr int N = 33;
    hipStream_t s = ctx->copy2;  // any idle stream of the context
    hipEvent_t ev[2 * N];
    for (auto &e : ev) PG_HIP(ctx, hipEventCreate(&e));
    for (int i = 0; i < 8; ++i) hipLaunchKernelGGL(noop_kernel, dim3(1), dim3(64), 0, s);
    for (int i = 0; i < N; ++i) {
        PG_HIP(ctx, hipEventRecord(ev[2 * i], s));
        hipLaunchKernelGGL(noop_kernel, dim3(1), dim3(64), 0, s);
        PG_HIP(ctx, hipEventRecord(ev[2 * i + 1], s));
    }
    PG_HIP(ctx, hipStreamSynchronize(s));
    float pair[N];
    for (int i = 0; i < N; ++i) PG_HIP(ctx, hipEventElapsedTime(&pair[i], ev[2 * i], ev[2 * i + 1]));
    std::sort(pair, pair + N);
    PG_HIP(ctx, hipEventRecord(ev[0], s));
    for (int i = 0; i < 64; ++i) hipLaunchKernelGGL(noop_kernel, dim3(1), dim3(64), 0, s);
    PG_HIP(ctx, hipEventRecord(ev[1], s));
    PG_HIP(ctx, hipStreamSynchronize(s));
    float run = 0.f;
    PG_HIP(ctx, hipEventElapsedTime(&run, ev[0], ev[1]));
    for (auto &e : ev) (void)hipEventDestroy(e);
    const float oh = pair[N / 2] - run / 64.f;
    *out_ms = oh > 0.f ? oh : 0.f;
    return PGMOE_OK;
}

static void free_timing(pgmoe_ctx *c) {
    for (int i = 0; i < c->tim_cap; ++i) {
        if (c->tim_begin && c->tim_begin[i]) (void)hipEventDestroy(c->tim_begin[i]);
        if (c->tim_end && c->tim_end[i]) (void)hipEventDestroy(c->tim_end[i]);
    }
    delete[] c->tim_begin;
    delete[] c->tim_end;
    c->tim_begin = c->tim_end = nullptr;
    c->tim_cap = c->tim_n = 0;
    c->tim_on = false;
}

extern "C" {

const char *pgmoe_last_error(const pgmoe_ctx *ctx) { return ctx ? ctx->err : g_err; }

size_t pgmoe_expert_bytes(const pgmoe_config *cfg) {
    char buf[256];
    if (check_config(cfg, buf, sizeof buf) != PGMOE_OK) return 0;
    return (size_t)2 * cfg->d_model * cfg->d_ff * (cfg->dtype == PGMOE_F32 ? 4 : 2);
}

int pgmoe_create(pgmoe_ctx **out, const pgmoe_config *cfg) {
    if (!out) return fail(nullptr, PGMOE_EINVAL, "pgmoe_create: out is NULL");
    *out = nullptr;
    char buf[256];
    if (check_config(cfg, buf, sizeof buf) != PGMOE_OK) return fail(nullptr, PGMOE_EINVAL, "pgmoe_create: %s", buf);
    if (cfg->dtype == PGMOE_BF16 && !ffn_supports_d_model(cfg->d_model))
        return fail(nullptr, PGMOE_EINVAL, "pgmoe_create: no bf16 expert kernel is built for d_model=%d (built: 64, 128, 256, 512, 768, 1024, 2048)",
                    cfg->d_model);
    pgmoe_ctx *c = new (std::nothrow) pgmoe_ctx();
    if (!c) return fail(nullptr, PGMOE_EINVAL, "pgmoe_create: out of host memory");
    c->cfg = *cfg;
    c->host_only = (cfg->flags & PGMOE_FLAG_HOST_ONLY) != 0;
    c->elem = cfg->dtype == PGMOE_F32 ? 4 : 2;
    c->expert_bytes = pgmoe_expert_bytes(cfg);
    c->slots = cfg->slots_per_gen > 0 ? cfg->slots_per_gen : default_slots(*cfg);
    c->pull = (cfg->flags & PGMOE_FLAG_FETCH_MEMCPY) == 0;
    if ((cfg->flags & PGMOE_FLAG_FETCH_AUTO) && cfg->cache_slots == 0 &&
        (size_t)c->slots * c->expert_bytes >= PGMOE_AUTO_COPY_ENGINE_BYTES)
        c->pull = false;
    c->distance = cfg->pregate_distance > 0 ? cfg->pregate_distance : 1;
    c->n_gen = c->distance + 1;
    c->store_mode = STORE_NONE;
    c->err[0] = 0;
    for (int g = 0; g < kGen; ++g) {
        c->fetched_block[g] = -1;
        c->live_slots[g] = 0;
        c->ffn_recorded[g] = false;
    }
    c->stats = new (std::nothrow) BlockStats[cfg->n_blocks]();
    c->routed = new (std::nothrow) bool[cfg->n_blocks]();
    if (!c->stats || !c->routed) {
        delete[] c->stats;
        delete[] c->routed;
        delete c;
        return fail(nullptr, PGMOE_EINVAL, "pgmoe_create: out of host memory");
    }
    if (!c->host_only) {
        int rc = PGMOE_OK;
        auto H = [&](hipError_t e, const char *what) {
            if (e != hipSuccess && rc == PGMOE_OK) rc = hip_fail(nullptr, e, what);
            return e == hipSuccess;
        };
        int ndev = 0;
        if (hipGetDeviceCount(&ndev) != hipSuccess || ndev < 1) {
            (void)hipGetLastError();
            pgmoe_destroy(c);
            return fail(nullptr, PGMOE_ENODEVICE, "pgmoe_create: no HIP device is visible");
        }
        H(hipGetDevice(&c->device), "hipGetDevice");
        if (rc == PGMOE_OK && (rc = resolve_static_scratch(c)) != PGMOE_OK) fail(nullptr, rc, "%s", c->err);
        // sticky flags and turn counters (64 bytes), then per block: copy clocks (2 x 8 bytes), distinct-expert count
        const size_t flag_bytes = 64 + (2 * sizeof(unsigned long long) + sizeof(int32_t)) * (size_t)cfg->n_blocks;
        H(hipMalloc((void **)&c->dev_flags, flag_bytes), "hipMalloc(flags)");
        if (rc == PGMOE_OK) H(hipMemset(c->dev_flags, 0, flag_bytes), "hipMemset(flags)");
        c->dev_copy_clock = reinterpret_cast<unsigned long long *>(reinterpret_cast<char *>(c->dev_flags) + 64);
        c->dev_unique = reinterpret_cast<int32_t *>(c->dev_copy_clock + 2 * (size_t)cfg->n_blocks);
        size_t n_idx = (size_t)cfg->max_tokens * cfg->top_k;
        if (rc == PGMOE_OK) H(hipMalloc((void **)&c->dev_src_row, (size_t)cfg->n_blocks * n_idx * sizeof(int32_t)), "hipMalloc(src_row)");
        if (rc == PGMOE_OK) H(hipHostMalloc((void **)&c->idx_staging, n_idx * sizeof(int32_t), hipHostMallocDefault), "hipHostMalloc(idx staging)");
        // idx_ready is the one event the host itself polls before it reads the staged indices (memcpy
        // mode): it keeps the default, system-scope release, so the copy before it is visible to the host
        if (rc == PGMOE_OK) H(hipEventCreateWithFlags(&c->idx_ready, hipEventDisableTiming), "hipEventCreate");
        if (rc == PGMOE_OK) H(hipEventCreateWithFlags(&c->step_start, hipEventDisableTiming | hipEventReleaseToDevice), "hipEventCreate");
        if (rc == PGMOE_OK) H(hipStreamCreateWithFlags(&c->copy2, hipStreamNonBlocking), "hipStreamCreate");
        for (int g = 0; g < kGen && rc == PGMOE_OK; ++g) {
            // these two only order device work against device work: no host-visible release needed
            H(hipEventCreateWithFlags(&c->fetch_done[g], hipEventDisableTiming | hipEventReleaseToDevice), "hipEventCreate");
            H(hipEventCreateWithFlags(&c->ffn_done[g], hipEventDisableTiming | hipEventReleaseToDevice), "hipEventCreate");
            H(hipEventCreateWithFlags(&c->fork[g], hipEventDisableTiming | hipEventReleaseToDevice), "hipEventCreate");
            H(hipEventCreateWithFlags(&c->join[g], hipEventDisableTiming | hipEventReleaseToDevice), "hipEventCreate");
        }
        if (rc == PGMOE_OK) {
            hipEvent_t **arrays[] = {&c->fetch_begin, &c->fetch_end, &c->ev_c0, &c->ev_ready, &c->ev_waited, &c->ev_c1};
            for (hipEvent_t **a : arrays) {
                *a = new (std::nothrow) hipEvent_t[cfg->n_blocks]();
                if (!*a && rc == PGMOE_OK) rc = fail(nullptr, PGMOE_EINVAL, "pgmoe_create: out of host memory");
                for (int b = 0; b < cfg->n_blocks && rc == PGMOE_OK; ++b) H(hipEventCreate(&(*a)[b]), "hipEventCreate");
            }
            c->traced = new (std::nothrow) bool[cfg->n_blocks]();
            if (!c->traced && rc == PGMOE_OK) rc = fail(nullptr, PGMOE_EINVAL, "pgmoe_create: out of host memory");
        }
        if (rc != PGMOE_OK) {
            pgmoe_destroy(c);
            return rc;
        }
    }
    *out = c;
    return PGMOE_OK;
}

int pgmoe_destroy(pgmoe_ctx *c) {
    if (!c) return PGMOE_OK;
    if (!c->host_only) {
        (void)hipDeviceSynchronize();
        if (c->slot_pool) (void)hipFree(c->slot_pool);
        if (c->cache_pool) (void)hipFree(c->cache_pool);
        if (c->cache_state) (void)hipFree(c->cache_state);
        if (c->dev_table) (void)hipFree(c->dev_table);
        if (c->cache_stats) (void)hipFree(c->cache_stats);
        delete[] c->cache_parity;
        if (c->dev_flags) (void)hipFree(c->dev_flags);
        if (c->dev_src_row) (void)hipFree(c->dev_src_row);
        if (c->idx_staging) (void)hipHostFree(c->idx_staging);
        if (c->idx_ready) (void)hipEventDestroy(c->idx_ready);
        if (c->step_start) (void)hipEventDestroy(c->step_start);
        if (c->copy2) (void)hipStreamDestroy(c->copy2);
        for (hipStream_t sp : c->spare_streams)
            if (sp) (void)hipStreamDestroy(sp);
        for (int g = 0; g < kGen; ++g) {
            if (c->fetch_done[g]) (void)hipEventDestroy(c->fetch_done[g]);
            if (c->ffn_done[g]) (void)hipEventDestroy(c->ffn_done[g]);
            if (c->fork[g]) (void)hipEventDestroy(c->fork[g]);
            if (c->join[g]) (void)hipEventDestroy(c->join[g]);
        }
        hipEvent_t *arrays[] = {c->fetch_begin, c->fetch_end, c->ev_c0, c->ev_ready, c->ev_waited, c->ev_c1};
        for (hipEvent_t *a : arrays) {
            for (int b = 0; a && b < c->cfg.n_blocks; ++b)
                if (a[b]) (void)hipEventDestroy(a[b]);
            delete[] a;
        }
        delete[] c->traced;
        free_timing(c);
    }
    delete[] c->stats;
    delete[] c->routed;
    delete c;
    return PGMOE_OK;
}

size_t pgmoe_workspace_bytes(const pgmoe_ctx *ctx) {
    if (!ctx) return 0;
    return ffn_workspace_bytes(ctx->cfg);
}

int pgmoe_pack_expert(const pgmoe_config *cfg, const void *w1, const void *w2, void *blob) {
    char buf[256];
    if (check_config(cfg, buf, sizeof buf) != PGMOE_OK) return fail(nullptr, PGMOE_EINVAL, "pgmoe_pack_expert: %s", buf);
    if (!w1 || !w2 || !blob) return fail(nullptr, PGMOE_EINVAL, "pgmoe_pack_expert: NULL pointer");
    const size_t n = (size_t)cfg->d_model * cfg->d_ff;
    if (cfg->dtype == PGMOE_F32) {
        memcpy(blob, w1, n * 4);
        memcpy((char *)blob + n * 4, w2, n * 4);
        return PGMOE_OK;
    }
    uint16_t *b = (uint16_t *)blob;
    tile_copy<true>(b, (uint16_t *)w1, cfg->d_model, cfg->d_ff, /*nt_major=*/true);
    tile_copy<true>(b + n, (uint16_t *)w2, cfg->d_ff, cfg->d_model, /*nt_major=*/false);
    return PGMOE_OK;
}

int pgmoe_unpack_expert(const pgmoe_config *cfg, const void *blob, void *w1, void *w2) {
    char buf[256];
    if (check_config(cfg, buf, sizeof buf) != PGMOE_OK) return fail(nullptr, PGMOE_EINVAL, "pgmoe_unpack_expert: %s", buf);
    if (!w1 || !w2 || !blob) return fail(nullptr, PGMOE_EINVAL, "pgmoe_unpack_expert: NULL pointer");
    const size_t n = (size_t)cfg->d_model * cfg->d_ff;
    if (cfg->dtype == PGMOE_F32) {
        memcpy(w1, blob, n * 4);
        memcpy(w2, (const char *)blob + n * 4, n * 4);
        return PGMOE_OK;
    }
    uint16_t *b = (uint16_t *)blob;
    tile_copy<false>(b, (uint16_t *)w1, cfg->d_model, cfg->d_ff, true);
    tile_copy<false>(b + n, (uint16_t *)w2, cfg->d_ff, cfg->d_model, false);
    return PGMOE_OK;
}

int pgmoe_unique_experts(const int32_t *idx, int n, int E, int32_t *unique_out) {
    if (n < 0 || E < 1 || E > PGMOE_MAX_EXPERTS) return fail(nullptr, PGMOE_EINVAL, "pgmoe_unique_experts: n=%d, E=%d out of range", n, E);
    if (n > 0 && (!idx || !unique_out)) return fail(nullptr, PGMOE_EINVAL, "pgmoe_unique_experts: NULL pointer");
    uint64_t seen[PGMOE_MAX_EXPERTS / 64] = {0, 0, 0, 0};
    for (int i = 0; i < n; ++i) {
        const int32_t e = idx[i];
        if (e < 0 || e >= E) return fail(nullptr, PGMOE_EBADINDEX, "pgmoe_unique_experts: idx[%d]=%d outside [0,%d)", i, e, E);
        seen[e >> 6] |= 1ull << (e & 63);
    }
    int u = 0;
    for (int e = 0; e < E; ++e)
        if (seen[e >> 6] >> (e & 63) & 1) unique_out[u++] = e;
    return u;
}

// ---------------------------------------------------------------- argument checks
static int check_common(pgmoe_ctx *ctx, const char *fn, int T) {
    if (!ctx) return fail(nullptr, PGMOE_EINVAL, "%s: ctx is NULL", fn);
    if (T < 0 || T > ctx->cfg.max_tokens) return fail(ctx, PGMOE_EINVAL, "%s: T=%d outside 0..max_tokens=%d", fn, T, ctx->cfg.max_tokens);
    return PGMOE_OK;
}

#define NEED_PTR(ctx, fn, p, a)                                                                        \
    do {                                                                                               \
        if (!(p)) return fail(ctx, PGMOE_EINVAL, "%s: %s is NULL", fn, #p);                            \
        if (!aligned(p, a)) return fail(ctx, PGMOE_EINVAL, "%s: %s is not %d-byte aligned", fn, #p, (int)(a)); \
    } while (0)
#define OPT_PTR(ctx, fn, p, a)                                                                         \
    do {                                                                                               \
        if ((p) && !aligned(p, a)) return fail(ctx, PGMOE_EINVAL, "%s: %s is not %d-byte aligned", fn, #p, (int)(a)); \
    } while (0)
#define NEED_DEVICE(ctx, fn)                                                                           \
    do {                                                                                               \
        if ((ctx)->host_only) return fail(ctx, PGMOE_ENODEVICE, "%s: context is host-only, nothing can be launched", fn); \
    } while (0)

int pgmoe_pregate_topk(pgmoe_ctx *ctx, const void *x, const void *w_gate, const float *bias, int T,
                       int32_t *topk_idx, float *topk_prob, float *probs_out, void *stream) {
    const char *fn = "pgmoe_pregate_topk";
    int rc = check_common(ctx, fn, T);
    if (rc) return rc;
    NEED_PTR(ctx, fn, x, 16);
    NEED_PTR(ctx, fn, w_gate, 16);
    OPT_PTR(ctx, fn, bias, 4);
    NEED_PTR(ctx, fn, topk_idx, 4);
    NEED_PTR(ctx, fn, topk_prob, 4);
    OPT_PTR(ctx, fn, probs_out, 4);
    NEED_DEVICE(ctx, fn);
    if (T == 0) return PGMOE_OK;
    return launch_gate(ctx, x, w_gate, bias, T, topk_idx, topk_prob, probs_out, (hipStream_t)stream);
}

int pgmoe_permute(pgmoe_ctx *ctx, const void *x, const int32_t *topk_idx, int T, void *x_perm,
                  int32_t *row_of, int32_t *expert_offsets, void *stream) {
    const char *fn = "pgmoe_permute";
    int rc = check_common(ctx, fn, T);
    if (rc) return rc;
    NEED_PTR(ctx, fn, x, 16);
    NEED_PTR(ctx, fn, topk_idx, 4);
    NEED_PTR(ctx, fn, x_perm, 16);
    NEED_PTR(ctx, fn, row_of, 4);
    NEED_PTR(ctx, fn, expert_offsets, 4);
    NEED_DEVICE(ctx, fn);
    return launch_permute(ctx, x, topk_idx, T, x_perm, row_of, expert_offsets, (hipStream_t)stream);
}

int pgmoe_combine(pgmoe_ctx *ctx, const void *y_perm, const int32_t *row_of, const float *topk_prob,
                  int T, void *y, const void *x_res, void *x_next, void *stream) {
    const char *fn = "pgmoe_combine";
    int rc = check_common(ctx, fn, T);
    if (rc) return rc;
    NEED_PTR(ctx, fn, y_perm, 16);
    NEED_PTR(ctx, fn, row_of, 4);
    NEED_PTR(ctx, fn, topk_prob, 4);
    OPT_PTR(ctx, fn, y, 16);
    OPT_PTR(ctx, fn, x_res, 16);
    OPT_PTR(ctx, fn, x_next, 16);
    if (!y && !x_next) return fail(ctx, PGMOE_EINVAL, "%s: both y and x_next are NULL", fn);
    if ((x_res == nullptr) != (x_next == nullptr)) return fail(ctx, PGMOE_EINVAL, "%s: x_res and x_next must be given together", fn);
    NEED_DEVICE(ctx, fn);
    if (T == 0) return PGMOE_OK;
    return launch_combine(ctx, y_perm, row_of, topk_prob, T, y, x_res, x_next, (hipStream_t)stream);
}

int pgmoe_migration_engine(const pgmoe_ctx *ctx) {
    if (!ctx) return fail(nullptr, PGMOE_EINVAL, "pgmoe_migration_engine: ctx is NULL");
    return ctx->pull ? 0 : 1;
}

const char *pgmoe_ffn_kernel_name(const pgmoe_ctx *ctx, int n_rows) {
    if (!ctx) return nullptr;
    return ffn_kernel_name(ctx->cfg, n_rows < 1 ? 1 : n_rows);
}

int pgmoe_ffn_timing_begin(pgmoe_ctx *ctx, int max_launches) {
    const char *fn = "pgmoe_ffn_timing_begin";
    if (!ctx) return fail(nullptr, PGMOE_EINVAL, "%s: ctx is NULL", fn);
    if (max_launches < 1 || max_launches > (1 << 20)) return fail(ctx, PGMOE_EINVAL, "%s: max_launches=%d outside 1..2^20", fn, max_launches);
    NEED_DEVICE(ctx, fn);
    if (ctx->tim_cap < max_launches) {
        free_timing(ctx);
        ctx->tim_begin = new (std::nothrow) hipEvent_t[max_launches]();
        ctx->tim_end = new (std::nothrow) hipEvent_t[max_launches]();
        if (!ctx->tim_begin || !ctx->tim_end) return fail(ctx, PGMOE_EINVAL, "%s: out of host memory", fn);
        ctx->tim_cap = max_launches;
        for (int i = 0; i < max_launches; ++i) {
            PG_HIP(ctx, hipEventCreate(&ctx->tim_begin[i]));
            PG_HIP(ctx, hipEventCreate(&ctx->tim_end[i]));
        }
    }
    int rc = measure_pair_overhead(ctx, &ctx->tim_overhead_ms);
    if (rc) return rc;
    ctx->tim_n = 0;
    ctx->tim_on = true;
    return PGMOE_OK;
}

int pgmoe_ffn_timing_end(pgmoe_ctx *ctx, int *n_out, float *total_ms_out, float *pair_overhead_ms_out) {
    const char *fn = "pgmoe_ffn_timing_end";
    if (!ctx) return fail(nullptr, PGMOE_EINVAL, "%s: ctx is NULL", fn);
    if (!n_out || !total_ms_out) return fail(ctx, PGMOE_EINVAL, "%s: NULL output pointer", fn);
    NEED_DEVICE(ctx, fn);
    ctx->tim_on = false;
    double total = 0.0;
    for (int i = 0; i < ctx->tim_n; ++i) {
        PG_HIP(ctx, hipEventSynchronize(ctx->tim_end[i]));
        float ms = 0.f;
        PG_HIP(ctx, hipEventElapsedTime(&ms, ctx->tim_begin[i], ctx->tim_end[i]));
        total += ms;
    }
    *n_out = ctx->tim_n;
    *total_ms_out = (float)total;
    if (pair_overhead_ms_out) *pair_overhead_ms_out = ctx->tim_overhead_ms;
    return PGMOE_OK;
}

int pgmoe_device_flags(pgmoe_ctx *ctx, uint32_t *flags_out) {
    const char *fn = "pgmoe_device_flags";
    if (!ctx) return fail(nullptr, PGMOE_EINVAL, "%s: ctx is NULL", fn);
    if (!flags_out) return fail(ctx, PGMOE_EINVAL, "%s: flags_out is NULL", fn);
    NEED_DEVICE(ctx, fn);
    PG_HIP(ctx, hipDeviceSynchronize());
    PG_HIP(ctx, hipMemcpy(flags_out, ctx->dev_flags, sizeof(uint32_t), hipMemcpyDeviceToHost));
    PG_HIP(ctx, hipMemset(ctx->dev_flags, 0, sizeof(uint32_t)));
    return PGMOE_OK;
}

}  // extern "C"
