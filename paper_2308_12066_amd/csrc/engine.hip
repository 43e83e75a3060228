// Expert store, preemptive expert migration and the whole-stack step.
//
// Sec. IV-C of the paper: all experts live in host memory; once the pre-gate of block N has
// picked block N+1's experts, only those are copied to the GPU while block N executes, and
// the GPU holds the activated experts of two consecutive blocks at most.  Here that is a
// slot pool of two generations (generation = block & 1; N + 1 generations, block mod (N + 1),
// when the pre-gate looks N blocks ahead).  Read-after-write: the FFN of a
// block waits on the generation's fetch_done event (unless the fetch ran on the FFN's own
// stream).  Write-after-read: a fetch into a generation must not start before the FFN that
// read it last has finished; the indices the fetch depends on are produced on the compute
// stream after that FFN, so waiting for them covers it, and only when the FFN ran on some
// other stream is an extra event recorded there (at fetch time, behind the FFN) and waited on.
// Every second block from block N+1 on is fetched on an internal second copy stream, so the
// migration of block i+1 does not queue behind that of block i: the host link stays busy across the
// hand-over (two pull kernels share the link while they overlap).
#include <algorithm>
#include <chrono>
#include <new>

#include "pgmoe_internal.h"

using namespace pgmoe;

namespace {

int check_store_args(pgmoe_ctx *ctx, const char *fn, const void *base, size_t expert_stride, size_t block_stride) {
    if (!ctx) return fail(nullptr, PGMOE_EINVAL, "%s: ctx is NULL", fn);
    if (!base) return fail(ctx, PGMOE_EINVAL, "%s: base is NULL", fn);
    if (!aligned(base, 256)) return fail(ctx, PGMOE_EINVAL, "%s: base is not 256-byte aligned", fn);
    if (expert_stride < ctx->expert_bytes || expert_stride % 256)
        return fail(ctx, PGMOE_EINVAL, "%s: expert_stride=%zu must be a multiple of 256 and >= %zu", fn, expert_stride, ctx->expert_bytes);
    if (block_stride < expert_stride * (size_t)ctx->cfg.n_experts || block_stride % 256)
        return fail(ctx, PGMOE_EINVAL, "%s: block_stride=%zu must be a multiple of 256 and >= n_experts*expert_stride", fn, block_stride);
    return PGMOE_OK;
}

// Make `ps` wait for the FFN that last read generation `gen`.  Work already queued on `cs`
// precedes the indices this fetch waits for, so an FFN on `cs` (or on `ps` itself) needs
// nothing; an FFN on any other stream gets an event recorded behind it now.
int wait_for_last_reader(pgmoe_ctx *ctx, int gen, hipStream_t cs, hipStream_t ps) {
    if (!ctx->ffn_recorded[gen]) return PGMOE_OK;
    const hipStream_t fs = ctx->ffn_stream[gen];
    if (fs == cs || fs == ps) return PGMOE_OK;
    PG_HIP(ctx, hipEventRecord(ctx->ffn_done[gen], fs));
    PG_HIP(ctx, hipStreamWaitEvent(ps, ctx->ffn_done[gen], 0));
    return PGMOE_OK;
}

int check_block(pgmoe_ctx *ctx, const char *fn, int block) {
    if (block < 0 || block >= ctx->cfg.n_blocks) return fail(ctx, PGMOE_EINVAL, "%s: block=%d outside 0..%d", fn, block, ctx->cfg.n_blocks - 1);
    return PGMOE_OK;
}

}  // namespace

extern "C" {

int pgmoe_register_host_experts(pgmoe_ctx *ctx, const void *host_base, size_t expert_stride, size_t block_stride) {
    const char *fn = "pgmoe_register_host_experts";
    int rc = check_store_args(ctx, fn, host_base, expert_stride, block_stride);
    if (rc) return rc;
    if (!ctx->host_only) {
        hipPointerAttribute_t attr;
        hipError_t e = hipPointerGetAttributes(&attr, host_base);
        if (e != hipSuccess || attr.type != hipMemoryTypeHost) {
            (void)hipGetLastError();
            return fail(ctx, PGMOE_ENOTPINNED, "%s: host_base is not pinned host memory (allocate it with hipHostMalloc)", fn);
        }
        void *dev_view = nullptr;
        PG_HIP(ctx, hipHostGetDevicePointer(&dev_view, const_cast<void *>(host_base), 0));
        ctx->store_dev = (const char *)dev_view;
        if (!ctx->slot_pool) {
            const size_t bytes = (size_t)ctx->n_gen * ctx->slots * ctx->expert_bytes;
            PG_HIP(ctx, hipMalloc((void **)&ctx->slot_pool, bytes));
        }
        if (ctx->cfg.cache_slots > 0 && !ctx->cache_pool) {
            const size_t L = ctx->cfg.n_blocks;
            PG_HIP(ctx, hipMalloc((void **)&ctx->cache_pool, L * ctx->cfg.cache_slots * ctx->expert_bytes));
            PG_HIP(ctx, hipMalloc((void **)&ctx->cache_state, cache_state_bytes(ctx->cfg)));
            PG_HIP(ctx, hipMalloc((void **)&ctx->dev_table, L * PGMOE_MAX_EXPERTS * sizeof(unsigned long long)));
            PG_HIP(ctx, hipMalloc((void **)&ctx->cache_stats, L * 4 * sizeof(int32_t)));
            ctx->cache_parity = new (std::nothrow) unsigned char[L]();
            if (!ctx->cache_parity) return fail(ctx, PGMOE_EINVAL, "%s: out of host memory", fn);
        }
        if (ctx->cfg.cache_slots > 0) {  // (re)start with an empty cache: every slot holds expert -1
            PG_HIP(ctx, hipDeviceSynchronize());
            PG_HIP(ctx, hipMemset(ctx->cache_state, 0xff, cache_state_bytes(ctx->cfg)));
            PG_HIP(ctx, hipMemset(ctx->cache_stats, 0, (size_t)ctx->cfg.n_blocks * 4 * sizeof(int32_t)));
            memset(ctx->cache_parity, 0, (size_t)ctx->cfg.n_blocks);
        }
    }
    ctx->store_mode = STORE_HOST;
    ctx->store_base = (const char *)host_base;
    ctx->expert_stride = expert_stride;
    ctx->block_stride = block_stride;
    for (int g = 0; g < kGen; ++g) {
        ctx->fetched_block[g] = -1;
        ctx->live_slots[g] = 0;
    }
    return PGMOE_OK;
}

int pgmoe_register_resident_experts(pgmoe_ctx *ctx, const void *dev_base, size_t expert_stride, size_t block_stride) {
    const char *fn = "pgmoe_register_resident_experts";
    int rc = check_store_args(ctx, fn, dev_base, expert_stride, block_stride);
    if (rc) return rc;
    ctx->store_mode = STORE_RESIDENT;
    ctx->store_base = (const char *)dev_base;
    ctx->expert_stride = expert_stride;
    ctx->block_stride = block_stride;
    return PGMOE_OK;
}

// Shared body of pgmoe_fetch_experts (all == false: the experts topk_idx selects) and
// pgmoe_fetch_all_experts (all == true: every expert of the block, slot = expert id).
static int fetch_impl(pgmoe_ctx *ctx, const char *fn, int block, bool all, const int32_t *topk_idx, int T,
                      void *compute_stream, void *copy_stream, int *n_unique_out) {
    if (!ctx) return fail(nullptr, PGMOE_EINVAL, "%s: ctx is NULL", fn);
    int rc = check_block(ctx, fn, block);
    if (rc) return rc;
    if (T < 0 || T > ctx->cfg.max_tokens) return fail(ctx, PGMOE_EINVAL, "%s: T=%d outside 0..max_tokens=%d", fn, T, ctx->cfg.max_tokens);
    if (!all && !topk_idx) return fail(ctx, PGMOE_EINVAL, "%s: topk_idx is NULL", fn);
    if (!all && !aligned(topk_idx, 4)) return fail(ctx, PGMOE_EINVAL, "%s: topk_idx is not 4-byte aligned", fn);
    if (ctx->store_mode == STORE_NONE) return fail(ctx, PGMOE_ESTATE, "%s: no expert store registered", fn);
    if (ctx->store_mode == STORE_RESIDENT) {
        if (n_unique_out) *n_unique_out = -1;
        return PGMOE_OK;
    }
    if (all && ctx->slots < ctx->cfg.n_experts)
        return fail(ctx, PGMOE_ENOSLOT, "%s: fetching all %d experts needs slots_per_gen = n_experts (have %d)", fn, ctx->cfg.n_experts, ctx->slots);
    if (ctx->host_only) return fail(ctx, PGMOE_ENODEVICE, "%s: context is host-only, nothing can be launched", fn);
    hipStream_t cs = (hipStream_t)compute_stream, ps = (hipStream_t)copy_stream;
    const int n = all ? 0 : T * ctx->cfg.top_k;
    const int gen = block % ctx->n_gen;
    const bool inline_fetch = ps == cs;  // exposed fetch on the compute stream itself: plain stream order
    if (!inline_fetch && ctx->pull_seq >= 0) {
        if (ctx->pull_seq & 1) ps = ctx->copy2;  // inside a step the migrations take turns on the link (fetch.hip): alternate from the first one on
    } else if (!inline_fetch && block > ctx->distance && ((block - ctx->distance) & 1)) {
        ps = ctx->copy2;  // blocks 0..N queue on the caller's stream, then alternate
    }
    BlockStats &st = ctx->stats[block];
    st = BlockStats();

    if (ctx->pull) {
        // device-side migration: the copy stream waits for the indices and for the generation
        // to be free, then one kernel dedupes and pulls; the host is not involved
        if (!inline_fetch && !ctx->routed_on_copy_stream) {
            PG_HIP(ctx, hipEventRecord(ctx->idx_ready, cs));
            PG_HIP(ctx, hipStreamWaitEvent(ps, ctx->idx_ready, 0));
        }
        rc = wait_for_last_reader(ctx, gen, cs, ps);
        if (rc) return rc;
        if (ctx->fetch_timing) PG_HIP(ctx, hipEventRecord(ctx->fetch_begin[block], ps));
        const int seq = ctx->pull_seq >= 0 ? ctx->pull_seq++ : -1;  // inside a step: its place in the queue for the link
        rc = launch_fetch_pull(ctx, block, all, topk_idx, n, ps, seq, seq >= 0 && seq == ctx->pull_last, ctx->turn_timeout_ticks);
        if (rc) return rc;
        if (ctx->fetch_timing) PG_HIP(ctx, hipEventRecord(ctx->fetch_end[block], ps));
        if (!inline_fetch) PG_HIP(ctx, hipEventRecord(ctx->fetch_done[gen], ps));
        ctx->fetch_stream[gen] = ps;
        ctx->gen_all[gen] = all;
        ctx->gen_table[gen] = ctx->cfg.cache_slots > 0 && !all;
        ctx->fetched_block[gen] = block;
        ctx->live_slots[gen] = -1;  // known on the device only
        st.timed = ctx->fetch_timing;
        st.in_line = inline_fetch;
        st.pulled = true;
        st.cached = ctx->gen_table[gen];
        st.s.n_unique = -1;
        if (n_unique_out) {
            PG_HIP(ctx, hipStreamSynchronize(ps));
            int32_t u = 0;
            PG_HIP(ctx, hipMemcpy(&u, ctx->dev_unique + block, sizeof u, hipMemcpyDeviceToHost));
            if (ctx->gen_table[gen]) PG_HIP(ctx, hipMemcpy(&u, ctx->cache_stats + (size_t)block * 4, sizeof u, hipMemcpyDeviceToHost));
            *n_unique_out = u;
        }
        return PGMOE_OK;
    }

    // The host waits for the routing below: under stream capture nothing executes, so that wait
    // would never end.  Refuse before anything is queued.
    {
        hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
        if (hipStreamIsCapturing(cs, &cap) == hipSuccess && cap != hipStreamCaptureStatusNone)
            return fail(ctx, PGMOE_ESTATE, "%s: this context migrates with the copy engines (the host reads the routing back), which cannot "
                        "be captured into a graph; create the context without PGMOE_FLAG_FETCH_MEMCPY / PGMOE_FLAG_FETCH_AUTO", fn);
    }
    // 1. bring the indices to the host (the only host wait of the block)
    const auto t0 = std::chrono::steady_clock::now();
    if (all && !inline_fetch) {
        // no indices to wait for: order the copies behind what is queued on the compute stream
        PG_HIP(ctx, hipEventRecord(ctx->idx_ready, cs));
        PG_HIP(ctx, hipStreamWaitEvent(ps, ctx->idx_ready, 0));
    }
    if (n > 0) {
        PG_HIP(ctx, hipMemcpyAsync(ctx->idx_staging, topk_idx, (size_t)n * sizeof(int32_t), hipMemcpyDeviceToHost, cs));
        PG_HIP(ctx, hipEventRecord(ctx->idx_ready, cs));
        hipError_t q;
        while ((q = hipEventQuery(ctx->idx_ready)) == hipErrorNotReady) {
        }
        if (q != hipSuccess) return hip_fail(ctx, q, "hipEventQuery(idx_ready)");
    }
    st.s.wait_ms = std::chrono::duration<float, std::milli>(std::chrono::steady_clock::now() - t0).count();

    // 2. distinct experts, ascending; slot j <- j-th of them
    int32_t uniq[PGMOE_MAX_EXPERTS];
    int nu = ctx->cfg.n_experts;
    if (all)
        for (int e = 0; e < nu; ++e) uniq[e] = e;
    else
        nu = pgmoe_unique_experts(ctx->idx_staging, n, ctx->cfg.n_experts, uniq);
    if (nu < 0) return fail(ctx, nu, "%s: %s", fn, pgmoe_last_error(nullptr));
    if (nu > ctx->slots) return fail(ctx, PGMOE_ENOSLOT, "%s: %d distinct experts selected but only %d slots per generation", fn, nu, ctx->slots);

    // 3. the generation may still be read by the FFN that used it last
    rc = wait_for_last_reader(ctx, gen, cs, ps);
    if (rc) return rc;
    if (ctx->fetch_timing) PG_HIP(ctx, hipEventRecord(ctx->fetch_begin[block], ps));
    // The copies of one block are dealt to two streams, the one chosen above and the other of the
    // pair (caller's copy stream, the context's own): a copy engine leaves the link idle for a few
    // microseconds between two dependent copies of one stream, and a second queue of copies fills
    // those gaps.  Both streams take every block's copies in block order, so the blocks still
    // arrive one after the other.
    hipStream_t ps2 = ps == ctx->copy2 ? (hipStream_t)copy_stream : ctx->copy2;
    const bool two = !inline_fetch && nu > 1 && ps2 != ps && ps2 != cs;
    if (two) {
        PG_HIP(ctx, hipEventRecord(ctx->fork[gen], ps));  // behind everything ps has waited for
        PG_HIP(ctx, hipStreamWaitEvent(ps2, ctx->fork[gen], 0));
    }
    char *gen_base = ctx->slot_pool + (size_t)gen * ctx->slots * ctx->expert_bytes;
    const char *src_block = ctx->store_base + (size_t)block * ctx->block_stride;
    for (int j = 0; j < nu; ++j)
        PG_HIP(ctx, hipMemcpyAsync(gen_base + (size_t)j * ctx->expert_bytes, src_block + (size_t)uniq[j] * ctx->expert_stride,
                                   ctx->expert_bytes, hipMemcpyHostToDevice, (two && (j & 1)) ? ps2 : ps));
    if (two) {
        PG_HIP(ctx, hipEventRecord(ctx->join[gen], ps2));
        PG_HIP(ctx, hipStreamWaitEvent(ps, ctx->join[gen], 0));
    }
    if (ctx->fetch_timing) PG_HIP(ctx, hipEventRecord(ctx->fetch_end[block], ps));
    if (!inline_fetch) PG_HIP(ctx, hipEventRecord(ctx->fetch_done[gen], ps));

    ctx->fetch_stream[gen] = ps;
    ctx->gen_all[gen] = all;
    ctx->gen_table[gen] = false;
    ctx->fetched_block[gen] = block;
    ctx->live_slots[gen] = nu;
    st.timed = ctx->fetch_timing;
    st.s.n_unique = nu;
    st.s.n_copied = nu;
    st.s.bytes_copied = (int64_t)nu * (int64_t)ctx->expert_bytes;
    // another generation is live only if it holds one of the N blocks that execute before
    // this one (block - N .. block - 1); anything else is left over from an earlier pass
    st.s.resident_slots = nu;
    for (int g = 0; g < ctx->n_gen; ++g)
        if (g != gen && ctx->fetched_block[g] >= block - ctx->distance && ctx->fetched_block[g] < block && ctx->fetched_block[g] >= 0)
            st.s.resident_slots += ctx->live_slots[g];
    if (n_unique_out) *n_unique_out = nu;
    return PGMOE_OK;
}

int pgmoe_fetch_experts(pgmoe_ctx *ctx, int block, const int32_t *topk_idx, int T, void *compute_stream,
                        void *copy_stream, int *n_unique_out) {
    return fetch_impl(ctx, "pgmoe_fetch_experts", block, false, topk_idx, T, compute_stream, copy_stream, n_unique_out);
}

int pgmoe_fetch_all_experts(pgmoe_ctx *ctx, int block, void *compute_stream, void *copy_stream) {
    return fetch_impl(ctx, "pgmoe_fetch_all_experts", block, true, nullptr, 0, compute_stream, copy_stream, nullptr);
}

int pgmoe_fetch_experts_as_turn(pgmoe_ctx *ctx, int block, const int32_t *topk_idx, int T, void *stream, int seq, float wait_us) {
    const char *fn = "pgmoe_fetch_experts_as_turn";
    if (!ctx) return fail(nullptr, PGMOE_EINVAL, "%s: ctx is NULL", fn);
    if (seq < 0 || seq > 4096) return fail(ctx, PGMOE_EINVAL, "%s: seq=%d outside 0..4096", fn, seq);
    if (!(wait_us >= 1.f && wait_us <= 500000.f)) return fail(ctx, PGMOE_EINVAL, "%s: wait_us=%g outside 1..500000", fn, (double)wait_us);
    if (ctx->store_mode != STORE_HOST || !ctx->pull)
        return fail(ctx, PGMOE_ESTATE, "%s: needs a host expert store and the pull engine", fn);
    // an exposed fetch in stream order (compute == copy stream), as migration number seq of a step
    // that has no other migrations: fetch_impl hands seq on to the kernel and the scope guard ends the "step"
    struct Scope {
        pgmoe_ctx *c;
        ~Scope() { c->pull_seq = c->pull_last = -1; c->turn_timeout_ticks = 0; }
    } scope{ctx};
    ctx->pull_seq = seq;
    ctx->pull_last = seq;  // it is also the "step's" last kernel: its last workgroup sets the turn counter back to 0
    ctx->turn_timeout_ticks = (unsigned long long)(wait_us * 100.f);
    return fetch_impl(ctx, fn, block, false, topk_idx, T, stream, stream, nullptr);
}

int pgmoe_set_schedule(pgmoe_ctx *ctx, int schedule) {
    if (!ctx) return fail(nullptr, PGMOE_EINVAL, "pgmoe_set_schedule: ctx is NULL");
    if (schedule < PGMOE_SCHED_PREGATED || schedule > PGMOE_SCHED_PREFETCH_ALL)
        return fail(ctx, PGMOE_EINVAL, "pgmoe_set_schedule: unknown schedule %d", schedule);
    ctx->schedule = schedule;
    return PGMOE_OK;
}

int pgmoe_set_nonmoe_standin(pgmoe_ctx *ctx, float microseconds) {
    if (!ctx) return fail(nullptr, PGMOE_EINVAL, "pgmoe_set_nonmoe_standin: ctx is NULL");
    if (!(microseconds >= 0.f && microseconds <= 100000.f))
        return fail(ctx, PGMOE_EINVAL, "pgmoe_set_nonmoe_standin: %g us outside 0..100000", (double)microseconds);
    ctx->standin_us = microseconds;
    return PGMOE_OK;
}

int pgmoe_get_fetch_stats(pgmoe_ctx *ctx, int block, pgmoe_fetch_stats *out) {
    const char *fn = "pgmoe_get_fetch_stats";
    if (!ctx) return fail(nullptr, PGMOE_EINVAL, "%s: ctx is NULL", fn);
    int rc = check_block(ctx, fn, block);
    if (rc) return rc;
    if (!out) return fail(ctx, PGMOE_EINVAL, "%s: out is NULL", fn);
    BlockStats &st = ctx->stats[block];
    if (!ctx->host_only) {
        if (st.timed) {
            PG_HIP(ctx, hipEventSynchronize(ctx->fetch_end[block]));
            float ms = 0.f;
            PG_HIP(ctx, hipEventElapsedTime(&ms, ctx->fetch_begin[block], ctx->fetch_end[block]));
            st.s.fetch_ms = ms;
        }
        if (st.pulled) {
            // the pull kernel left the distinct-expert counts on the device
            PG_HIP(ctx, hipStreamSynchronize(ctx->fetch_stream[block % ctx->n_gen]));
            // the counts of this block and of the N blocks that execute before it, in one copy
            int32_t u[PGMOE_MAX_PREGATE_DISTANCE + 1] = {};
            const int first = block - ctx->distance > 0 ? block - ctx->distance : 0;
            PG_HIP(ctx, hipMemcpy(u, ctx->dev_unique + first, sizeof(int32_t) * (size_t)(block - first + 1), hipMemcpyDeviceToHost));
            const int32_t u0 = u[block - first];
            int copied = u0 < ctx->slots ? u0 : ctx->slots;
            st.s.n_unique = u0;
            st.s.resident_slots = copied;
            for (int b = block - 1; b >= first; --b) {
                if (!ctx->stats[b].pulled) continue;
                const int32_t ub = u[b - first];
                st.s.resident_slots += ub < ctx->slots ? ub : ctx->slots;
            }
            if (st.cached) {  // unique, copies, hits as the cache-aware kernel counted them
                int32_t cs3[3] = {0, 0, 0};
                PG_HIP(ctx, hipMemcpy(cs3, ctx->cache_stats + (size_t)block * 4, sizeof cs3, hipMemcpyDeviceToHost));
                st.s.n_unique = cs3[0];
                copied = cs3[1];
                st.s.cache_hits = cs3[2];
                st.s.resident_slots = cs3[0];
            }
            st.s.n_copied = copied;
            st.s.bytes_copied = (int64_t)copied * (int64_t)ctx->expert_bytes;
        }
    }
    *out = st.s;
    return PGMOE_OK;
}

int pgmoe_fetch_timing(pgmoe_ctx *ctx, int enable) {
    if (!ctx) return fail(nullptr, PGMOE_EINVAL, "pgmoe_fetch_timing: ctx is NULL");
    ctx->fetch_timing = enable != 0;
    return PGMOE_OK;
}

int pgmoe_trace(pgmoe_ctx *ctx, int enable) {
    if (!ctx) return fail(nullptr, PGMOE_EINVAL, "pgmoe_trace: ctx is NULL");
    ctx->trace = enable != 0;
    ctx->fetch_timing = enable != 0;
    for (int b = 0; ctx->traced && b < ctx->cfg.n_blocks; ++b) ctx->traced[b] = false;
    return PGMOE_OK;
}

int pgmoe_get_block_trace(pgmoe_ctx *ctx, int block, pgmoe_block_trace *out) {
    const char *fn = "pgmoe_get_block_trace";
    if (!ctx) return fail(nullptr, PGMOE_EINVAL, "%s: ctx is NULL", fn);
    int rc = check_block(ctx, fn, block);
    if (rc) return rc;
    if (!out) return fail(ctx, PGMOE_EINVAL, "%s: out is NULL", fn);
    if (ctx->host_only) return fail(ctx, PGMOE_ENODEVICE, "%s: context is host-only", fn);
    if (!ctx->traced || !ctx->traced[block])
        return fail(ctx, PGMOE_ESTATE, "%s: block %d has no trace (tracing on, host store, a stack step run?)", fn, block);
    PG_HIP(ctx, hipEventSynchronize(ctx->ev_c1[block]));
    PG_HIP(ctx, hipEventSynchronize(ctx->fetch_end[block]));
    auto el = [&](hipEvent_t a, hipEvent_t b, float *ms) { return hipEventElapsedTime(ms, a, b); };
    float stall = 0.f, total = 0.f;
    memset(out, 0, sizeof *out);
    PG_HIP(ctx, el(ctx->fetch_begin[block], ctx->fetch_end[block], &out->fetch_ms));
    PG_HIP(ctx, el(ctx->ev_ready[block], ctx->ev_waited[block], &stall));
    PG_HIP(ctx, el(ctx->ev_c0[block], ctx->ev_c1[block], &total));
    PG_HIP(ctx, el(ctx->ev_c0[0], ctx->fetch_begin[block], &out->fetch_start_ms));
    PG_HIP(ctx, el(ctx->ev_c0[0], ctx->fetch_end[block], &out->fetch_end_ms));
    PG_HIP(ctx, el(ctx->ev_c0[0], ctx->ev_c0[block], &out->block_start_ms));
    PG_HIP(ctx, el(ctx->ev_c0[0], ctx->ev_c1[block], &out->block_end_ms));
    // the copy itself: the pull kernel's own clock readings (its duration above includes the wait for
    // its turn on the link); the copy engines have no such wait, their copies span fetch_ms
    out->copy_ms = out->fetch_ms;
    if (ctx->stats[block].pulled) {
        unsigned long long clk[2] = {0, 0};
        PG_HIP(ctx, hipMemcpy(clk, ctx->dev_copy_clock + 2 * (size_t)block, sizeof clk, hipMemcpyDeviceToHost));
        out->copy_ms = clk[1] > clk[0] ? (float)((double)(clk[1] - clk[0]) * 1e-5) : 0.f;  // 100 MHz ticks
    }
    out->stall_ms = stall > 0.f ? stall : 0.f;
    // a fetch on the compute stream itself is waited for in stream order, not at the event wait
    if (ctx->stats[block].in_line) out->stall_ms += out->fetch_ms;
    out->compute_ms = total - out->stall_ms;
    return PGMOE_OK;
}

int pgmoe_slot_address(pgmoe_ctx *ctx, int block, int slot, void **dev_out) {
    const char *fn = "pgmoe_slot_address";
    if (!ctx) return fail(nullptr, PGMOE_EINVAL, "%s: ctx is NULL", fn);
    int rc = check_block(ctx, fn, block);
    if (rc) return rc;
    if (!dev_out) return fail(ctx, PGMOE_EINVAL, "%s: dev_out is NULL", fn);
    if (slot < 0 || slot >= ctx->slots) return fail(ctx, PGMOE_EINVAL, "%s: slot=%d outside 0..%d", fn, slot, ctx->slots - 1);
    if (!ctx->slot_pool) return fail(ctx, PGMOE_ESTATE, "%s: no slot pool (register a host expert store first)", fn);
    *dev_out = ctx->slot_pool + ((size_t)(block % ctx->n_gen) * ctx->slots + slot) * ctx->expert_bytes;
    return PGMOE_OK;
}

// pgmoe_expert_ffn with the option to leave the float32 partial sums unreduced in the workspace
// (keep_partials != NULL; see launch_ffn), which pgmoe_stack_step feeds to the fused combine.
static int expert_ffn_impl(pgmoe_ctx *ctx, int block, const void *x_perm, const int32_t *expert_offsets, int n_rows,
                           void *y_perm, void *workspace, void *stream, int *keep_partials,
                           const int32_t *src_row = nullptr,  // src_row: x_perm holds the un-grouped rows (see launch_ffn)
                           const FusedGate *gate = nullptr, bool *gate_done = nullptr) {  // resident store only (see launch_ffn)
    const char *fn = "pgmoe_expert_ffn";
    if (!ctx) return fail(nullptr, PGMOE_EINVAL, "%s: ctx is NULL", fn);
    int rc = check_block(ctx, fn, block);
    if (rc) return rc;
    const int64_t max_rows = (int64_t)ctx->cfg.max_tokens * ctx->cfg.top_k;
    if (n_rows < 0 || n_rows > max_rows) return fail(ctx, PGMOE_EINVAL, "%s: n_rows=%d outside 0..%lld", fn, n_rows, (long long)max_rows);
    if (!x_perm || !expert_offsets || !y_perm || !workspace) return fail(ctx, PGMOE_EINVAL, "%s: NULL pointer", fn);
    if (!aligned(x_perm, 16) || !aligned(y_perm, 16) || !aligned(expert_offsets, 4) || !aligned(workspace, 256))
        return fail(ctx, PGMOE_EINVAL, "%s: misaligned pointer (x_perm/y_perm 16, expert_offsets 4, workspace 256 bytes)", fn);
    if (ctx->store_mode == STORE_NONE) return fail(ctx, PGMOE_ESTATE, "%s: no expert store registered", fn);
    if (ctx->host_only) return fail(ctx, PGMOE_ENODEVICE, "%s: context is host-only, nothing can be launched", fn);
    hipStream_t s = (hipStream_t)stream;
    if (ctx->store_mode == STORE_RESIDENT)
        return launch_ffn(ctx, ctx->store_base + (size_t)block * ctx->block_stride, ctx->expert_stride, false,
                          ctx->cfg.n_experts, x_perm, expert_offsets, n_rows, y_perm, workspace, s, keep_partials, nullptr,
                          src_row, gate, gate_done);
    const int gen = block % ctx->n_gen;
    if (ctx->fetched_block[gen] != block)
        return fail(ctx, PGMOE_ESTATE, "%s: block %d was not fetched (generation holds block %d)", fn, block, ctx->fetched_block[gen]);
    if (ctx->trace) PG_HIP(ctx, hipEventRecord(ctx->ev_ready[block], s));
    if (ctx->fetch_stream[gen] != s) PG_HIP(ctx, hipStreamWaitEvent(s, ctx->fetch_done[gen], 0));
    if (ctx->trace) PG_HIP(ctx, hipEventRecord(ctx->ev_waited[block], s));
    // a generation filled by pgmoe_fetch_all_experts is indexed by expert id, else by rank
    rc = launch_ffn(ctx, ctx->slot_pool + (size_t)gen * ctx->slots * ctx->expert_bytes, ctx->expert_bytes, !ctx->gen_all[gen],
                    ctx->slots, x_perm, expert_offsets, n_rows, y_perm, workspace, s, keep_partials,
                    ctx->gen_table[gen] ? ctx->dev_table + (size_t)block * PGMOE_MAX_EXPERTS : nullptr, src_row);
    if (rc) return rc;
    ctx->ffn_recorded[gen] = true;
    ctx->ffn_stream[gen] = s;
    return PGMOE_OK;
}

int pgmoe_expert_ffn(pgmoe_ctx *ctx, int block, const void *x_perm, const int32_t *expert_offsets, int n_rows,
                     void *y_perm, void *workspace, void *stream) {
    return expert_ffn_impl(ctx, block, x_perm, expert_offsets, n_rows, y_perm, workspace, stream, nullptr);
}

int pgmoe_expert_ffn_static(pgmoe_ctx *ctx, int block, const void *x_perm, const int32_t *expert_offsets, int n_rows,
                            void *y_perm, void *stream) {
    const char *fn = "pgmoe_expert_ffn_static";
    if (!ctx) return fail(nullptr, PGMOE_EINVAL, "%s: ctx is NULL", fn);
    const int64_t max_rows = (int64_t)ctx->cfg.max_tokens * ctx->cfg.top_k;
    if (n_rows < 0 || n_rows > max_rows) return fail(ctx, PGMOE_EINVAL, "%s: n_rows=%d outside 0..%lld", fn, n_rows, (long long)max_rows);
    const size_t need = ffn_launch_workspace_bytes(ctx->cfg, n_rows);
    if (need > (size_t)PGMOE_STATIC_SCRATCH_BYTES)
        return fail(ctx, PGMOE_EINVAL, "%s: a launch of %d rows needs %zu bytes of scratch, the static buffer has %zu: use pgmoe_expert_ffn "
                    "with a workspace of the caller's", fn, n_rows, need, (size_t)PGMOE_STATIC_SCRATCH_BYTES);
    if (ctx->host_only) {  // no device, no buffer: validate as pgmoe_expert_ffn does, with a stand-in address
        alignas(256) static char host_stand_in[256];
        return expert_ffn_impl(ctx, block, x_perm, expert_offsets, n_rows, y_perm, host_stand_in, stream, nullptr);
    }
    if (!ctx->static_scratch) return fail(ctx, PGMOE_ESTATE, "%s: the static scratch buffer was not resolved at pgmoe_create", fn);
    return expert_ffn_impl(ctx, block, x_perm, expert_offsets, n_rows, y_perm, ctx->static_scratch, stream, nullptr);
}

// Stand-in for the non-MoE layers between two MoE blocks: one wavefront watches the constant
// 100 MHz clock until `ticks` have passed; the loop is also bounded by a fixed number of clock
// reads (each takes well over 10 ns), so the kernel ends in any case.
__global__ void nonmoe_standin_kernel(unsigned long long ticks, unsigned long long max_reads) {
    const unsigned long long t0 = wall_clock64();
    for (unsigned long long i = 0; i < max_reads; ++i)
        if (wall_clock64() - t0 >= ticks) break;
}

static int launch_standin(pgmoe_ctx *ctx, void *stream) {
    if (ctx->standin_us <= 0.f) return PGMOE_OK;
    const unsigned long long ticks = (unsigned long long)(ctx->standin_us * 100.f);  // 100 MHz
    hipLaunchKernelGGL(nonmoe_standin_kernel, dim3(1), dim3(64), 0, (hipStream_t)stream, ticks, ticks * 10ull + 1000ull);
    PG_HIP(ctx, hipGetLastError());
    return PGMOE_OK;
}

// Do kernels on streams a and b run side by side?  One clock-watching kernel of `us` microseconds
// on each, started together: side by side they take about `us`, on a shared hardware queue 2 * us.
static int streams_run_side_by_side(pgmoe_ctx *ctx, hipStream_t a, hipStream_t b, float us, bool *yes) {
    const unsigned long long ticks = (unsigned long long)(us * 100.f);
    *yes = false;
    // a second trial if the first one says no: a host thread that loses the CPU between the two
    // launches looks like a shared queue
    for (int trial = 0; trial < 2 && !*yes; ++trial) {
        PG_HIP(ctx, hipDeviceSynchronize());
        const auto t0 = std::chrono::steady_clock::now();
        hipLaunchKernelGGL(nonmoe_standin_kernel, dim3(1), dim3(64), 0, a, ticks, ticks * 10ull + 1000ull);
        hipLaunchKernelGGL(nonmoe_standin_kernel, dim3(1), dim3(64), 0, b, ticks, ticks * 10ull + 1000ull);
        PG_HIP(ctx, hipGetLastError());
        PG_HIP(ctx, hipStreamSynchronize(a));
        PG_HIP(ctx, hipStreamSynchronize(b));
        const float took = std::chrono::duration<float, std::micro>(std::chrono::steady_clock::now() - t0).count();
        *yes = took < 1.6f * us;
    }
    return PGMOE_OK;
}

int pgmoe_check_streams(pgmoe_ctx *ctx, void *compute_stream, void *copy_stream, int *shared_out) {
    const char *fn = "pgmoe_check_streams";
    if (!ctx) return fail(nullptr, PGMOE_EINVAL, "%s: ctx is NULL", fn);
    if (!shared_out) return fail(ctx, PGMOE_EINVAL, "%s: shared_out is NULL", fn);
    if (ctx->host_only) return fail(ctx, PGMOE_ENODEVICE, "%s: context is host-only, nothing can be launched", fn);
    hipStream_t cs = (hipStream_t)compute_stream, ps = (hipStream_t)copy_stream;
    const float us = 200.f;
    int shared = 0;
    bool ok = true;
    hipLaunchKernelGGL(nonmoe_standin_kernel, dim3(1), dim3(64), 0, cs, 100ull, 2000ull);  // first launch loads the code: not timed
    PG_HIP(ctx, hipGetLastError());
    // the context's own copy stream first: it is replaced until it shares a queue with neither of
    // the caller's streams (the old ones are kept until pgmoe_destroy, so that a new stream does
    // not simply get the queue that was just given back)
    for (int attempt = 0;; ++attempt) {
        shared = 0;
        int rc = streams_run_side_by_side(ctx, cs, ctx->copy2, us, &ok);
        if (rc) return rc;
        if (!ok) shared |= PGMOE_STREAMS_COMPUTE_OWN;
        if (ps != cs) {
            rc = streams_run_side_by_side(ctx, ps, ctx->copy2, us, &ok);
            if (rc) return rc;
            if (!ok) shared |= PGMOE_STREAMS_COPY_OWN;
        }
        if (!shared || attempt == kSpareStreams) break;
        hipStream_t fresh = nullptr;
        PG_HIP(ctx, hipStreamCreateWithFlags(&fresh, hipStreamNonBlocking));
        ctx->spare_streams[attempt] = ctx->copy2;
        ctx->copy2 = fresh;
    }
    if (ps == cs) {
        shared |= PGMOE_STREAMS_COMPUTE_COPY;
    } else {
        int rc = streams_run_side_by_side(ctx, cs, ps, us, &ok);
        if (rc) return rc;
        if (!ok) shared |= PGMOE_STREAMS_COMPUTE_COPY;
    }
    *shared_out = shared;
    return PGMOE_OK;
}

// The gate that routes block g, evaluated on hidden state x, inside pgmoe_stack_step.  For a
// decode-sized bf16 batch the gate kernel also groups block g's tokens by expert (offsets, row_of,
// inverse map) and routed[g] says so; pgmoe_stack_step has validated the buffers.
// finish_routing (bf16 contexts): the call must leave the block fully grouped on `stream`, so the
// grouping kernel follows the gate there when the gate kernel did not do it itself.
static int gate_for_block(pgmoe_ctx *ctx, const pgmoe_step_buffers *io, int g, const void *x, int T, void *stream,
                          bool finish_routing = false) {
    const pgmoe_config &c = ctx->cfg;
    const size_t nk = (size_t)T * c.top_k;
    const float *bias = io->gate_b ? io->gate_b[g] : nullptr;
    if (!aligned(x, 16) || !aligned(io->gate_w[g], 16) || !aligned(bias, 4))
        return fail(ctx, PGMOE_EINVAL, "pgmoe_stack_step: misaligned hidden state, gate weight or bias of block %d", g);
    int32_t *row_of = io->row_of + (size_t)g * nk, *offs = io->expert_offsets + (size_t)g * (c.n_experts + 1);
    int32_t *src_row = ctx->dev_src_row + (size_t)g * c.max_tokens * c.top_k;
    int rc = launch_gate(ctx, x, io->gate_w[g], bias, T, io->topk_idx + (size_t)g * nk, io->topk_prob + (size_t)g * nk, nullptr,
                         (hipStream_t)stream, row_of, offs, src_row, &ctx->routed[g]);
    if (rc || !finish_routing || c.dtype != PGMOE_BF16 || ctx->routed[g]) return rc;
    rc = launch_route(ctx, io->topk_idx + (size_t)g * nk, T, row_of, offs, src_row, (hipStream_t)stream);
    if (rc == PGMOE_OK) ctx->routed[g] = true;
    return rc;
}

// Token grouping and expert FFN of one block inside pgmoe_stack_step.  bf16: only the integer
// half of the grouping runs (offsets, row_of and the inverse map grouped row -> token); the FFN
// kernels read their rows of x through that map, so the gather kernel and the x_perm round trip
// are skipped (same values, hence the same results as pgmoe_permute + pgmoe_expert_ffn).
static int group_and_run_experts(pgmoe_ctx *ctx, const pgmoe_step_buffers *io, int block, int T, const void *x,
                                 const int32_t *idx, int32_t *row_of, int32_t *offs, void *stream, int *n_partial,
                                 const FusedGate *gate = nullptr, bool *gate_done = nullptr) {
    const int nk = T * ctx->cfg.top_k;
    if (gate_done) *gate_done = false;
    if (ctx->cfg.dtype != PGMOE_BF16) {
        int rc = pgmoe_permute(ctx, x, idx, T, io->x_perm, row_of, offs, stream);
        if (rc) return rc;
        return expert_ffn_impl(ctx, block, io->x_perm, offs, nk, io->y_perm, io->workspace, stream, n_partial);
    }
    int32_t *src_row = ctx->dev_src_row + (size_t)block * ctx->cfg.max_tokens * ctx->cfg.top_k;
    if (!ctx->routed[block]) {  // the gate kernel that routed this block did not group its tokens itself
        int rc = launch_route(ctx, idx, T, row_of, offs, src_row, (hipStream_t)stream);
        if (rc) return rc;
    }
    return expert_ffn_impl(ctx, block, x, offs, nk, io->y_perm, io->workspace, stream, n_partial, src_row, gate, gate_done);
}

int pgmoe_stack_step(pgmoe_ctx *ctx, const pgmoe_step_buffers *io, int T, void *compute_stream, void *copy_stream) {
    const char *fn = "pgmoe_stack_step";
    if (!ctx) return fail(nullptr, PGMOE_EINVAL, "%s: ctx is NULL", fn);
    if (!io) return fail(ctx, PGMOE_EINVAL, "%s: io is NULL", fn);
    if (T < 0 || T > ctx->cfg.max_tokens) return fail(ctx, PGMOE_EINVAL, "%s: T=%d outside 0..max_tokens=%d", fn, T, ctx->cfg.max_tokens);
    if (!io->gate_w || !io->x_states || !io->topk_idx || !io->topk_prob || !io->row_of || !io->expert_offsets ||
        !io->x_perm || !io->y_perm || !io->workspace)
        return fail(ctx, PGMOE_EINVAL, "%s: a required buffer is NULL", fn);
    if (!aligned(io->x_states, 16) || !aligned(io->x_perm, 16) || !aligned(io->y_perm, 16) || !aligned(io->workspace, 256) ||
        !aligned(io->topk_idx, 4) || !aligned(io->topk_prob, 4) || !aligned(io->row_of, 4) || !aligned(io->expert_offsets, 4) ||
        !aligned(io->y_blocks, 16))
        return fail(ctx, PGMOE_EINVAL, "%s: misaligned buffer (activations 16, workspace 256, index arrays 4 bytes)", fn);
    const pgmoe_config &c = ctx->cfg;
    const int L = c.n_blocks;
    for (int g = 0; g < L; ++g)
        if (!io->gate_w[g]) return fail(ctx, PGMOE_EINVAL, "%s: gate_w[%d] is NULL", fn, g);
    if (ctx->store_mode == STORE_NONE) return fail(ctx, PGMOE_ESTATE, "%s: no expert store registered", fn);
    if (ctx->host_only) return fail(ctx, PGMOE_ENODEVICE, "%s: context is host-only, nothing can be launched", fn);
    if (T == 0) return PGMOE_OK;
    for (int b = 0; b < L; ++b) ctx->routed[b] = false;
    // the migrations of this step that run beside the compute stream (one per block in the pre-gated
    // and the prefetch-all schedule) take turns on the host link; whatever path leaves this
    // function, later stand-alone fetches are not part of a step
    struct StepScope {
        pgmoe_ctx *c;
        ~StepScope() { c->pull_seq = c->pull_last = -1; }
    } step_scope{ctx};
    if (ctx->store_mode == STORE_HOST && ctx->pull && ctx->schedule != PGMOE_SCHED_ON_DEMAND && copy_stream != compute_stream) {
        ctx->pull_seq = 0;
        ctx->pull_last = L - 1;
    }

    const size_t xbytes = (size_t)T * c.d_model * ctx->elem;
    const size_t nk = (size_t)T * c.top_k;
    auto x_at = [&](int i) { return (char *)io->x_states + (size_t)i * xbytes; };
    auto idx_at = [&](int i) { return io->topk_idx + (size_t)i * nk; };
    auto prob_at = [&](int i) { return io->topk_prob + (size_t)i * nk; };
    int rc;

    if (ctx->schedule != PGMOE_SCHED_PREGATED) {
        // Conventional MoE wiring (Sec. II-B; the paper's comparison systems of Sec. III / Fig.
        // "timeline"): gate g routes block g from the block's own input.  ON_DEMAND migrates the
        // selected experts after the gate, serially; PREFETCH_ALL migrates every expert of block
        // i+1 while block i executes.  With a resident store both are the GPU-only design point.
        const bool host = ctx->store_mode == STORE_HOST;
        const bool prefetch = ctx->schedule == PGMOE_SCHED_PREFETCH_ALL;
        if (host && prefetch) {
            rc = pgmoe_fetch_all_experts(ctx, 0, compute_stream, copy_stream);
            if (rc) return rc;
        }
        for (int i = 0; i < L; ++i) {
            if (ctx->trace) PG_HIP(ctx, hipEventRecord(ctx->ev_c0[i], (hipStream_t)compute_stream));
            rc = gate_for_block(ctx, io, i, x_at(i), T, compute_stream);
            if (rc) return rc;
            if (host && !prefetch) {
                rc = pgmoe_fetch_experts(ctx, i, idx_at(i), T, compute_stream, ctx->pull ? compute_stream : copy_stream, nullptr);
                if (rc) return rc;
            }
            if (host && prefetch && i + 1 < L) {
                rc = pgmoe_fetch_all_experts(ctx, i + 1, compute_stream, copy_stream);
                if (rc) return rc;
            }
            int32_t *row_of = io->row_of + (size_t)i * nk;
            int32_t *offs = io->expert_offsets + (size_t)i * (c.n_experts + 1);
            int n_partial = 0;
            rc = group_and_run_experts(ctx, io, i, T, x_at(i), idx_at(i), row_of, offs, compute_stream, &n_partial);
            if (rc) return rc;
            void *y = io->y_blocks ? (char *)io->y_blocks + (size_t)i * xbytes : nullptr;
            if (n_partial > 0)
                rc = launch_combine_partials(ctx, (const float *)io->workspace, n_partial, (int)nk, row_of, prob_at(i), T, y,
                                             x_at(i), x_at(i + 1), (hipStream_t)compute_stream);
            else
                rc = pgmoe_combine(ctx, io->y_perm, row_of, prob_at(i), T, y, x_at(i), x_at(i + 1), compute_stream);
            if (rc) return rc;
            rc = launch_standin(ctx, compute_stream);
            if (rc) return rc;
            if (ctx->trace) {
                PG_HIP(ctx, hipEventRecord(ctx->ev_c1[i], (hipStream_t)compute_stream));
                ctx->traced[i] = host && ctx->fetch_timing;
            }
        }
        return PGMOE_OK;
    }

    if (ctx->trace) PG_HIP(ctx, hipEventRecord(ctx->ev_c0[0], (hipStream_t)compute_stream));
    // Block 0: its own (conventional) gate and, on the same input, the pre-gates of blocks
    // 1..N (N = pre-gate distance, 1 in the paper's design).  All these routings are known
    // before anything can execute, so block 0's exposed fetch and the fetches of blocks 1..N are
    // queued back to back on the copy stream: the link never idles between them.
    const int N = ctx->distance;
    const int head = std::min(N, L - 1);
    // Resident store, pre-gate distance 1: nothing waits for a routing, so the pre-gate evaluated
    // on x_i is offered to block i's expert launch, which carries it as one extra workgroup when
    // it is a decode-sized launch with one of the smallest gates (one launch fewer per block);
    // a launch that cannot leaves it to a gate launch of its own right behind it.
    const bool carry_gate = ctx->store_mode == STORE_RESIDENT && N == 1 && c.dtype == PGMOE_BF16;
    if (ctx->pull_seq >= 0 && c.dtype == PGMOE_BF16) {
        // Block 0's fetch is exposed whatever is done, so it runs on the compute stream itself,
        // right behind its gate: no stream hand-over (11-13 us) before the link starts working,
        // and none before block 0's experts either.  Block 1's pre-gate and fetch go to the
        // context's own copy stream together (stream order between them); that stream only has to
        // be behind the start of this step, where x_0 is in place, block 1's buffers are free and
        // the last reader of block 1's slot generation (an FFN of the previous step) is queued.
        hipStream_t cs = (hipStream_t)compute_stream;
        if (L > 1) {
            PG_HIP(ctx, hipEventRecord(ctx->step_start, cs));
            PG_HIP(ctx, hipStreamWaitEvent(ctx->copy2, ctx->step_start, 0));
        }
        rc = gate_for_block(ctx, io, 0, x_at(0), T, compute_stream);
        if (rc) return rc;
        rc = pgmoe_fetch_experts(ctx, 0, idx_at(0), T, compute_stream, compute_stream, nullptr);  // takes turn 0
        if (rc) return rc;
        if (L > 1) {
            rc = gate_for_block(ctx, io, 1, x_at(0), T, ctx->copy2, /*finish_routing=*/true);
            if (rc) return rc;
            ctx->routed_on_copy_stream = true;  // turn 1 is odd: the fetch goes to the same stream
            rc = pgmoe_fetch_experts(ctx, 1, idx_at(1), T, compute_stream, copy_stream, nullptr);
            ctx->routed_on_copy_stream = false;
            if (rc) return rc;
        }
        // blocks 2..N (pre-gate distance N > 1) are routed from x_0 as well; their gates queue on the
        // compute stream behind block 0's migration, early enough: their turn on the link comes
        // only after blocks 0 and 1 have been copied
        for (int g = 2; g <= head; ++g) {
            rc = gate_for_block(ctx, io, g, x_at(0), T, compute_stream);
            if (rc) return rc;
            rc = pgmoe_fetch_experts(ctx, g, idx_at(g), T, compute_stream, copy_stream, nullptr);
            if (rc) return rc;
        }
    } else {
        for (int g = 0; g <= (carry_gate ? 0 : head); ++g) {
            rc = gate_for_block(ctx, io, g, x_at(0), T, compute_stream);
            if (rc) return rc;
            rc = pgmoe_fetch_experts(ctx, g, idx_at(g), T, compute_stream, copy_stream, nullptr);
            if (rc) return rc;
        }
    }

    for (int i = 0; i < L; ++i) {
        if (ctx->trace && i > 0) PG_HIP(ctx, hipEventRecord(ctx->ev_c0[i], (hipStream_t)compute_stream));
        // the pre-gate of block i routes block i+N; its experts start moving before block i executes
        if (!carry_gate && i > 0 && i + N < L) {
            const int g = i + N;
            rc = gate_for_block(ctx, io, g, x_at(i), T, compute_stream);
            if (rc) return rc;
            rc = pgmoe_fetch_experts(ctx, g, idx_at(g), T, compute_stream, copy_stream, nullptr);
            if (rc) return rc;
        }
        int32_t *row_of = io->row_of + (size_t)i * nk;
        int32_t *offs = io->expert_offsets + (size_t)i * (c.n_experts + 1);
        // grouping + FFN, then the weighted combine; when the FFN left float32 partial sums, the
        // combine kernel adds them itself (same order as the stand-alone reduction) and y_perm is skipped
        int n_partial = 0;
        const int g = i + N;
        if (carry_gate && g < L) {
            const float *bias = io->gate_b ? io->gate_b[g] : nullptr;
            if (!aligned(x_at(i), 16) || !aligned(io->gate_w[g], 16) || !aligned(bias, 4))
                return fail(ctx, PGMOE_EINVAL, "%s: misaligned hidden state, gate weight or bias of block %d", fn, g);
            const FusedGate fg = {x_at(i), io->gate_w[g], bias, T, idx_at(g), prob_at(g), io->row_of + (size_t)g * nk,
                                  io->expert_offsets + (size_t)g * (c.n_experts + 1),
                                  ctx->dev_src_row + (size_t)g * c.max_tokens * c.top_k};
            bool carried = false;
            rc = group_and_run_experts(ctx, io, i, T, x_at(i), idx_at(i), row_of, offs, compute_stream, &n_partial, &fg, &carried);
            if (rc) return rc;
            if (carried) ctx->routed[g] = true;  // the smallest-gate code groups the tokens as well
            else rc = gate_for_block(ctx, io, g, x_at(i), T, compute_stream);
        } else {
            rc = group_and_run_experts(ctx, io, i, T, x_at(i), idx_at(i), row_of, offs, compute_stream, &n_partial);
        }
        if (rc) return rc;
        void *y = io->y_blocks ? (char *)io->y_blocks + (size_t)i * xbytes : nullptr;
        if (n_partial > 0)
            rc = launch_combine_partials(ctx, (const float *)io->workspace, n_partial, (int)nk, row_of, prob_at(i), T, y,
                                         x_at(i), x_at(i + 1), (hipStream_t)compute_stream);
        else
            rc = pgmoe_combine(ctx, io->y_perm, row_of, prob_at(i), T, y, x_at(i), x_at(i + 1), compute_stream);
        if (rc) return rc;
        rc = launch_standin(ctx, compute_stream);
        if (rc) return rc;
        if (ctx->trace) {
            PG_HIP(ctx, hipEventRecord(ctx->ev_c1[i], (hipStream_t)compute_stream));
            ctx->traced[i] = ctx->store_mode == STORE_HOST && ctx->fetch_timing;
        }
    }
    return PGMOE_OK;
}

}  // extern "C"
