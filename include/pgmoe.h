/*
 * pgmoe.h - C ABI of libpgmoe: the per-layer sparse MoE block of Pre-gated MoE
 * (arXiv 2308.12066) on one AMD MI355X (gfx950).
 *
 * What the library computes, per MoE block i of a stack of L blocks (Sec. II-B for the
 * block, Sec. IV-B for the pre-gate wiring, Sec. IV-C for the migration):
 *   1. a gate scores all E experts for every token (softmax over x.W) and the k best are
 *      activated.  The gate that sits in block i is a PRE-gate: its result routes block i+1.
 *      Block 0 additionally carries a conventional gate for itself; the last block has none.
 *   2. only the activated experts of block i+1 are copied from pinned host memory into HBM,
 *      on a copy stream, while block i executes (preemptive expert migration).  At most two
 *      blocks' activated experts are resident (the peak-memory rule of Sec. IV-C).
 *   3. block i's activated experts, each a dense FFN ReLU(x.W1).W2, process the tokens
 *      routed to them, and each token's output is the sum over its experts of
 *      (gate probability) x (expert output).
 *
 * Conventions
 *   - Every function returns 0 on success or a negative pgmoe_status; pgmoe_last_error()
 *     gives the text.  Arguments are validated before anything is launched.
 *   - "dev" pointers are device (HBM) addresses, "host" pointers ordinary host addresses,
 *     "pinned" host memory obtained from hipHostMalloc.  The caller owns every buffer it
 *     passes and keeps it alive until the stream work that uses it has completed.  The
 *     library owns only the context: the expert slot pool, events and a small pinned
 *     staging area.  Allocation happens in set-up calls only: pgmoe_create() (flags, maps,
 *     events, staging), the first pgmoe_register_host_experts() on a context (slot pool and,
 *     if configured, the expert cache), pgmoe_check_streams() (may create streams) and
 *     pgmoe_ffn_timing_begin() (its events).  The calls of the hot path (pgmoe_pregate_topk,
 *     pgmoe_fetch_experts, pgmoe_permute, pgmoe_expert_ffn, pgmoe_combine, pgmoe_stack_step)
 *     allocate nothing.
 *   - Streams are hipStream_t passed as void* (NULL = the default stream).  All device work
 *     is asynchronous on the given stream, except that pgmoe_fetch_experts() waits until the
 *     routing indices have reached the host (it must read them to issue the copies).
 *   - Matrices are row-major.  T = tokens in this call, d = d_model, f = d_ff, E = n_experts,
 *     k = top_k.  Activations and gate weights have the context's dtype (float32 or
 *     bfloat16); probabilities are float32; indices are int32.  T = 0 is a valid no-op.
 *   - One context serves one stack on one device, from one host thread at a time.
 */
#ifndef PGMOE_H
#define PGMOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct pgmoe_ctx pgmoe_ctx;

typedef enum {
    PGMOE_OK = 0,
    PGMOE_EINVAL = -1,     /* null/misaligned pointer, size out of range, k > E, bad block ... */
    PGMOE_ENOTPINNED = -2, /* host expert store is not pinned host memory */
    PGMOE_ENOSLOT = -3,    /* more distinct experts selected than slots_per_gen */
    PGMOE_EBADINDEX = -4,  /* an expert index outside [0, E) was seen on the host */
    PGMOE_EHIP = -5,       /* a HIP runtime call failed (text has the HIP error) */
    PGMOE_ENODEVICE = -6,  /* context was created host-only, or no GPU is present */
    PGMOE_ESTATE = -7      /* call order violated (e.g. FFN of a block that was never fetched) */
} pgmoe_status;

typedef enum { PGMOE_F32 = 0, PGMOE_BF16 = 1 } pgmoe_dtype;

/* Bits of pgmoe_config.flags */
#define PGMOE_FLAG_HOST_ONLY 1u /* create no device resources: argument checks and host logic
                                   work, every launch returns PGMOE_ENODEVICE */

#define PGMOE_FLAG_FETCH_MEMCPY 2u /* migrate experts with hipMemcpyAsync (one per expert, issued
                                      by the host after it has read the routing indices back)
                                      instead of the default device-side pull kernel */

#define PGMOE_FLAG_FETCH_AUTO 4u   /* let pgmoe_create pick the migration engine from the configuration: the
                                      copy engines (as PGMOE_FLAG_FETCH_MEMCPY) when one block's migration can
                                      reach PGMOE_AUTO_COPY_ENGINE_BYTES (slots_per_gen * expert bytes) and no
                                      expert cache is configured, the pull kernel otherwise.  Why: the pull
                                      kernel needs no host round trip and keeps the link busier (it wins by
                                      5 % at one 9.4 MB expert per block, by 0.6 % at 25 experts of 16.8 MB),
                                      but its host-link loads slow every kernel that reads HBM beside it (an
                                      expert FFN by 1.5x, a plain read by 2.7x); copy-engine traffic does not
                                      (1.08x).  pgmoe_migration_engine() tells which one a context uses. */
#define PGMOE_AUTO_COPY_ENGINE_BYTES ((size_t)256 << 20)

#define PGMOE_MAX_EXPERTS 256 /* the paper's largest model has 256 experts per block */

typedef struct {
    int32_t d_model;       /* bf16: 64, 128, 256, 512, 768, 1024 or 2048 (the sizes expert kernels are
                              built for; pack/unpack take any multiple of 64); f32: any >= 1 */
    int32_t d_ff;          /* bf16: multiple of 64 */
    int32_t n_experts;     /* 1 .. PGMOE_MAX_EXPERTS */
    int32_t top_k;         /* 1 .. n_experts */
    int32_t n_blocks;      /* L >= 1 */
    int32_t max_tokens;    /* largest T of any call */
    int32_t dtype;         /* pgmoe_dtype of activations, gate weights and expert weights */
    int32_t slots_per_gen; /* expert slots per block generation; 0 => min(E, max_tokens*k),
                              which can never overflow.  Ignored without a host store.  On a context
                              that migrates with the pull kernel, (slots + cache_slots) * expert bytes
                              must stay below 64 GiB (32-bit unit numbers in the pull kernels). */
    uint32_t flags;
    int32_t cache_slots;   /* expert cache on top of the migration (Sec. VI "Caching experts"): slots
                              per block that keep experts in HBM across steps; 0 = no cache (the
                              base design), at most PGMOE_MAX_CACHE_SLOTS.  Pull mode only. */
    int32_t cache_policy;  /* pgmoe_cache_policy: which cached expert a missing one replaces */
    int32_t pregate_distance; /* N of Sec. VI-D "pre-gating to activate experts at different blocks":
                              the pre-gate evaluated on x_i routes block i+N, so block i is routed
                              from x_{max(0, i-N)} and N+1 block generations of experts are
                              resident.  0 or 1 = the paper's default (next block); at most
                              PGMOE_MAX_PREGATE_DISTANCE.  Used by pgmoe_stack_step with
                              PGMOE_SCHED_PREGATED and by the slot pool's size. */
} pgmoe_config;
#define PGMOE_MAX_PREGATE_DISTANCE 3

/* Replacement policies the paper evaluates.  A slot whose expert is used by the current fetch
 * is never a victim; empty slots are filled first (lowest index); ties go to the lowest slot.
 *   LRU  victim = least recently used;
 *   LFU  victim = least often used (then least recently used);
 *   LIFO victim = most recently inserted. */
typedef enum { PGMOE_CACHE_LRU = 0, PGMOE_CACHE_LFU = 1, PGMOE_CACHE_LIFO = 2 } pgmoe_cache_policy;
#define PGMOE_MAX_CACHE_SLOTS 64

/* Counters of the last pgmoe_fetch_experts() for a block (host). */
typedef struct {
    int32_t n_unique;       /* distinct experts selected */
    int32_t n_copied;       /* experts actually copied (== n_unique in the base design) */
    int64_t bytes_copied;   /* n_copied * expert_bytes */
    int32_t resident_slots; /* slots holding live experts over all generations right after
                               this fetch was issued: the quantity the peak-memory rule bounds
                               (cache slots, when a cache is configured, come on top) */
    int32_t cache_hits;     /* selected experts found in the block's cache (0 without a cache) */
    float fetch_ms;         /* copy-stream time of the batch; 0 unless pgmoe_fetch_timing() is on */
    float wait_ms;          /* host time spent waiting for the indices (memcpy mode) */
} pgmoe_fetch_stats;

/* ---- context ---------------------------------------------------------------------- */
int pgmoe_create(pgmoe_ctx **out, const pgmoe_config *cfg);
int pgmoe_destroy(pgmoe_ctx *ctx);
/* Text of the last error on this context (ctx == NULL: last error of a failed create or of
 * a context-free call on this thread).  Never NULL; owned by the library. */
const char *pgmoe_last_error(const pgmoe_ctx *ctx);

/* Bytes of one expert blob (W1 then W2, contiguous): 2*d*f*sizeof(element). 0 if cfg invalid. */
size_t pgmoe_expert_bytes(const pgmoe_config *cfg);
/* Bytes of device scratch that pgmoe_expert_ffn() needs for up to max_tokens*k rows. */
size_t pgmoe_workspace_bytes(const pgmoe_ctx *ctx);

/* ---- expert weight layout (host) --------------------------------------------------
 * An expert is handed to the library as one blob of pgmoe_expert_bytes().
 *   f32 : W1 [d,f] row-major followed by W2 [f,d] row-major.
 *   bf16: both matrices are stored as 32x16 (k x n) tiles of 512 elements so that one
 *         64-lane load instruction fetches one matrix-core operand: element (k, n) of a
 *         [K, N] matrix sits in tile (kt = k/32, nt = n/16) at in-tile position
 *         ((n%16) + 16*((k%32)/8))*8 + k%8.  W1 (K=d, N=f) orders its tiles nt-major
 *         (tile index nt*(K/32) + kt), W2 (K=f, N=d) kt-major (tile index kt*(N/16) + nt).
 * pack/unpack convert between the logical row-major matrices and the blob; they are pure
 * permutations (bit-exact, unpack(pack(W)) == W).  All pointers host. */
int pgmoe_pack_expert(const pgmoe_config *cfg, const void *w1, const void *w2, void *blob);
int pgmoe_unpack_expert(const pgmoe_config *cfg, const void *blob, void *w1, void *w2);

/* ---- a-1: gate / pre-gate (Sec. II-B gate; Sec. IV-B pre-gate) ----------------------
 * z = x.w_gate (+ bias); p = softmax over the E experts; the k largest z are selected, in
 * descending order, equal values to the lowest index; a NaN logit ranks as -infinity.
 *   x         dev [T,d]   ctx dtype      w_gate dev [d,E] ctx dtype     bias dev [E] f32 | NULL
 *   topk_idx  dev [T,k]   int32 out      topk_prob dev [T,k] f32 out: p at the selected
 *             experts, NOT renormalised  probs_out dev [T,E] f32 out | NULL (full softmax)
 * Arithmetic: float32 accumulation and softmax.  The same call serves block 0's
 * conventional gate and every pre-gate; which block its result routes is the caller's
 * wiring (pgmoe_stack_step implements the paper's). */
int pgmoe_pregate_topk(pgmoe_ctx *ctx, const void *x, const void *w_gate, const float *bias, int T,
                       int32_t *topk_idx, float *topk_prob, float *probs_out, void *stream);

/* ---- a-2: expert store and migration (Sec. IV-C) ------------------------------------
 * Host store: blob of (block b, expert e) at host_base + b*block_stride + e*expert_stride,
 * pinned.  Resident store: the same addressing in device memory (the GPU-only design point:
 * nothing is migrated).  Exactly one of the two is active; registering one replaces the
 * other.  Strides are multiples of 256 bytes and >= pgmoe_expert_bytes(). */
int pgmoe_register_host_experts(pgmoe_ctx *ctx, const void *host_base, size_t expert_stride,
                                size_t block_stride);
int pgmoe_register_resident_experts(pgmoe_ctx *ctx, const void *dev_base, size_t expert_stride,
                                    size_t block_stride);
/* Copy the experts that `topk_idx` (dev [T,k], produced on compute_stream) selects for
 * `block` into that block's slot generation (block mod (pregate_distance + 1)).  The j-th
 * smallest selected expert id goes to slot j.  Blocks 0..N (N = pregate_distance) are copied
 * on copy_stream; from block N+1 on the blocks alternate between a second copy stream the
 * context owns and copy_stream (so that consecutive blocks' migrations do not queue behind
 * each other); passing copy_stream == compute_stream instead runs the copy in plain stream order on
 * compute_stream (an exposed fetch, as block 0's).  The copy first waits for compute_stream to
 * have produced the indices and for the FFN that last used this generation (block-N-1, or the
 * previous step's) to have finished; pgmoe_expert_ffn(block) waits for the copy.
 *   default (pull) mode : one kernel on copy_stream reads the indices, forms the distinct
 *       expert list and pulls the blobs out of the pinned host store over the host link.
 *       Nothing waits on the host: the call returns at once unless n_unique_out is given, in
 *       which case it blocks until the copy has finished and returns the count.
 *   PGMOE_FLAG_FETCH_MEMCPY (or PGMOE_FLAG_FETCH_AUTO on a context it gave the copy engines):
 *       the host waits for the indices (small D2H copy), dedupes them and issues one
 *       hipMemcpyAsync per distinct expert, dealt to two streams (copy_stream and the context's
 *       own) so that one queue of copies fills the gaps the other leaves between two copies;
 *       both streams take the blocks in order.
 * If more distinct experts are selected than slots_per_gen, memcpy mode returns
 * PGMOE_ENOSLOT; pull mode copies the first slots_per_gen of them, sets device flag bit 2 and
 * the FFN skips the rows of the others (their output rows are zero).
 * With an expert cache (cache_slots > 0) a selected expert that is still cached is not
 * copied; a missing one replaces a victim chosen by cache_policy and is copied straight into
 * that cache slot, or into the generation's slots when every cache slot is in use by this
 * fetch.  The FFN then finds each expert through a per-block pointer table the fetch wrote.
 * With a resident store the call only validates and returns n_unique = -1.
 * n_unique_out host | NULL. */
int pgmoe_fetch_experts(pgmoe_ctx *ctx, int block, const int32_t *topk_idx, int T,
                        void *compute_stream, void *copy_stream, int *n_unique_out);
/* Copy EVERY expert of `block` into the block's generation, slot = expert id (what the
 * prefetch-all comparison system of the paper migrates; Sec. III "Prefetch-all").  Needs
 * slots_per_gen == n_experts.  Ordering as pgmoe_fetch_experts, except that there are no
 * indices to wait for: the copy is ordered behind everything queued on compute_stream so far. */
int pgmoe_fetch_all_experts(pgmoe_ctx *ctx, int block, void *compute_stream, void *copy_stream);
int pgmoe_get_fetch_stats(pgmoe_ctx *ctx, int block, pgmoe_fetch_stats *out /* host */);
/* The migration engine of this context: 0 = device-side pull kernel, 1 = copy engines
 * (hipMemcpyAsync issued by the host); negative status if ctx is NULL. */
int pgmoe_migration_engine(const pgmoe_ctx *ctx);
/* Bracket every following fetch with a pair of timing events on the copy stream (fetch_ms of
 * pgmoe_fetch_stats).  Off by default: each event record costs microseconds between the
 * migration kernels of consecutive blocks. */
int pgmoe_fetch_timing(pgmoe_ctx *ctx, int enable);
/* Device address of slot `slot` of the generation that serves `block` (for inspection: after
 * the fetch of `block` has completed it holds the blob of the slot-th smallest selected
 * expert).  dev_out host. */
int pgmoe_slot_address(pgmoe_ctx *ctx, int block, int slot, void **dev_out);

/* Test hook for the bounded wait of the pull engine.  Inside pgmoe_stack_step the migration
 * kernels of a step take turns on the host link: kernel number seq starts copying when the seq
 * kernels before it have passed the turn on, or when its wait has lasted half a second (the
 * wait orders link traffic only; no result depends on it).  This call runs the migration of
 * `block` on `stream`, in stream order, as kernel number seq of a step that has no other
 * kernels, with the wait bounded by wait_us microseconds (1 .. 500000) instead: nobody passes
 * the turn on, so for seq > 0 the kernel waits that long, gives up, copies and leaves normally.
 * Otherwise as pgmoe_fetch_experts(ctx, block, topk_idx, T, stream, stream, NULL).  Pull engine
 * and host store only (PGMOE_ESTATE otherwise). */
int pgmoe_fetch_experts_as_turn(pgmoe_ctx *ctx, int block, const int32_t *topk_idx, int T, void *stream,
                                int seq, float wait_us);

/* Host-only helper used by the fetch engine, exported for testing: ascending list of the
 * distinct values of idx[0..n) (all must lie in [0, E)); returns their number or a negative
 * status.  unique_out host [min(E, n)]. */
int pgmoe_unique_experts(const int32_t *idx /* host */, int n, int E, int32_t *unique_out);

/* ---- a-3: group tokens by expert (Sec. II-B: an expert processes the tokens routed to it)
 * Entry n = t*k + j is token t's j-th selection.  counts[e] = entries routed to e;
 * expert_offsets = exclusive prefix sum (E+1 values, last = T*k); row_of[n] = offsets[e] +
 * number of earlier entries with the same expert (stable); x_perm[row_of[n]] = x[t].
 *   x dev [T,d]; topk_idx dev [T,k]; x_perm dev [T*k,d] out; row_of dev [T*k] int32 out;
 *   expert_offsets dev [E+1] int32 out.  An index outside [0,E) is clamped into range for
 *   addressing and flagged: pgmoe_device_flags() reports it. */
int pgmoe_permute(pgmoe_ctx *ctx, const void *x, const int32_t *topk_idx, int T, void *x_perm,
                  int32_t *row_of, int32_t *expert_offsets, void *stream);

/* ---- a-4: expert FFN -----------------------------------------------------------------
 * For every expert e with rows [expert_offsets[e], expert_offsets[e+1]) of x_perm:
 * y_perm[rows] = ReLU(x_perm[rows].W1_e).W2_e, weights taken from `block`'s slot generation
 * (slot = rank of e among the experts with at least one row) or from the resident store.
 * bf16: products on the matrix cores with float32 accumulation, the hidden activation
 * rounded to bf16 between the two products; f32: float32 throughout.
 *   x_perm dev [n_rows,d]; expert_offsets dev [E+1]; y_perm dev [n_rows,d] out;
 *   workspace dev, pgmoe_workspace_bytes(), 256-byte aligned; n_rows = T*k <= max_tokens*k.
 * With a host store the call first makes `stream` wait for the fetch of `block`
 * (PGMOE_ESTATE if none was issued) and afterwards records the event that guards the slots'
 * reuse. */
int pgmoe_expert_ffn(pgmoe_ctx *ctx, int block, const void *x_perm, const int32_t *expert_offsets,
                     int n_rows, void *y_perm, void *workspace, void *stream);

/* ---- for callers that cannot allocate ----------------------------------------------------
 * pgmoe_expert_ffn() for code under HIP graph capture, tight serving loops and harnesses that
 * forbid hipMalloc: same operation, same results bit for bit, but the float32 partial sums (for
 * launches with hundreds of rows per expert also the packed hidden activation) go to a buffer
 * of PGMOE_STATIC_SCRATCH_BYTES that is part of the library's device image instead of a
 * workspace the caller had to allocate.  Every GPU the library runs on holds one such buffer
 * from the moment the library is loaded there until the process ends.  The call allocates
 * nothing (no hipMalloc / hipFree, no allocating library routine) and otherwise behaves as
 * pgmoe_expert_ffn() (same arguments without `workspace`, same waits and events).
 *   - A launch that needs more scratch than the buffer holds is refused with PGMOE_EINVAL and a
 *     text that names both sizes (decode-sized launches need a few MiB; 4096 rows over 128
 *     experts would need 201 MB: use pgmoe_expert_ffn with a workspace there).
 *   - All calls on one GPU, from every context, share the buffer and it keeps the last call's
 *     contents: nothing in it has to start at zero (every partial sum that is read was written
 *     by the same call), but two calls whose stream work overlaps on one GPU race.  Calls on
 *     one stream, or otherwise ordered, are safe. */
#define PGMOE_STATIC_SCRATCH_BYTES (32u << 20)
int pgmoe_expert_ffn_static(pgmoe_ctx *ctx, int block, const void *x_perm, const int32_t *expert_offsets,
                            int n_rows, void *y_perm, void *stream);

/* ---- a-5: weighted combine -------------------------------------------------------------
 * y[t] = sum_{j<k} topk_prob[t,j] * y_perm[row_of[t*k+j]]  (gather form, no atomics, float32
 * accumulation, stored in ctx dtype).  If x_res and x_next are given, additionally
 * x_next[t] = x_res[t] + (that sum), rounded once: the residual stand-in for the non-MoE
 * layers between two MoE blocks.  y may be NULL when x_next is given.
 *   y_perm dev [T*k,d]; row_of dev [T*k]; topk_prob dev [T,k]; y dev [T,d] out | NULL;
 *   x_res dev [T,d] | NULL; x_next dev [T,d] out | NULL. */
int pgmoe_combine(pgmoe_ctx *ctx, const void *y_perm, const int32_t *row_of, const float *topk_prob,
                  int T, void *y, const void *x_res, void *x_next, void *stream);

/* ---- a-6: one pass of the whole stack (Sec. IV-B wiring + Sec. IV-C overlap) ------------
 * Runs blocks 0..L-1 for one batch of T tokens:
 *   block 0   : conventional gate and pre-gate 0 on x_0 -> fetch(0) (exposed), fetch(1) behind it
 *   block i   : [pre-gate i on x_i -> fetch(i+1) on the copy stream]  ||  permute, FFN_i,
 *               combine on the compute stream, x_{i+1} = x_i + y_i
 *   block L-1 : no gate.
 * gate_w[0] / gate_b[0] is block 0's conventional gate, gate_w[g] / gate_b[g] for g >= 1 the
 * pre-gate that sits in block g-1 (routes block g).
 * The call only enqueues work (no host wait, no allocation, no memset) when the migration runs
 * in pull mode without an expert cache and neither tracing nor fetch timing is on, so it may be
 * captured into a HIP graph on compute_stream and replayed (the copy streams join the capture
 * through the call's own events and are joined back before it returns).  Not capturable: a
 * context that migrates with the copy engines (PGMOE_FLAG_FETCH_MEMCPY, or the choice of
 * PGMOE_FLAG_FETCH_AUTO; the host waits for the routing) and cache_slots > 0 (the cache
 * bookkeeping alternates between two device copies from call to call).
 * In pull mode the migrations of one call alternate between copy_stream and a second stream the
 * context owns, and their kernels take turns on the host link in block order (a device-side
 * wait that orders link traffic only, bounded by the clock: no result depends on it); block 0's
 * (exposed) migration runs on compute_stream itself and block 1's pre-gate runs on the
 * context's stream beside it (bf16 contexts).  All of this overlaps only if compute_stream,
 * copy_stream and the context's stream sit on different hardware queues: ask
 * pgmoe_check_streams() once at set-up.
 * With a resident store and pregate_distance 1, a decode-sized expert launch (up to 4 tokens, 8
 * or 16 experts) carries the pre-gate evaluated on the same hidden state as one extra workgroup:
 * results are those of the separate gate launch, bit for bit.
 * With pregate_distance N > 1 the gate that routes block g is evaluated on x_{max(0, g-N)}:
 * block 0 runs the gates of blocks 0..N on x_0 and queues their fetches back to back, block
 * i >= 1 runs the gate of block i+N; the last N blocks run none.  Arrays of pointers are host arrays of
 * device pointers; gate_b or any gate_b[g] may be NULL. */
/* Schedules of pgmoe_stack_step.  PREGATED is the paper's method and the default.  The other
 * two are the paper's comparison systems on the same kernels (Sec. III and the timeline figure
 * of Sec. IV-C): conventional wiring, i.e. gate_w[g] is block g's own gate applied to x_g, with
 *   ON_DEMAND    gate_i -> migrate the selected experts -> FFN_i, serially;
 *   PREFETCH_ALL all E experts of block i+1 migrate while block i executes (slots_per_gen = E).
 * With a resident expert store nothing migrates and either gives the GPU-only design point. */
#define PGMOE_SCHED_PREGATED 0
#define PGMOE_SCHED_ON_DEMAND 1
#define PGMOE_SCHED_PREFETCH_ALL 2
int pgmoe_set_schedule(pgmoe_ctx *ctx, int schedule);

/* Sensitivity aid, off by default (0): after every block's combine, pgmoe_stack_step keeps the
 * compute stream busy for `microseconds` with a kernel that does nothing but watch the clock: a
 * stand-in for the non-MoE layers (attention, the dense FFN layers) that sit between two MoE
 * blocks in the real model and that the paper's migration also hides behind (Sec. IV-C).  It
 * changes no result.  The kernel leaves after the given time or after a fixed number of clock
 * reads, whichever comes first.  0 <= microseconds <= 100000. */
int pgmoe_set_nonmoe_standin(pgmoe_ctx *ctx, float microseconds);

/* Diagnostic for pgmoe_stack_step's streams.  HIP maps streams onto a small number of hardware
 * queues (4 by default) and two streams that share one run their kernels in submission order:
 * the migration then silently serialises against the compute stream, or two consecutive
 * migrations against each other, and the step gets slower without any error.  This call starts a
 * clock-watching kernel of 200 us on two streams at a time and reports, as a bit mask in
 * *shared_out (host), which pairs did NOT run side by side.  The context's own copy stream is
 * replaced (up to 6 times) until it shares a queue with neither of the caller's streams; a caller
 * whose own two streams share one should pick another copy stream and ask again.  Synchronises
 * the device; call it at set-up, not in the hot path.  compute_stream == copy_stream (everything
 * in line) reports PGMOE_STREAMS_COMPUTE_COPY by definition. */
#define PGMOE_STREAMS_COMPUTE_COPY 1 /* the caller's compute and copy stream */
#define PGMOE_STREAMS_COMPUTE_OWN 2  /* the caller's compute stream and the context's own copy stream */
#define PGMOE_STREAMS_COPY_OWN 4     /* the caller's copy stream and the context's own copy stream */
int pgmoe_check_streams(pgmoe_ctx *ctx, void *compute_stream, void *copy_stream, int *shared_out);

typedef struct {
    const void *const *gate_w;  /* host [L] -> dev [d,E] */
    const float *const *gate_b; /* host [L] -> dev [E] | NULL; may itself be NULL */
    void *x_states;             /* dev [(L+1), T, d]: in: x_states[0] = x_0; out: x_1..x_L */
    void *y_blocks;             /* dev [L, T, d] out: y_i of every block | NULL */
    int32_t *topk_idx;          /* dev [L, T, k] out: routing used by block i */
    float *topk_prob;           /* dev [L, T, k] out */
    int32_t *row_of;            /* dev [L, T*k] out */
    int32_t *expert_offsets;    /* dev [L, E+1] out */
    void *x_perm;               /* dev [T*k, d] scratch */
    void *y_perm;               /* dev [T*k, d] scratch */
    void *workspace;            /* dev, pgmoe_workspace_bytes() */
} pgmoe_step_buffers;
/* T in the shapes above is the T of the call (0 <= T <= max_tokens): the arrays are packed for it,
 * whatever max_tokens the context was created with. */
int pgmoe_stack_step(pgmoe_ctx *ctx, const pgmoe_step_buffers *io, int T, void *compute_stream,
                     void *copy_stream);

/* ---- observability: duration of the expert-FFN kernel ------------------------------------
 * pgmoe_ffn_timing_begin() makes every following pgmoe_expert_ffn() bracket its main kernel
 * (the fused bf16 kernel, or the two f32 kernels; not the small partial-sum reduction) with a
 * pair of HIP events on the stream it is launched on, for up to max_launches launches (the
 * events are created here, not in the hot path; later launches are not timed).
 * pgmoe_ffn_timing_begin() also measures what an event pair itself adds: the median
 * event-to-event time around an empty kernel minus the period of back-to-back empty kernels
 * (the part of that time the empty kernel itself accounts for).
 * pgmoe_ffn_timing_end() waits for the recorded events, returns the number of timed launches,
 * the sum of their event-to-event times in milliseconds and that per-pair overhead (to be
 * subtracted per launch), and switches timing off.
 * n_out, total_ms_out host; pair_overhead_ms_out host | NULL. */
int pgmoe_ffn_timing_begin(pgmoe_ctx *ctx, int max_launches);
/* Name of the main kernel pgmoe_expert_ffn() launches for n_rows permuted rows in this context
 * ("ffn_decode_kernel", "ffn_fused_kernel", "ffn_gemm_pack_rows_kernel+ffn_gemm_tile_kernel" or
 * "ffn_f32_hidden_kernel+ffn_f32_out_kernel"): the
 * name to look for in a profiler's kernel trace.  Static string; NULL if ctx is NULL or no kernel
 * is built for that launch (pgmoe_expert_ffn() would return PGMOE_EINVAL; no accepted
 * configuration has such a launch). */
const char *pgmoe_ffn_kernel_name(const pgmoe_ctx *ctx, int n_rows);
int pgmoe_ffn_timing_end(pgmoe_ctx *ctx, int *n_out, float *total_ms_out, float *pair_overhead_ms_out);

/* ---- observability: per-block timeline of pgmoe_stack_step -------------------------------
 * With tracing on, every stack step records timing events per block: on the copy stream
 * around the migration, on the compute stream at the start of the block, just before and just
 * after the point where the FFN waits for its experts, and at the end of the block.  The event
 * records cost several microseconds each, so tracing is for instrumented passes only.
 * pgmoe_get_block_trace() waits for the block's events of the LAST step and fills:
 *   fetch_ms   duration of the block's migration kernel (copy stream), which includes the time it
 *              waits for its turn on the host link behind the migration before it;
 *   stall_ms   time the compute stream spent waiting for it (0 if the experts were there; all of
 *              fetch_ms and more when the migration ran on the compute stream itself);
 *   compute_ms duration of the block on the compute stream (pre-gate, grouping, FFN, combine)
 *              minus stall_ms;
 *   fetch_start_ms, fetch_end_ms, block_start_ms, block_end_ms: the same events as offsets
 *              from the start of block 0 on the compute stream;
 *   copy_ms    the copy alone: from the moment the migration kernel starts copying (its turn has
 *              come) to the return of its last load, by the kernel's own readings of the 100 MHz
 *              clock; bytes_copied / copy_ms is the link rate of that migration.  With the copy
 *              engines it equals fetch_ms. */
typedef struct {
    float fetch_ms, stall_ms, compute_ms;
    float fetch_start_ms, fetch_end_ms, block_start_ms, block_end_ms;
    float copy_ms;
} pgmoe_block_trace;
int pgmoe_trace(pgmoe_ctx *ctx, int enable);
int pgmoe_get_block_trace(pgmoe_ctx *ctx, int block, pgmoe_block_trace *out /* host */);

/* Sticky device-side condition bits since the last call of this function (synchronises the
 * device): bit 0 = a NaN logit was seen by a gate, bit 1 = an expert index outside [0,E)
 * reached pgmoe_permute or the pull kernel, bit 2 = more distinct experts than slots. */
int pgmoe_device_flags(pgmoe_ctx *ctx, uint32_t *flags_out /* host */);

#ifdef __cplusplus
}
#endif
#endif /* PGMOE_H */
