"""GPU parity: every entry point of libpgmoe, called through the C ABI, against the CPU oracle
on the same seeded inputs.  Integer results (expert indices away from near-ties, offsets,
row_of, permuted rows) must be bit-exact; floating point within the stated tolerances:
normalised max-abs error 1e-5 (f32) and 2e-2 (bf16).
"""
import sys

import numpy as np
import pytest

torch = pytest.importorskip("torch")

import workloads as W
from oracle import reference as R

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 2e-2}
TIE = 1e-4     # logit margin below which a token's selection is exempt from the exact check
HOST_THREADS = 16


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def hx():
    from paper_2308_12066_amd import binding, harness
    assert torch.cuda.is_available()
    return harness, binding


def nerr(a, ref):
    """max |a - ref| / max |ref| (normalised max-abs error)."""
    ref = np.asarray(ref, np.float64)
    den = np.abs(ref).max() if ref.size else 1.0
    return float(np.abs(np.asarray(a, np.float64) - ref).max() / (den if den > 0 else 1.0)) if ref.size else 0.0


def small_workload(dtype, T, d, f, E, k, L=2, zipf=0.0, offloaded=False, index=40):
    return W.Workload(f"t_{dtype}_{T}_{d}_{f}_{E}_{k}", index, L, d, f, E, k, T, 1, dtype, zipf, offloaded)


# ------------------------------------------------------------------------------ gate
GATE_CASES = [
    ("f32", 32, 64, 8, 1), ("f32", 37, 100, 5, 2), ("f32", 9, 1500, 12, 3), ("bf16", 1, 768, 8, 1),
    ("bf16", 16, 768, 64, 1), ("bf16", 64, 1024, 128, 2), ("bf16", 333, 768, 128, 1), ("bf16", 7, 256, 256, 4),
    ("bf16", 8, 64, 100, 100), ("f32", 5, 64, 1, 1), ("bf16", 20, 2048, 16, 2),
    # the smallest gates (at most 4 tokens, 8 or 16 experts) have a kernel of their own
    ("bf16", 4, 768, 8, 2), ("bf16", 3, 2048, 16, 16), ("bf16", 1, 64, 16, 1), ("bf16", 2, 1024, 8, 8), ("bf16", 5, 768, 8, 1),
]


@pytest.mark.parametrize("dtype,T,d,E,k", GATE_CASES)
def test_gate_topk_matches_oracle(hx, dtype, T, d, E, k):
    H, B = hx
    say(f"gate case dtype={dtype} T={T} d={d} E={E} k={k}")
    w = small_workload(dtype, T, d, 64 if dtype == "bf16" else 8, E, k)
    if dtype == "bf16" and d % 64:
        pytest.skip("bf16 needs d % 64 == 0")
    g = np.random.default_rng(1000 + T + d + E)
    x = g.standard_normal((T, d)).astype(np.float32)
    wg = (g.standard_normal((d, E)) * 0.05).astype(np.float32)
    bias = (g.standard_normal(E) * 0.3).astype(np.float32)
    if dtype == "bf16":
        x, wg = W.round_to_bf16(x), W.round_to_bf16(wg)
    ctx = B.Context(H.config_for(w))
    xd, wd, bd = H.to_device(x, dtype), H.to_device(wg, dtype), torch.from_numpy(bias).cuda()
    idx = torch.full((T, k), -1, dtype=torch.int32, device="cuda")
    prob = torch.zeros((T, k), dtype=torch.float32, device="cuda")
    probs = torch.zeros((T, E), dtype=torch.float32, device="cuda")
    for b_np, b_dev in ((bias, bd), (None, None)):
        ctx.pregate_topk(xd, wd, b_dev, T, idx, prob, probs)
        torch.cuda.synchronize()
        o = R.gate(x, wg, b_np, k)
        exact = o["gaps"].min(axis=1) >= TIE
        gi = idx.cpu().numpy()
        assert np.array_equal(gi[exact], o["idx"][exact]), "expert indices differ away from near-ties"
        assert exact.mean() > 0.5 or E <= 2 or k == E
        # near-tie tokens must still pick a valid set of distinct experts
        assert gi.min() >= 0 and gi.max() < E
        assert all(len(set(r)) == k for r in gi.tolist())
        assert nerr(probs.cpu().numpy(), o["p"]) <= 1e-5
        assert nerr(prob.cpu().numpy()[exact], o["prob"][exact]) <= 1e-5
        np.testing.assert_allclose(probs.cpu().numpy().sum(1), 1.0, atol=1e-5)
    assert ctx.device_flags() == 0
    ctx.close()


@pytest.mark.parametrize("dtype,T", [("f32", 6), ("bf16", 6), ("bf16", 3)])   # plain, matrix-core and smallest-gate kernel
def test_gate_ties_go_to_lowest_index_and_nan_is_flagged(hx, dtype, T):
    H, B = hx
    d, E, k = 64, 16, 3
    w = small_workload(dtype, T, d, 64, E, k)
    ctx = B.Context(H.config_for(w))
    x = np.random.default_rng(5).standard_normal((T, d)).astype(np.float32)
    if dtype == "bf16":
        x = W.round_to_bf16(x)
    wg = np.zeros((d, E), dtype=np.float32)
    idx = torch.zeros((T, k), dtype=torch.int32, device="cuda")
    prob = torch.zeros((T, k), dtype=torch.float32, device="cuda")
    ctx.pregate_topk(H.to_device(x, dtype), H.to_device(wg, dtype), None, T, idx, prob)
    torch.cuda.synchronize()
    assert np.array_equal(idx.cpu().numpy(), np.tile(np.arange(k, dtype=np.int32), (T, 1)))
    assert np.all(prob.cpu().numpy() == np.float32(1.0 / E))
    assert ctx.device_flags() == 0
    # a NaN logit ranks last and raises the flag (bias carries the NaN for expert 2 of all tokens)
    bias = np.zeros(E, dtype=np.float32)
    bias[2] = np.nan
    bias[7] = 1.0
    ctx.pregate_topk(H.to_device(x, dtype), H.to_device(wg, dtype), torch.from_numpy(bias).cuda(), T, idx, prob)
    torch.cuda.synchronize()
    o = R.gate(x, wg, bias, k)
    assert np.array_equal(idx.cpu().numpy(), o["idx"]) and o["idx"][0].tolist() == [7, 0, 1]
    assert ctx.device_flags() & 1
    assert ctx.device_flags() == 0           # reading clears
    ctx.close()


# ------------------------------------------------------------------------------ permute
@pytest.mark.parametrize("dtype,T,d,E,k,mode", [
    ("f32", 32, 64, 8, 1, "rand"), ("bf16", 1, 768, 8, 1, "rand"), ("bf16", 64, 1024, 128, 2, "rand"),
    ("bf16", 4096, 768, 128, 1, "rand"), ("bf16", 1500, 64, 7, 3, "rand"), ("bf16", 1111, 64, 256, 1, "one"),
    ("f32", 3, 5, 4, 4, "rand"), ("bf16", 2500, 128, 64, 2, "zipf"),
    ("bf16", 6000, 64, 33, 2, "zipf"),      # 12000 entries: more rounds per wavefront than the grouping kernel keeps in registers
])
def test_permute_is_bit_exact(hx, dtype, T, d, E, k, mode):
    H, B = hx
    say(f"permute case dtype={dtype} T={T} d={d} E={E} k={k} mode={mode}")
    w = small_workload(dtype, T, d, 64, E, k)
    ctx = B.Context(H.config_for(w))
    g = np.random.default_rng(T * 7 + E)
    if mode == "one":
        idx = np.full((T, k), E - 3, dtype=np.int32)
    else:
        p = None if mode == "rand" else W.zipf_probabilities(E, 1.1)
        idx = np.stack([g.choice(E, size=k, replace=False, p=p) for _ in range(T)]).astype(np.int32)
    x = g.standard_normal((T, d)).astype(np.float32)
    if dtype == "bf16":
        x = W.round_to_bf16(x)
    xd = H.to_device(x, dtype)
    x_perm = torch.zeros((T * k, d), dtype=xd.dtype, device="cuda")
    row_of = torch.full((T * k,), -1, dtype=torch.int32, device="cuda")
    offs = torch.full((E + 1,), -1, dtype=torch.int32, device="cuda")
    ctx.permute(xd, torch.from_numpy(idx).cuda(), T, x_perm, row_of, offs)
    torch.cuda.synchronize()
    r = R.route(idx, E)
    assert np.array_equal(offs.cpu().numpy(), r["offsets"])
    assert np.array_equal(row_of.cpu().numpy(), r["row_of"])
    expect = np.empty((T * k, d), dtype=np.float64)
    expect[r["row_of"]] = np.repeat(x.astype(np.float64), k, axis=0)
    assert np.array_equal(H.to_numpy64(x_perm), expect)
    assert ctx.device_flags() == 0
    ctx.close()


def test_permute_empty_and_bad_index(hx):
    H, B = hx
    w = small_workload("bf16", 8, 64, 64, 4, 1)
    ctx = B.Context(H.config_for(w))
    x = H.to_device(np.ones((8, 64), np.float32), "bf16")
    x_perm = torch.zeros((8, 64), dtype=torch.bfloat16, device="cuda")
    row_of = torch.zeros(8, dtype=torch.int32, device="cuda")
    offs = torch.full((5,), -1, dtype=torch.int32, device="cuda")
    ctx.permute(x, torch.zeros(8, dtype=torch.int32, device="cuda"), 0, x_perm, row_of, offs)
    torch.cuda.synchronize()
    assert offs.cpu().tolist() == [0, 0, 0, 0, 0]
    bad = torch.tensor([0, 1, 9, 2, -4, 3, 1, 0], dtype=torch.int32, device="cuda")
    ctx.permute(x, bad, 8, x_perm, row_of, offs)
    torch.cuda.synchronize()
    assert ctx.device_flags() & 2
    assert offs.cpu().tolist()[-1] == 8 and sorted(row_of.cpu().tolist()) == list(range(8))
    ctx.close()


@pytest.mark.parametrize("fetch", ["pull", "memcpy"])
def test_every_call_takes_an_empty_batch(hx, fetch):
    """T = 0 (n_rows = 0) is a valid no-op everywhere: nothing is written, nothing is migrated."""
    H, B = hx
    w = small_workload("bf16", 8, 64, 64, 4, 2, L=2, offloaded=True, index=62)
    stack, gates, cache = make_stack(H, w, threads=2, flags=B.FLAG_FETCH_MEMCPY if fetch == "memcpy" else 0)
    ctx, T, k, d = stack.ctx, w.tokens, w.top_k, w.d_model
    x = H.to_device(W.step_input(w, 0), "bf16")
    idx = torch.full((T, k), -7, dtype=torch.int32, device="cuda")
    prob = torch.full((T, k), -7.0, dtype=torch.float32, device="cuda")
    row_of = torch.full((T * k,), -7, dtype=torch.int32, device="cuda")
    offs = torch.full((w.n_experts + 1,), -7, dtype=torch.int32, device="cuda")
    y = torch.full((T * k, d), 7.0, dtype=torch.bfloat16, device="cuda")
    ctx.pregate_topk(x, stack.gate_w[0], stack.gate_b[0], 0, idx, prob, None, stack.compute)
    assert ctx.fetch_experts(0, idx, 0, stack.compute, stack.copy) == 0
    ctx.expert_ffn(0, x, offs, 0, y, stack.workspace, stack.compute)
    ctx.combine(y, row_of, prob, 0, y, None, None, stack.compute)
    torch.cuda.synchronize()
    assert (idx == -7).all() and (prob == -7).all() and (y == 7).all() and (row_of == -7).all()
    fs = ctx.fetch_stats(0)
    assert fs.n_unique == 0 and fs.bytes_copied == 0
    before = stack.x_states.clone()
    stack.step(T=0)
    torch.cuda.synchronize()
    assert torch.equal(stack.x_states, before)
    assert ctx.device_flags() == 0
    stack.close()


# ------------------------------------------------------------------------------ expert FFN
def run_ffn_case(H, B, dtype, d, f, E, counts, seed, scale=0.05):
    """Resident store of E experts; counts[e] rows for expert e.  Returns (gpu y_perm, oracle y_perm)."""
    counts = np.asarray(counts, dtype=np.int64)
    n = int(counts.sum())
    w = W.Workload("ffn_case", 50, 1, d, f, E, 1, max(n, 1), 1, dtype, 0.0, False)
    cfg = H.config_for(w)
    g = np.random.default_rng(seed)
    weights = {}

    def get(b, e):
        w1 = (g.standard_normal((d, f)) * scale).astype(np.float32)
        w2 = (g.standard_normal((f, d)) * scale).astype(np.float32)
        if dtype == "bf16":
            w1, w2 = W.round_to_bf16(w1), W.round_to_bf16(w2)
        weights[e] = (w1, w2)
        return w1, w2

    store = H.ExpertStore(w, cfg, threads=1, get_expert=get)
    ctx = B.Context(cfg)
    ctx.register_resident_experts(store.to_hbm(), store.expert_stride, store.block_stride)
    x = g.standard_normal((n, d)).astype(np.float32)
    if dtype == "bf16":
        x = W.round_to_bf16(x)
    offs = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    xd = H.to_device(x, dtype)
    y = torch.full((max(n, 1), d), 7.0, dtype=xd.dtype, device="cuda")
    ws = torch.zeros(ctx.workspace_bytes, dtype=torch.uint8, device="cuda")
    ctx.expert_ffn(0, xd, torch.from_numpy(offs).cuda(), n, y, ws)
    torch.cuda.synchronize()
    ref = np.zeros((n, d))
    for e in range(E):
        if counts[e]:
            ref[offs[e]: offs[e + 1]] = R.ffn_rows(x[offs[e]: offs[e + 1]], *weights[e])
    out = H.to_numpy64(y)[:n]
    ctx.close()
    return out, ref


FFN_CASES = [
    # dtype, d, f, E, counts
    ("f32", 64, 256, 8, [3, 0, 5, 1, 0, 0, 9, 14]),
    ("f32", 20, 36, 3, [1, 2, 3]),
    ("bf16", 64, 128, 4, [1, 0, 2, 0]),
    ("bf16", 128, 256, 8, [17, 0, 1, 33, 0, 16, 2, 70]),       # ragged tails, >1 chunk per expert
    ("bf16", 256, 512, 5, [0, 0, 0, 0, 1]),
    ("bf16", 768, 3072, 8, [0, 0, 0, 1, 0, 0, 0, 0]),          # decode, batch 1 (Switch-Base-8 shape)
    ("bf16", 768, 3072, 16, [4, 0, 1, 0, 0, 2, 0, 1, 0, 0, 0, 3, 1, 0, 0, 4]),
    ("bf16", 1024, 4096, 6, [16, 1, 0, 31, 2, 14]),
    ("bf16", 768, 3072, 4, [40, 25, 33, 64]),                  # prefill-like rows per expert
    ("bf16", 512, 1024, 3, [200, 3, 90]),
    # few active experts with <= 16 rows per chunk: the decode kernel (full chunk + second chunk, ragged, d_model 1024)
    ("bf16", 768, 3072, 5, [17, 0, 0, 0, 2]),
    ("bf16", 768, 3072, 4, [4, 0, 3, 0]),
    ("bf16", 1024, 4096, 3, [1, 0, 2]),
    # hundreds of rows per expert: the two tiled GEMMs (ragged 256-row chunks, an idle expert, a 5-row expert)
    ("bf16", 768, 3072, 2, [300, 217]),
    ("bf16", 256, 512, 3, [0, 700, 5]),
    ("bf16", 512, 1024, 4, [600, 700, 500, 760]),              # enough row chunks for two K slices instead of four
    ("bf16", 1024, 4096, 2, [333, 290]),                       # the two GEMMs on the Switch-Large expert shape
    # the largest d_model the bf16 path takes (16-row chunks only there), fused kernel and the two GEMMs
    ("bf16", 2048, 256, 3, [5, 0, 40]),
    ("bf16", 2048, 256, 2, [200, 260]),
    ("bf16", 1024, 4096, 3, [40, 25, 33]),                     # 64-row chunks at d_model 1024: the largest LDS footprint
    ("bf16", 768, 192, 2, [30, 50]),                           # 64-row chunks with a d_ff that has no 128-column sub-slabs
]


@pytest.mark.parametrize("dtype,d,f,E,counts", FFN_CASES)
def test_expert_ffn_matches_oracle(hx, dtype, d, f, E, counts):
    H, B = hx
    say(f"ffn case dtype={dtype} d={d} f={f} E={E} counts={counts}")
    out, ref = run_ffn_case(H, B, dtype, d, f, E, counts, seed=d + f + E)
    err = nerr(out, ref)
    say(f"  normalised max-abs error {err:.3e}")
    assert err <= TOL[dtype]
    # per-expert errors too, so that one wrong small expert cannot hide behind a big one
    offs = np.concatenate([[0], np.cumsum(counts)])
    for e in range(E):
        if counts[e]:
            assert nerr(out[offs[e]: offs[e + 1]], ref[offs[e]: offs[e + 1]]) <= TOL[dtype], f"expert {e}"


@pytest.mark.parametrize("d,f,E,counts", [
    (768, 3072, 4, [300, 217, 512, 200]),     # the two tiled GEMMs (LDS ring filled by direct loads)
    (768, 3072, 16, [40, 25, 33, 64, 7, 0, 16, 12, 3, 50, 9, 1, 0, 30, 22, 18]),   # fused kernel
    (768, 3072, 8, [0, 0, 1, 0, 0, 2, 0, 0]),  # decode kernel
])
def test_expert_ffn_is_bit_reproducible_run_after_run(hx, d, f, E, counts):
    """The kernels add in a fixed order and use no atomics on floats, so repeating a launch must give
    the same bits; a race in an LDS ring or a missed wait would show up here as a difference."""
    H, B = hx
    n = int(sum(counts))
    w = W.Workload("ffn_repeat_case", 51, 1, d, f, E, 1, n, 1, "bf16", 0.0, False)
    cfg = H.config_for(w)
    g = np.random.default_rng(d + E)
    store = H.ExpertStore(w, cfg, threads=4, get_expert=lambda b, e: (
        W.round_to_bf16((np.random.default_rng(1000 + e).standard_normal((d, f)) * 0.05).astype(np.float32)),
        W.round_to_bf16((np.random.default_rng(2000 + e).standard_normal((f, d)) * 0.05).astype(np.float32))))
    ctx = B.Context(cfg)
    ctx.register_resident_experts(store.to_hbm(), store.expert_stride, store.block_stride)
    xd = H.to_device(W.round_to_bf16(g.standard_normal((n, d)).astype(np.float32)), "bf16")
    offs = torch.from_numpy(np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)).cuda()
    ws = torch.zeros(ctx.workspace_bytes, dtype=torch.uint8, device="cuda")
    y = torch.zeros((n, d), dtype=torch.bfloat16, device="cuda")
    ctx.expert_ffn(0, xd, offs, n, y, ws)
    torch.cuda.synchronize()
    first = y.clone()
    assert float(first.float().abs().max()) > 0
    for rep in range(100):
        y.fill_(3.0)
        ctx.expert_ffn(0, xd, offs, n, y, ws)
        if rep % 10 == 9:
            torch.cuda.synchronize()
            assert torch.equal(y.view(torch.int16), first.view(torch.int16)), f"repeat {rep} differs"
    ctx.close()


# ------------------------------------------------------------------------------ combine
@pytest.mark.parametrize("dtype,T,d,k", [("f32", 32, 64, 1), ("f32", 5, 7, 3), ("bf16", 64, 1024, 2), ("bf16", 300, 768, 1)])
def test_combine_matches_definition(hx, dtype, T, d, k):
    H, B = hx
    w = small_workload(dtype, T, d if dtype == "f32" else d, 64, 8, k)
    ctx = B.Context(H.config_for(w))
    g = np.random.default_rng(T + d + k)
    yp = g.standard_normal((T * k, d)).astype(np.float32)
    xr = g.standard_normal((T, d)).astype(np.float32)
    if dtype == "bf16":
        yp, xr = W.round_to_bf16(yp), W.round_to_bf16(xr)
    row_of = g.permutation(T * k).astype(np.int32)
    prob = g.uniform(0.05, 1.0, size=(T, k)).astype(np.float32)
    ypd, xrd = H.to_device(yp, dtype), H.to_device(xr, dtype)
    y = torch.zeros((T, d), dtype=ypd.dtype, device="cuda")
    xn = torch.zeros((T, d), dtype=ypd.dtype, device="cuda")
    ctx.combine(ypd, torch.from_numpy(row_of).cuda(), torch.from_numpy(prob).cuda(), T, y, xrd, xn)
    torch.cuda.synchronize()
    ref = (prob.astype(np.float64)[:, :, None] * yp.astype(np.float64)[row_of.reshape(T, k)]).sum(1)
    tol = 1e-6 if dtype == "f32" else 2.0 ** -8
    assert nerr(H.to_numpy64(y), ref) <= tol
    assert nerr(H.to_numpy64(xn), ref + xr) <= tol
    y2 = torch.zeros_like(y)
    ctx.combine(ypd, torch.from_numpy(row_of).cuda(), torch.from_numpy(prob).cuda(), T, y2)
    torch.cuda.synchronize()
    assert torch.equal(y, y2)
    ctx.close()


# ------------------------------------------------------------------------------ whole stack
def check_stack_step(H, w, stack, gates, expert_cache, sample_tokens=None, label="", wiring="pregated", distance=1):
    """Block-by-block check of one executed step against the oracle evaluated on the GPU's own
    hidden states (x_{i-1} routes block i, x_i feeds its experts).  Returns statistics."""
    torch.cuda.synchronize()
    L, T, k, E = w.n_blocks, w.tokens, w.top_k, w.n_experts
    xs = H.to_numpy64(stack.x_states)
    ys = H.to_numpy64(stack.y_blocks)
    idx_g = stack.topk_idx.cpu().numpy()
    prob_g = stack.topk_prob.cpu().numpy()
    row_g = stack.row_of.cpu().numpy()
    off_g = stack.expert_offsets.cpu().numpy()
    stats = dict(near_tie=0, tokens=0, max_err=0.0, max_prob_err=0.0)
    for i in range(L):
        gw, gb = gates[i]
        o = R.gate(xs[R.routing_source(i, wiring, distance)], gw, gb, k)
        exact = o["gaps"].min(axis=1) >= TIE
        stats["near_tie"] += int((~exact).sum())
        stats["tokens"] += T
        assert np.array_equal(idx_g[i][exact], o["idx"][exact]), f"{label} block {i}: routing differs"
        stats["max_prob_err"] = max(stats["max_prob_err"], nerr(prob_g[i][exact], o["prob"][exact]))
        assert stats["max_prob_err"] <= 1e-5
        r = R.route(idx_g[i], E)                      # integer bookkeeping from the GPU's own indices
        assert np.array_equal(off_g[i], r["offsets"]) and np.array_equal(row_g[i], r["row_of"])
        toks = np.flatnonzero(exact)
        if len(toks) == 0:      # every token of the block sits on a near-tie (e.g. k = E, where the last gap is to nothing)
            continue
        if sample_tokens is not None and len(toks) > sample_tokens:
            toks = np.sort(np.random.default_rng(i).choice(toks, sample_tokens, replace=False))
        need = np.unique(o["idx"][toks])
        if hasattr(expert_cache, "prefetch"):      # a source that generates a block's experts in parallel
            expert_cache.prefetch(i, need)
        experts = {int(e): expert_cache(i, int(e)) for e in need}
        y_ref = R.block(xs[i][toks], o["p"][toks], o["idx"][toks], experts, w.d_ff)
        err = nerr(ys[i][toks], y_ref)
        stats["max_err"] = max(stats["max_err"], err)
        assert err <= TOL[w.dtype], f"{label} block {i}: y error {err:.3e}"
        # residual stand-in x_{i+1} = x_i + y_i: y_i itself is held to the oracle above, so the sum is
        # checked against the GPU's own y_i (one rounding of y, one of the sum); measuring it against
        # the oracle's y would count the expert error a second time, scaled by |y| / |x|
        x_ref = xs[i][toks] + ys[i][toks]
        xerr = nerr(xs[i + 1][toks], x_ref)
        unit = 2.0 ** -23 if w.dtype == "f32" else 2.0 ** -8      # largest relative error of one rounding
        x_tol = unit * (1.0 + np.abs(ys[i][toks]).max() / np.abs(x_ref).max())
        assert xerr <= x_tol, f"{label} block {i}: x_next error {xerr:.3e} (bound {x_tol:.3e})"
    return stats


def make_stack(H, w, threads=HOST_THREADS, flags=0, pregate_distance=0, weight_scale=1.0):
    """weight_scale: a power of two (keeps bf16 values exact) that makes the blocks' outputs
    comparable to the hidden state, so that consecutive hidden states route differently."""
    cfg = H.config_for(w, flags=flags)
    cache = {}

    def get(b, e):
        w1, w2 = W.expert_weights(w, b, e)
        if weight_scale != 1.0:
            w1, w2 = w1 * np.float32(weight_scale), w2 * np.float32(weight_scale)
        cache[(b, e)] = (W.to_bf16_bits(w1), W.to_bf16_bits(w2)) if w.dtype == "bf16" else (w1, w2)
        return w1, w2

    store = H.ExpertStore(w, cfg, threads=threads, get_expert=get)
    gates = W.gate_tensors(w)
    stack = H.Stack(w, store, gates=gates, flags=flags, pregate_distance=pregate_distance)
    return stack, gates, (lambda b, e: cache[(b, e)])


@pytest.mark.parametrize("T,E,k,fetch", [(8, 16, 2, "pull"), (1, 8, 1, "pull"), (300, 8, 1, "pull"), (8, 16, 2, "memcpy")])
def test_offloaded_stack_repeats_bit_for_bit_over_many_steps(hx, T, E, k, fetch):
    """300 steps that alternate between two inputs, all queued back to back: every step must give
    the bits its input gave the first time.  A migration that overwrote slots still in use, an
    FFN that started before its experts had arrived or a stale routing would show up here."""
    H, B = hx
    w = small_workload("bf16", T, 128, 256, E, k, L=4, offloaded=True, index=58)
    stack, gates, cache = make_stack(H, w, flags=0 if fetch == "pull" else B.FLAG_FETCH_MEMCPY, weight_scale=4.0)
    inputs = [H.to_device(W.step_input(w, s), "bf16") for s in range(2)]
    first = []
    for x0 in inputs:
        stack.x_states[0].copy_(x0)
        torch.cuda.synchronize()
        stack.step()
        torch.cuda.synchronize()
        first.append((stack.x_states.clone(), stack.topk_idx.clone()))
    assert not torch.equal(first[0][1], first[1][1]), "the two inputs should route differently"
    cs = torch.cuda.current_stream()
    for s in range(300):
        want_x, want_idx = first[s & 1]
        # the input copy and the check run on the stack's compute stream, in order with the steps
        with torch.cuda.stream(stack.compute):
            stack.x_states[0].copy_(inputs[s & 1], non_blocking=True)
        stack.step()
        if s % 25 >= 23:   # two consecutive steps (both inputs) out of every 25
            torch.cuda.synchronize()
            assert torch.equal(stack.topk_idx, want_idx), f"step {s}: routing differs"
            assert torch.equal(stack.x_states.view(torch.int16), want_x.view(torch.int16)), f"step {s}: hidden states differ"
    torch.cuda.synchronize()
    assert stack.ctx.device_flags() == 0
    stack.close()


def test_cfg1_tiny_f32_stack_all_tokens(hx):
    H, B = hx
    w = W.CONFIGS["cfg1"]
    say("stack cfg1")
    stack, gates, cache = make_stack(H, w)
    stack.set_input(W.step_input(w, 0))
    stack.step()
    st = check_stack_step(H, w, stack, gates, cache, label="cfg1")
    say(f"  cfg1 {st}")
    # the free-running fp64 chain agrees as well at this size (f32 drift is far below the tie margin)
    out, x_last = R.stack_forward(W.step_input(w, 0), gates, w.top_k, lambda b, e: cache(b, e), w.d_ff)
    torch.cuda.synchronize()
    assert nerr(H.to_numpy64(stack.x_states[-1]), x_last) <= 1e-5
    for i in range(w.n_blocks):
        assert np.array_equal(stack.topk_idx[i].cpu().numpy(), out[i]["gate"]["idx"])
    stack.close()


@pytest.mark.parametrize("name,blocks,steps,sample,fetch", [
    ("cfg2", 6, 6, None, "pull"), ("cfg2", 6, 4, None, "memcpy"), ("cfg3", 6, 3, None, "pull"),
    ("cfg4", 2, 1, 192, "-"), ("base8_prefill", 2, 1, 96, "-"), ("cfg4_offloaded", 2, 1, 64, "pull"), ("cfg5", 3, 2, None, "pull"),
    ("cfg5_top2", 3, 2, None, "pull"), ("cfg5_top2", 3, 2, None, "memcpy"),
    ("sweep64_k4", 2, 2, None, "pull"), ("sweep64_k16", 2, 1, None, "memcpy"), ("sweep64_k64", 2, 2, None, "pull"),
])
def test_switch_shaped_stacks(hx, name, blocks, steps, sample, fetch):
    """Full d_model / d_ff / E / T of the Switch-shaped workloads; the number of blocks and steps
    is cut down to keep host-side weight generation within the test budget (each block runs
    the same launches)."""
    H, B = hx
    w = W.CONFIGS[name].replace(n_blocks=blocks)
    say(f"stack {name}: L={blocks} steps={steps} T={w.tokens} E={w.n_experts} k={w.top_k} offloaded={w.offloaded} fetch={fetch}")
    stack, gates, cache = make_stack(H, w, flags=B.FLAG_FETCH_MEMCPY if fetch == "memcpy" else 0)
    stack.ctx.fetch_timing(True)
    near = tot = 0
    for s in range(steps):
        stack.set_input(W.step_input(w, s))
        stack.step()
        st = check_stack_step(H, w, stack, gates, cache, sample_tokens=sample, label=f"{name} step {s}")
        near += st["near_tie"]
        tot += st["tokens"]
        say(f"  step {s}: {st}")
        if w.offloaded:
            for b in range(blocks):
                fs = stack.ctx.fetch_stats(b)
                u = len(np.unique(stack.topk_idx[b].cpu().numpy()))
                assert fs.n_unique == u and fs.bytes_copied == u * w.expert_bytes
                nb = [len(np.unique(stack.topk_idx[j].cpu().numpy())) for j in (b - 1, b + 1) if 0 <= j < blocks]
                assert fs.resident_slots <= u + max(nb, default=0)      # two generations at most
    say(f"  {name}: near-tie tokens exempted {near} of {tot}")
    assert stack.ctx.device_flags() == 0
    stack.close()


def test_migrations_of_a_step_take_turns_on_the_host_link(hx):
    """Switch-Base-8 decode shape (one 9.4 MB expert per block): the migration kernels of a step
    finish one after the other, in block order, instead of sharing the link in pairs.  Only the
    order is asserted (a loaded box stretches every interval); the distances, about one 165 us
    copy each, are printed."""
    H, B = hx
    w = W.CONFIGS["cfg2"]
    stack, gates, cache = make_stack(H, w)
    stack.ctx.trace(True)
    worst = []
    for s in range(4):
        stack.set_input(W.step_input(w, s))
        stack.step()
        torch.cuda.synchronize()
        ends = [stack.ctx.block_trace(b).fetch_end_ms for b in range(w.n_blocks)]
        gaps = np.diff(ends) * 1e3
        say(f"  step {s}: fetches end {np.round(np.array(ends) * 1e3).astype(int).tolist()} us after the step's start")
        worst.append(float(gaps.min()))
        # block 0's experts are needed at once: nothing hides that migration, wherever it runs
        t0 = stack.ctx.block_trace(0)
        assert t0.stall_ms >= 0.5 * t0.fetch_ms > 0.0, (t0.stall_ms, t0.fetch_ms)
    stack.ctx.trace(False)
    say(f"  smallest distance between consecutive fetch ends per step: {[round(x) for x in worst]} us")
    assert min(worst) > 0.0, worst
    stack.close()


@pytest.mark.parametrize("distance,fetch,T,E,k", [(2, "pull", 16, 16, 1), (3, "pull", 5, 8, 2), (2, "memcpy", 16, 16, 1),
                                                   (3, "memcpy", 33, 12, 1)])
def test_pregate_distance_routes_from_the_earlier_state_and_keeps_more_generations(hx, distance, fetch, T, E, k):
    """Pre-gate looking N = 2 / 3 blocks ahead (Sec. VI-D): block i is routed from x_{max(0,i-N)},
    its experts are fetched N blocks early and N + 1 generations are resident."""
    H, B = hx
    L = 7
    w = small_workload("bf16", T, 128, 256, E, k, L=L, offloaded=True, index=46 + distance)
    say(f"pre-gate distance {distance}: fetch={fetch} T={T} E={E} k={k} L={L}")
    stack, gates, cache = make_stack(H, w, flags=B.FLAG_FETCH_MEMCPY if fetch == "memcpy" else 0, pregate_distance=distance,
                                     weight_scale=4.0)
    for s in range(3):
        stack.set_input(W.step_input(w, s))
        stack.step()
        st = check_stack_step(H, w, stack, gates, cache, label=f"distance {distance} step {s}", distance=distance)
        say(f"  step {s}: {st}")
        idx = stack.topk_idx.cpu().numpy()
        u = [len(np.unique(idx[b])) for b in range(L)]
        for b in range(L):
            fs = stack.ctx.fetch_stats(b)
            assert fs.n_unique == u[b] and fs.bytes_copied == u[b] * w.expert_bytes
            assert u[b] <= fs.resident_slots <= sum(u[max(0, b - distance): b + 1])    # N + 1 generations at most
            # the generation holds exactly the selected experts, in ascending order
            for j, e in enumerate(np.unique(idx[b])):
                if b >= L - 1 - distance:      # still resident after the step: not overwritten by a later block
                    got = _device_bytes(stack.ctx.slot_address(b, j), w.expert_bytes)
                    assert np.array_equal(got, stack.store.blob(b, int(e)))
    assert stack.ctx.device_flags() == 0
    # the wiring is really the distant one: on this data the default wiring selects differently
    xs = H.to_numpy64(stack.x_states)
    differs = any(not np.array_equal(R.gate(xs[max(0, i - 1)], gates[i][0], gates[i][1], k)["idx"], idx[i]) for i in range(2, L))
    assert differs
    stack.close()


@pytest.mark.parametrize("offloaded,shape", [(False, "small"), (True, "small"), (False, "decode"), (True, "decode")])
def test_stack_step_replays_from_a_captured_graph(hx, offloaded, shape):
    """pgmoe_stack_step only enqueues (pull-mode migration, no host wait, no memset), so a caller
    can capture one step into a HIP graph and replay it: every replay, with the program's own
    eager work and synchronisations in between, must give exactly what the eager step gives."""
    H, B = hx
    if shape == "small":
        w = small_workload("bf16", 6, 128, 256, 8, 2, L=4, offloaded=offloaded, index=53)
    else:   # batch-size-2 decode of the 8-expert shape: smallest-gate kernel, decode expert kernel (which carries the
        # next pre-gate when the experts are resident), turn-taking migrations with block 0's on the compute stream
        w = small_workload("bf16", 2, 768, 3072, 8, 1, L=4, offloaded=offloaded, index=64)
    say(f"graph replay: offloaded={offloaded} shape={shape}")
    stack, gates, cache = make_stack(H, w, weight_scale=4.0)
    xs_in = [H.to_device(W.step_input(w, s), w.dtype) for s in range(4)]
    eager = []
    for x in xs_in:                                  # eager results (and warm-up of every kernel)
        stack.x_states[0].copy_(x)
        torch.cuda.synchronize()
        stack.step()
        torch.cuda.synchronize()
        eager.append((stack.x_states.clone(), stack.topk_idx.clone(), stack.topk_prob.clone(), stack.row_of.clone()))
    graph = torch.cuda.CUDAGraph()
    stack.x_states[0].copy_(xs_in[0])
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=stack.compute):
        stack.step()
    torch.cuda.synchronize()
    for rep in range(2):
        for s, x in enumerate(xs_in):
            stack.x_states[0].copy_(x)
            stack.x_states[1:].zero_()              # eager work between replays
            stack.topk_idx.zero_()
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            ex, ei, ep, er = eager[s]
            assert torch.equal(stack.topk_idx, ei) and torch.equal(stack.row_of, er), f"replay {rep}/{s}: routing"
            assert torch.equal(stack.topk_prob, ep)
            assert torch.equal(stack.x_states.view(torch.int16), ex.view(torch.int16)), f"replay {rep}/{s}: hidden states"
    # and the eager path still works after the capture
    stack.x_states[0].copy_(xs_in[1])
    torch.cuda.synchronize()
    stack.step()
    torch.cuda.synchronize()
    assert torch.equal(stack.x_states.view(torch.int16), eager[1][0].view(torch.int16))
    assert stack.ctx.device_flags() == 0
    del graph
    stack.close()


def test_a_copy_engine_context_refuses_to_be_captured(hx):
    """With the copy engines the host waits for the routing inside the call; under stream capture
    nothing runs, so the call must refuse (before it queues anything) instead of waiting for ever."""
    H, B = hx
    w = small_workload("bf16", 6, 128, 256, 8, 2, L=3, offloaded=True, index=54)
    stack, gates, cache = make_stack(H, w, flags=B.FLAG_FETCH_MEMCPY)
    stack.set_input(W.step_input(w, 0))
    stack.step()
    torch.cuda.synchronize()
    want = stack.x_states.clone()
    graph = torch.cuda.CUDAGraph()
    with pytest.raises(B.PgmoeError) as ei:
        with torch.cuda.graph(graph, stream=stack.compute):
            stack.ctx.fetch_experts(0, stack.topk_idx[0], w.tokens, stack.compute, stack.copy)
    assert ei.value.code == B.ESTATE and "captured" in str(ei.value)
    del graph
    torch.cuda.synchronize()
    stack.x_states[1:].zero_()
    stack.step()                                     # and the context still works
    torch.cuda.synchronize()
    assert torch.equal(stack.x_states.view(torch.int16), want.view(torch.int16))
    stack.close()


def test_nonmoe_standin_changes_the_time_not_the_results(hx):
    """The clock-watching stand-in for the non-MoE layers only occupies the compute stream."""
    import time
    H, B = hx
    w = small_workload("bf16", 4, 128, 256, 8, 1, L=4, offloaded=True, index=57)
    stack, gates, cache = make_stack(H, w)
    stack.set_input(W.step_input(w, 0))
    stack.step()
    torch.cuda.synchronize()
    ref = stack.x_states.clone()
    t0 = time.perf_counter()
    stack.step()
    torch.cuda.synchronize()
    plain = time.perf_counter() - t0
    stack.ctx.set_nonmoe_standin(2000.0)
    stack.x_states[1:].zero_()
    t0 = time.perf_counter()
    stack.step()
    torch.cuda.synchronize()
    slow = time.perf_counter() - t0
    assert torch.equal(stack.x_states.view(torch.int16), ref.view(torch.int16))
    # 4 blocks x 2 ms of clock watching at least (the kernel cannot leave earlier), and it does end
    assert slow > plain + 4 * 1.5e-3 and slow < plain + 1.0, (plain, slow)
    with pytest.raises(B.PgmoeError):
        stack.ctx.set_nonmoe_standin(-1.0)
    stack.ctx.set_nonmoe_standin(0.0)
    stack.close()


# ------------------------------------------------------------------------------ migration engine
def _device_bytes(addr, nbytes):
    """Copy nbytes from a raw device address to host (plumbing: hipMemcpy through ctypes)."""
    import ctypes
    hip = ctypes.CDLL("libamdhip64.so")
    out = np.empty(nbytes, dtype=np.uint8)
    rc = hip.hipMemcpy(ctypes.c_void_p(out.ctypes.data), ctypes.c_void_p(addr), ctypes.c_size_t(nbytes), ctypes.c_int(2))
    assert rc == 0
    return out


@pytest.mark.parametrize("fetch", ["pull", "memcpy"])
def test_fetch_copies_exactly_the_selected_experts(hx, fetch):
    """Slot j of the block's generation holds, byte for byte, the blob of the j-th smallest
    selected expert, and nothing but the selected experts is counted as copied."""
    H, B = hx
    w = W.Workload("fetch_case", 70, 3, 128, 256, 16, 2, 12, 1, "bf16", 0.0, True)
    cfg = H.config_for(w, flags=B.FLAG_FETCH_MEMCPY if fetch == "memcpy" else 0)
    store = H.ExpertStore(w, cfg, threads=4)
    ctx = B.Context(cfg)
    ctx.register_host_experts(store.host, store.expert_stride, store.block_stride)
    comp, copy = torch.cuda.Stream(), torch.cuda.Stream()
    g = np.random.default_rng(9)
    for block in (0, 1, 2, 1):
        idx = np.stack([g.choice(16, size=2, replace=False) for _ in range(12)]).astype(np.int32)
        idx_d = torch.from_numpy(idx).cuda()
        torch.cuda.synchronize()
        nu = ctx.fetch_experts(block, idx_d, 12, comp, copy)
        torch.cuda.synchronize()
        uniq = np.unique(idx)
        assert nu == len(uniq)
        fs = ctx.fetch_stats(block)
        assert fs.n_unique == len(uniq) and fs.n_copied == len(uniq) and fs.bytes_copied == len(uniq) * store.expert_bytes
        for j, e in enumerate(uniq):
            got = _device_bytes(ctx.slot_address(block, j), store.expert_bytes)
            assert np.array_equal(got, store.blob(block, int(e))), f"block {block} slot {j} != expert {e}"
    assert ctx.device_flags() == 0
    ctx.close()


def test_a_migration_whose_turn_never_comes_gives_up_waiting_and_copies(hx):
    """The migration kernels of a step wait for their turn on the host link, bounded by the clock.
    Through the test hook a kernel is started as number 3 of a step in which nobody ever passes the
    turn on, with the bound set to 300 us: it must wait about that long, then copy exactly the
    selected experts and leave normally, and the stack must step as before afterwards."""
    import time
    H, B = hx
    w = W.Workload("turn_case", 73, 3, 128, 256, 16, 2, 12, 1, "bf16", 0.0, True)
    stack, gates, cache = make_stack(H, w, threads=4, weight_scale=4.0)
    ctx, store = stack.ctx, stack.store
    stack.set_input(W.step_input(w, 0))
    stack.step()
    torch.cuda.synchronize()
    want = stack.x_states.clone()
    idx = np.stack([np.random.default_rng(5).choice(16, size=2, replace=False) for _ in range(12)]).astype(np.int32)
    idx_d = torch.from_numpy(idx).cuda()
    uniq = np.unique(idx)
    torch.cuda.synchronize()
    took = {}
    for seq, wait_us in ((0, 300.0), (3, 300.0), (3, 20000.0)):
        t0 = time.perf_counter()
        ctx.fetch_experts_as_turn(1, idx_d, 12, stack.compute, seq, wait_us)
        torch.cuda.synchronize()
        took[(seq, wait_us)] = time.perf_counter() - t0
        fs = ctx.fetch_stats(1)
        assert fs.n_unique == len(uniq) and fs.bytes_copied == len(uniq) * store.expert_bytes
        for j, e in enumerate(uniq):
            got = _device_bytes(ctx.slot_address(1, j), store.expert_bytes)
            assert np.array_equal(got, store.blob(1, int(e))), f"seq {seq}: slot {j} != expert {e}"
    say(f"  turn hook: {dict((k, round(v * 1e6)) for k, v in took.items())} us")
    assert took[(3, 20000.0)] >= 0.020                 # the kernel cannot start copying before its bound has passed
    assert took[(3, 20000.0)] < 5.0 and took[(3, 300.0)] < 5.0       # ... and it does give up
    with pytest.raises(B.PgmoeError):
        ctx.fetch_experts_as_turn(1, idx_d, 12, stack.compute, 3, 0.0)
    # the turn counter is back at zero: a whole step runs as before, bit for bit
    stack.x_states[1:].zero_()
    torch.cuda.synchronize()
    stack.step()
    torch.cuda.synchronize()
    assert torch.equal(stack.x_states.view(torch.int16), want.view(torch.int16))
    assert ctx.device_flags() == 0
    stack.close()


@pytest.mark.parametrize("shape", ["decode", "gemm"])
def test_pull_fetch_with_too_few_slots_flags_and_zeroes(hx, shape):
    """slots_per_gen smaller than the number of distinct experts: the pull kernel copies the
    first slots_per_gen experts, raises the device flag, and the FFN zeroes the other rows
    (fused kernel for the decode shape, the two tiled GEMMs for 250 rows per expert)."""
    H, B = hx
    if shape == "decode":
        w = W.Workload("noslot_case", 71, 1, 128, 256, 8, 1, 8, 1, "bf16", 0.0, True)
        idx = np.array([[1], [1], [3], [5], [5], [6], [3], [1]], dtype=np.int32)      # distinct: 1, 3, 5, 6
        kept, dropped = (1, 3), (5, 6)
    else:
        w = W.Workload("noslot_gemm_case", 72, 1, 128, 256, 4, 1, 1000, 1, "bf16", 0.0, True)
        idx = np.random.default_rng(9).permutation(np.repeat(np.arange(4, dtype=np.int32), 250)).reshape(-1, 1)
        kept, dropped = (0, 1), (2, 3)
    T, E = w.tokens, w.n_experts
    cfg = H.config_for(w, slots_per_gen=2)
    cache = {}

    def get(b, e):
        cache[e] = W.expert_weights(w, b, e)
        return cache[e]

    store = H.ExpertStore(w, cfg, threads=1, get_expert=get)
    ctx = B.Context(cfg)
    ctx.register_host_experts(store.host, store.expert_stride, store.block_stride)
    comp, copy = torch.cuda.Stream(), torch.cuda.Stream()
    x = W.round_to_bf16(np.random.default_rng(2).standard_normal((T, 128)).astype(np.float32))
    xd, idx_d = H.to_device(x, "bf16"), torch.from_numpy(idx).cuda()
    x_perm = torch.zeros((T, 128), dtype=torch.bfloat16, device="cuda")
    y_perm = torch.full((T, 128), 3.0, dtype=torch.bfloat16, device="cuda")
    row_of = torch.zeros(T, dtype=torch.int32, device="cuda")
    offs = torch.zeros(E + 1, dtype=torch.int32, device="cuda")
    ws = torch.zeros(ctx.workspace_bytes, dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()
    assert ("gemm" in ctx.ffn_kernel_name(T)) == (shape == "gemm")
    assert ctx.fetch_experts(0, idx_d, T, comp, copy) == 4
    ctx.permute(xd, idx_d, T, x_perm, row_of, offs, comp)
    ctx.expert_ffn(0, x_perm, offs, T, y_perm, ws, comp)
    torch.cuda.synchronize()
    assert ctx.device_flags() & 4
    r = R.route(idx, E)
    y = H.to_numpy64(y_perm)
    for e in kept:
        rows = slice(r["offsets"][e], r["offsets"][e + 1])
        ref = R.ffn_rows(x[idx[:, 0] == e], *cache[e])
        assert nerr(y[rows], ref) <= TOL["bf16"]
    for e in dropped:
        assert np.all(y[r["offsets"][e]: r["offsets"][e + 1]] == 0.0)
    ctx.close()


@pytest.mark.parametrize("dtype,T,d,f,E,k,L,offloaded", [
    ("bf16", 40, 128, 256, 16, 2, 4, True), ("bf16", 1, 768, 3072, 8, 1, 3, True), ("bf16", 300, 256, 512, 8, 1, 3, False),
    ("f32", 32, 64, 256, 8, 1, 2, False),
    # decode-sized batches, where the gate kernel groups the tokens itself: at its limit of 256
    # selections, just beyond it (separate grouping kernel again), and with 256 experts
    ("bf16", 16, 128, 256, 32, 16, 3, False), ("bf16", 16, 128, 256, 32, 17, 3, False), ("bf16", 7, 128, 256, 256, 3, 3, True),
    # resident store, smallest gates: the decode-sized expert launch of block i carries the pre-gate that routes block
    # i+1 as an extra workgroup (first two); an expert launch that cannot carry it leaves it to a launch of its own (third)
    ("bf16", 1, 768, 3072, 8, 1, 4, False), ("bf16", 3, 1024, 4096, 16, 2, 4, False), ("bf16", 4, 128, 256, 8, 2, 3, False),
])
def test_stack_step_equals_the_primitive_call_sequence(hx, dtype, T, d, f, E, k, L, offloaded):
    """pgmoe_stack_step (which fuses the partial-sum reduction into the combine and orders the
    fetches itself) must give bit-identical hidden states to the five primitives called one by
    one in the paper's order: pre-gate i on x_i routes block i+1; block 0 has its own gate."""
    H, B = hx
    w = W.Workload("seq_case", 80, L, d, f, E, k, T, 1, dtype, 0.0, offloaded)
    stack, gates, cache = make_stack(H, w, threads=4)
    stack.set_input(W.step_input(w, 0))
    stack.step()
    torch.cuda.synchronize()
    ctx = stack.ctx
    xs = [stack.x_states[0].clone()]
    idx = torch.zeros((L, T, k), dtype=torch.int32, device="cuda")
    prob = torch.zeros((L, T, k), dtype=torch.float32, device="cuda")
    x_perm, y_perm = torch.zeros_like(stack.x_perm), torch.zeros_like(stack.y_perm)
    row_of = torch.zeros(T * k, dtype=torch.int32, device="cuda")
    offs = torch.zeros(E + 1, dtype=torch.int32, device="cuda")
    comp, copy = stack.compute, stack.copy
    ctx.pregate_topk(xs[0], stack.gate_w[0], stack.gate_b[0], T, idx[0], prob[0], None, comp)
    ctx.fetch_experts(0, idx[0], T, comp, copy)
    for i in range(L):
        if i + 1 < L:
            ctx.pregate_topk(xs[i], stack.gate_w[i + 1], stack.gate_b[i + 1], T, idx[i + 1], prob[i + 1], None, comp)
            ctx.fetch_experts(i + 1, idx[i + 1], T, comp, copy)
        ctx.permute(xs[i], idx[i], T, x_perm, row_of, offs, comp)
        ctx.expert_ffn(i, x_perm, offs, T * k, y_perm, stack.workspace, comp)
        y = torch.zeros_like(xs[i])
        xn = torch.zeros_like(xs[i])
        ctx.combine(y_perm, row_of, prob[i], T, y, xs[i], xn, comp)
        torch.cuda.synchronize()
        assert torch.equal(idx[i], stack.topk_idx[i]) and torch.equal(prob[i], stack.topk_prob[i])
        assert torch.equal(row_of, stack.row_of[i]) and torch.equal(offs, stack.expert_offsets[i]), f"block {i}: grouping"
        assert torch.equal(y, stack.y_blocks[i]), f"block {i}: y differs between stack_step and the primitives"
        assert torch.equal(xn, stack.x_states[i + 1])
        xs.append(xn)
    stack.close()


def test_a_step_with_fewer_tokens_than_max_tokens_packs_its_arrays_for_that_T(hx):
    """pgmoe_stack_step lays every per-step array out for the T of the call.  A context created for
    64 tokens, stepped with 5, must give exactly what a context created for 5 tokens gives."""
    H, B = hx
    T, L, d, k, E = 5, 3, 128, 2, 8
    w = small_workload("bf16", T, d, 256, E, k, L=L, offloaded=True, index=61)
    tight, gates, cache = make_stack(H, w, threads=4, weight_scale=4.0)
    tight.set_input(W.step_input(w, 0))
    tight.step()
    st = check_stack_step(H, w, tight, gates, cache, label="tight")
    say(f"  tight context: {st}")
    roomy = H.Stack(w, tight.store, gates=gates, max_tokens=64)

    def packed(t, *shape):      # the first prod(shape) elements of a buffer allocated for 64 tokens
        n = int(np.prod(shape))
        return t.reshape(-1)[:n].view(*shape)

    packed(roomy.x_states, L + 1, T, d)[0].copy_(tight.x_states[0])
    torch.cuda.synchronize()
    roomy.step(T=T)
    torch.cuda.synchronize()
    assert torch.equal(packed(roomy.x_states, L + 1, T, d), tight.x_states)
    assert torch.equal(packed(roomy.y_blocks, L, T, d), tight.y_blocks)
    assert torch.equal(packed(roomy.topk_idx, L, T, k), tight.topk_idx)
    assert torch.equal(packed(roomy.topk_prob, L, T, k), tight.topk_prob)
    assert torch.equal(packed(roomy.row_of, L, T * k), tight.row_of)
    assert torch.equal(roomy.expert_offsets, tight.expert_offsets)
    assert roomy.ctx.device_flags() == 0
    roomy.close()
    tight.close()


STACK_SHAPES = [
    # dtype, T, d, f, E, k, L, offloaded, fetch, pre-gate distance
    ("bf16", 1, 64, 64, 8, 1, 1, True, "pull", 0),        # one block: the step's first migration is also its last
    ("bf16", 3, 128, 192, 12, 2, 2, True, "pull", 0),     # E no multiple of 8 (plain gate kernel), d_ff = 3 * 64
    ("bf16", 50, 256, 320, 4, 4, 3, True, "memcpy", 0),   # every expert selected by every token
    ("bf16", 129, 512, 64, 24, 3, 3, True, "pull", 2),    # more than 256 selections: grouping kernel of its own
    ("bf16", 17, 2048, 128, 8, 2, 2, False, "-", 0),      # largest d_model
    ("bf16", 600, 128, 256, 2, 1, 2, True, "pull", 0),    # 300 rows per expert: the two GEMMs behind a migration
    ("f32", 8, 5, 3, 3, 2, 3, True, "pull", 0),           # 120-byte experts: the pull kernel's 4-byte path
    ("f32", 32, 100, 36, 5, 5, 2, True, "memcpy", 0),
    ("bf16", 5, 64, 64, 256, 8, 4, True, "pull", 3),      # 256 experts, looking three blocks ahead in a four-block stack
    ("bf16", 2, 768, 3072, 8, 2, 2, True, "pull", 0),     # decode kernel with two experts per token
    ("bf16", 4, 1024, 4096, 16, 1, 1, False, "-", 0),     # a single resident block
    ("bf16", 2, 768, 3072, 8, 2, 3, False, "-", 0),       # resident decode: pre-gates carried by the expert launches
]


@pytest.mark.parametrize("dtype,T,d,f,E,k,L,offloaded,fetch,distance", STACK_SHAPES)
def test_stacks_of_unusual_shapes_match_the_oracle(hx, dtype, T, d, f, E, k, L, offloaded, fetch, distance):
    """Corners of the accepted configuration space, each checked block by block against the oracle
    evaluated on the GPU's own hidden states, over two steps."""
    H, B = hx
    say(f"stack shape dtype={dtype} T={T} d={d} f={f} E={E} k={k} L={L} offloaded={offloaded} fetch={fetch} N={distance}")
    w = W.Workload("shape_case", 95, L, d, f, E, k, T, 2, dtype, 0.0, offloaded)
    stack, gates, cache = make_stack(H, w, threads=4, flags=B.FLAG_FETCH_MEMCPY if fetch == "memcpy" else 0,
                                     pregate_distance=distance, weight_scale=4.0 if dtype == "bf16" else 1.0)
    for s in range(2):
        stack.set_input(W.step_input(w, s))
        stack.step()
        st = check_stack_step(H, w, stack, gates, cache, label=f"shape step {s}", distance=max(distance, 1))
        say(f"  step {s}: {st}")
        if offloaded:
            for b in range(L):
                fs = stack.ctx.fetch_stats(b)
                u = len(np.unique(stack.topk_idx[b].cpu().numpy()))
                assert fs.n_unique == u and fs.bytes_copied == u * w.expert_bytes
    assert stack.ctx.device_flags() == 0
    stack.close()


# ------------------------------------------------------------------------------ comparison schedules
@pytest.mark.parametrize("schedule,fetch,offloaded", [
    ("on_demand", "pull", True), ("on_demand", "memcpy", True), ("prefetch_all", "pull", True),
    ("prefetch_all", "memcpy", True), ("on_demand", "-", False),
])
def test_comparison_schedules_match_the_conventional_oracle(hx, schedule, fetch, offloaded):
    """The paper's comparison systems on the same kernels: conventional wiring (every block routed
    by its own gate on its own input), experts fetched on demand or all prefetched; with a
    resident store this is the GPU-only design point."""
    H, B = hx
    w = W.Workload("sched_case", 90, 4, 256, 512, 16, 2, 24, 1, "bf16", 1.1, offloaded)
    stack, gates, cache = make_stack(H, w, threads=4, flags=B.FLAG_FETCH_MEMCPY if fetch == "memcpy" else 0)
    stack.ctx.set_schedule(B.SCHED_ON_DEMAND if schedule == "on_demand" else B.SCHED_PREFETCH_ALL)
    stack.ctx.fetch_timing(True)
    for s in range(2):
        stack.set_input(W.step_input(w, s))
        stack.step()
        st = check_stack_step(H, w, stack, gates, cache, label=f"{schedule} step {s}", wiring="conventional")
        say(f"  {schedule}/{fetch} step {s}: {st}")
        if offloaded:
            for b in range(w.n_blocks):
                fs = stack.ctx.fetch_stats(b)
                u = len(np.unique(stack.topk_idx[b].cpu().numpy()))
                expect = w.n_experts if schedule == "prefetch_all" else u
                assert fs.n_copied == expect and fs.bytes_copied == expect * w.expert_bytes
    assert stack.ctx.device_flags() == 0
    stack.close()


# ------------------------------------------------------------------------------ expert cache
@pytest.mark.parametrize("policy,shape,distance", [("lru", "decode", 0), ("lfu", "decode", 0), ("lifo", "decode", 0),
                                                   ("lru", "gemm", 0), ("lru", "decode", 2)])
def test_expert_cache_changes_the_copies_not_the_results(hx, policy, shape, distance):
    """A stack with an expert cache gives bit-identical hidden states to the same stack without
    one, and the device's hit / copy counts equal the reference model of the policy.  The "gemm"
    shape sends 256 rows to each expert, so the two tiled GEMM kernels find their weights through
    the cache's pointer table too."""
    from oracle.cache_policy import ExpertCache, LRU, LFU, LIFO
    H, B = hx
    pol = {"lru": (B.CACHE_LRU, LRU), "lfu": (B.CACHE_LFU, LFU), "lifo": (B.CACHE_LIFO, LIFO)}[policy]
    if shape == "decode":
        w = W.Workload("cache_case", 95, 4, 256, 512, 32, 2, 12, 1, "bf16", 1.1, True)
        C = 6
    else:
        w = W.Workload("cache_gemm_case", 96, 3, 256, 512, 4, 1, 1024, 1, "bf16", 0.0, True)
        C = 2
    cfg = H.config_for(w)
    store = H.ExpertStore(w, cfg, threads=4)
    gates = W.gate_tensors(w)
    plain = H.Stack(w, store, gates=gates, pregate_distance=distance)
    cached = H.Stack(w, store, gates=gates, cache_slots=C, cache_policy=pol[0], pregate_distance=distance)
    models = [ExpertCache(C, pol[1]) for _ in range(w.n_blocks)]
    hits_total = 0
    if shape == "gemm":
        assert "gemm" in cached.ctx.ffn_kernel_name(w.tokens * w.top_k)
    for s in range(10 if shape == "decode" else 4):
        x0 = W.step_input(w, s)
        for st in (plain, cached):
            st.set_input(x0)
            st.step()
        torch.cuda.synchronize()
        assert torch.equal(plain.x_states, cached.x_states), f"step {s}: the cache changed the hidden states"
        assert torch.equal(plain.topk_idx, cached.topk_idx)
        for b in range(w.n_blocks):
            ref = models[b].fetch(np.unique(cached.topk_idx[b].cpu().numpy()))
            fs = cached.ctx.fetch_stats(b)
            assert (fs.n_unique, fs.cache_hits, fs.n_copied) == (ref["unique"], ref["hits"], len(ref["copies"])), \
                f"step {s} block {b}: device {(fs.n_unique, fs.cache_hits, fs.n_copied)} vs model {ref}"
            assert fs.bytes_copied == len(ref["copies"]) * w.expert_bytes
            hits_total += fs.cache_hits
    # the trace of a cached stack: every block's copy time (the cache-aware kernel's own clock readings)
    # lies inside the kernel's duration, and a block that copied nothing spent next to no time copying
    cached.ctx.trace(True)
    cached.set_input(W.step_input(w, 0))
    cached.step()
    torch.cuda.synchronize()
    for b in range(w.n_blocks):
        tr, fs = cached.ctx.block_trace(b), cached.ctx.fetch_stats(b)
        models[b].fetch(np.unique(cached.topk_idx[b].cpu().numpy()))      # keep the reference model in step
        assert 0.0 <= tr.copy_ms <= tr.fetch_ms + 0.05, (b, tr.copy_ms, tr.fetch_ms)
        if fs.n_copied == 0:
            assert tr.copy_ms < 0.05
    cached.ctx.trace(False)
    say(f"  cache {policy}: {hits_total} hits over 10 steps x {w.n_blocks} blocks")
    assert hits_total > 0
    assert cached.ctx.device_flags() == 0
    plain.close()
    cached.close()


def test_streams_of_a_stack_run_side_by_side(hx):
    """The harness asks the library whether its three streams (compute, copy, the context's own
    copy stream) share a hardware queue and replaces streams until none do; a stream paired with
    itself is reported as shared."""
    H, B = hx
    w = small_workload("bf16", 4, 128, 256, 8, 1, L=2, offloaded=True, index=63)
    stacks = []
    for _ in range(5):          # later stacks of a process get other streams, hence other queues
        stack, gates, cache = make_stack(H, w, threads=2)
        assert stack.shared_streams == 0, f"stream pairs that share a hardware queue: {stack.shared_streams}"
        assert stack.ctx.check_streams(stack.compute, stack.copy) == 0
        stacks.append(stack)
    assert stacks[0].ctx.check_streams(stacks[0].compute, stacks[0].compute) & B.STREAMS_COMPUTE_COPY
    for stack in stacks:
        stack.close()
