"""pgmoe_expert_ffn_static (the expert FFN for callers that cannot allocate: its scratch is a
buffer inside the library's device image) against pgmoe_expert_ffn with a caller workspace:
bit-identical outputs, on two calls in a row of which the second is smaller, for the three bf16
kernel families and the float32 kernels.  (That a launch which does not fit the buffer is refused
is checked on a host-only context, which cannot launch anything: tests/test_abi_host.py.)"""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

import workloads as W

pytestmark = pytest.mark.gpu


def one_call(H, B, ctx, w, counts, seed, static):
    """Rows grouped by expert (counts[e] rows each) through the expert FFN of block 0."""
    E, d = w.n_experts, w.d_model
    n = int(sum(counts))
    x = np.random.default_rng(seed).standard_normal((n, d)).astype(np.float32)
    xd = H.to_device(W.round_to_bf16(x) if w.dtype == "bf16" else x, w.dtype)
    offs = torch.from_numpy(np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)).cuda()
    y = torch.full((n, d), 7.0, dtype=xd.dtype, device="cuda")
    if static:
        ctx.expert_ffn_static(0, xd, offs, n, y)
    else:
        ws = torch.full((ctx.workspace_bytes,), 0x5A, dtype=torch.uint8, device="cuda")
        ctx.expert_ffn(0, xd, offs, n, y, ws)
    torch.cuda.synchronize()
    return y


@pytest.mark.parametrize("dtype,d,f,E,first,second", [
    ("bf16", 768, 3072, 8, [9, 0, 16, 1, 0, 30, 2, 6], [1, 0, 0, 0, 0, 0, 0, 0]),     # fused kernel with partial sums, then the decode kernel
    ("bf16", 128, 256, 2, [300, 260], [7, 40]),                                      # the two tiled GEMMs, then the fused kernel
    ("f32", 64, 256, 8, [3, 0, 5, 1, 0, 0, 2, 4], [0, 2, 0, 0, 0, 0, 0, 1]),
])
def test_static_scratch_ffn_equals_the_workspace_ffn(dtype, d, f, E, first, second):
    from paper_2308_12066_amd import binding as B, harness as H
    rows = max(sum(first), sum(second))
    w = W.Workload("static_case", 77, 1, d, f, E, 1, rows, 1, dtype, 0.0, False)
    cfg = H.config_for(w)
    store = H.ExpertStore(w, cfg, threads=4)
    ctx = B.Context(cfg)
    ctx.register_resident_experts(store.to_hbm(), store.expert_stride, store.block_stride)
    names = []
    for call, counts in enumerate((first, second)):
        names.append(ctx.ffn_kernel_name(int(sum(counts))))
        print(f"static scratch FFN: dtype={dtype} d={d} f={f} rows={sum(counts)} kernel={names[-1]}", flush=True)
        got = one_call(H, B, ctx, w, counts, 100 + call, static=True)
        want = one_call(H, B, ctx, w, counts, 100 + call, static=False)
        assert torch.equal(got.view(torch.int16 if dtype == "bf16" else torch.int32),
                           want.view(torch.int16 if dtype == "bf16" else torch.int32)), f"call {call} ({names[-1]})"
        assert float(want.float().abs().max()) > 0.0
    if dtype == "bf16":
        assert names[0] != names[1]      # the two calls went through different kernels
    assert ctx.device_flags() == 0
    ctx.close()


def test_static_scratch_ffn_replays_from_a_captured_graph():
    """What the entry point is for: grouping, expert FFN and combine captured into one HIP graph
    with no workspace to bring, replayed several times with the program's own eager work in
    between; every replay gives the bits the eager calls give."""
    from paper_2308_12066_amd import binding as B, harness as H
    T, d, f, E, k = 24, 768, 3072, 8, 2
    w = W.Workload("static_graph", 79, 1, d, f, E, k, T, 1, "bf16", 0.0, False)
    cfg = H.config_for(w)
    store = H.ExpertStore(w, cfg, threads=4)
    ctx = B.Context(cfg)
    ctx.register_resident_experts(store.to_hbm(), store.expert_stride, store.block_stride)
    g = np.random.default_rng(3)
    xs = [H.to_device(W.round_to_bf16(g.standard_normal((T, d)).astype(np.float32)), "bf16") for _ in range(3)]
    idx = torch.from_numpy(np.stack([g.choice(E, size=k, replace=False) for _ in range(T)]).astype(np.int32)).cuda()
    prob = torch.from_numpy(g.random((T, k)).astype(np.float32)).cuda()
    x = torch.zeros((T, d), dtype=torch.bfloat16, device="cuda")
    x_perm, y_perm = torch.zeros((T * k, d), dtype=torch.bfloat16, device="cuda"), torch.zeros((T * k, d), dtype=torch.bfloat16, device="cuda")
    row_of = torch.zeros(T * k, dtype=torch.int32, device="cuda")
    offs = torch.zeros(E + 1, dtype=torch.int32, device="cuda")
    y = torch.zeros((T, d), dtype=torch.bfloat16, device="cuda")
    stream = torch.cuda.Stream()

    def block():
        ctx.permute(x, idx, T, x_perm, row_of, offs, stream)
        ctx.expert_ffn_static(0, x_perm, offs, T * k, y_perm, stream)
        ctx.combine(y_perm, row_of, prob, T, y, None, None, stream)

    eager = []
    for xi in xs:                                    # eager results; also warms every kernel up
        x.copy_(xi)
        torch.cuda.synchronize()
        block()
        torch.cuda.synchronize()
        eager.append(y.clone())
    assert not torch.equal(eager[0], eager[1])
    graph = torch.cuda.CUDAGraph()
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=stream):
        block()
    torch.cuda.synchronize()
    for rep in range(2):
        for xi, want in zip(xs, eager):
            x.copy_(xi)
            y.zero_()                                # eager work between the replays
            y_perm.zero_()
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(y.view(torch.int16), want.view(torch.int16)), f"replay {rep}"
    del graph
    assert ctx.device_flags() == 0
    ctx.close()
