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
