"""GPU parity at the full size of the stated workloads: every block of the stack, every token,
in the launch configuration the benchmark times (the migration engine the library picks for the
configuration, no fetch timing, no tracing) unless a case says otherwise.

Each block is checked in shadow mode against the CPU oracle (the oracle evaluates block i on the
GPU's own x_{i-1} for the routing and x_i for the experts).  Expert weights are regenerated from
the seed on a thread pool block by block instead of being kept (the Switch-Large-128 store alone
is 25.8 GB), and workloads that share a seed index (top-1 and top-2 of Switch-Large-128; the
resident and the offloaded prefill) share one expert store.
"""
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest

torch = pytest.importorskip("torch")

import workloads as W

from test_gpu_parity import HOST_THREADS, check_stack_step, say

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def hx():
    from paper_2308_12066_amd import binding, harness
    assert torch.cuda.is_available()
    return harness, binding


class RegeneratedExperts:
    """expert(block, e) -> (W1, W2) as bf16 bit patterns, regenerated from the workload's seed.
    prefetch(block, experts) generates a block's experts on a thread pool and drops the block
    before it, so at most one block's selected experts are held."""

    def __init__(self, w, threads=HOST_THREADS):
        self.w, self.threads, self.have = w, threads, {}

    def _gen(self, be):
        w1, w2 = W.expert_weights(self.w, *be)
        return be, (W.to_bf16_bits(w1), W.to_bf16_bits(w2))

    def prefetch(self, block, experts):
        self.have = {be: v for be, v in self.have.items() if be[0] == block}
        missing = [(block, int(e)) for e in experts if (block, int(e)) not in self.have]
        with ThreadPoolExecutor(max_workers=self.threads) as pool:
            self.have.update(pool.map(self._gen, missing))

    def __call__(self, block, e):
        if (block, e) not in self.have:
            self.prefetch(block, [e])
        return self.have[(block, e)]


def run_case(H, B, name, store, steps, fetch, timing, first_step=0):
    w = W.CONFIGS[name]
    gates = W.gate_tensors(w)
    stack = H.Stack(w, store, gates=gates, flags={"memcpy": B.FLAG_FETCH_MEMCPY, "auto": B.FLAG_FETCH_AUTO}.get(fetch, 0))
    if fetch == "auto":      # what the benchmark runs: the library picks the engine from the configuration
        assert stack.ctx.migration_engine == ("copy_engine" if w.top_k * w.tokens * w.expert_bytes >= B.AUTO_COPY_ENGINE_BYTES
                                              and w.n_experts * w.expert_bytes >= B.AUTO_COPY_ENGINE_BYTES else "pull")
    stack.ctx.fetch_timing(timing)
    experts = RegeneratedExperts(w)
    near = tot = 0
    worst = 0.0
    for s in range(first_step, first_step + steps):
        stack.set_input(W.step_input(w, s))
        stack.step()
        st = check_stack_step(H, w, stack, gates, experts, label=f"{name} step {s}")
        near += st["near_tie"]
        tot += st["tokens"]
        worst = max(worst, st["max_err"])
        if steps <= 4 or s % 16 == 0:
            say(f"  {name} step {s}: {st}")
        if w.offloaded:
            idx = stack.topk_idx.cpu().numpy()
            u = [len(np.unique(idx[b])) for b in range(w.n_blocks)]
            for b in range(w.n_blocks):
                fs = stack.ctx.fetch_stats(b)
                assert fs.n_unique == u[b] and fs.bytes_copied == u[b] * w.expert_bytes, f"{name} step {s} block {b}"
                assert fs.resident_slots <= u[b] + (u[b - 1] if b else 0)      # peak-memory rule of Sec. IV-C
    say(f"  {name} ({fetch}, fetch timing {'on' if timing else 'off'}): {steps} steps x {w.n_blocks} blocks x {w.tokens} tokens, "
        f"near-tie tokens exempted {near} of {tot}, worst block error {worst:.2e}")
    assert stack.ctx.device_flags() == 0
    stack.close()


def test_switch_large_128_all_twelve_blocks_top1_and_top2(hx):
    """Switch-Large-128 decode (the largest workload): 12 blocks, 64 tokens per step, 25.8 GB of
    experts in pinned host memory, top-1 and top-2 routing, both migration engines."""
    H, B = hx
    w = W.CONFIGS["cfg5"]
    say(f"full depth: Switch-Large-128, L={w.n_blocks}, building the expert store")
    store = H.ExpertStore(w, H.config_for(w), threads=HOST_THREADS)
    run_case(H, B, "cfg5", store, steps=2, fetch="auto", timing=False)
    run_case(H, B, "cfg5_top2", store, steps=2, fetch="pull", timing=False)
    run_case(H, B, "cfg5_top2", store, steps=1, fetch="auto", timing=True, first_step=2)
    run_case(H, B, "cfg5", store, steps=1, fetch="pull", timing=False, first_step=2)


def test_switch_base_128_prefill_all_six_blocks_resident_and_offloaded(hx):
    """The 4096-token prefill over 128 experts, six blocks, every token of every block, with the
    experts resident in HBM and again with them offloaded."""
    H, B = hx
    w = W.CONFIGS["cfg4"]
    say(f"full depth: Switch-Base-128 prefill, L={w.n_blocks}, building the expert store")
    store = H.ExpertStore(w, H.config_for(w), threads=HOST_THREADS)
    run_case(H, B, "cfg4", store, steps=1, fetch="-", timing=False)
    run_case(H, B, "cfg4_offloaded", store, steps=1, fetch="auto", timing=False)


def test_switch_base_8_and_64_decode_over_many_steps(hx):
    """Batch-1 decode of the 8-expert model over all of its 128 steps and the 16-token decode of the
    64-expert model over 16, all six blocks, untimed streams."""
    H, B = hx
    for name, steps in (("cfg2", 128), ("cfg3", 16)):
        w = W.CONFIGS[name]
        store = H.ExpertStore(w, H.config_for(w), threads=HOST_THREADS)
        run_case(H, B, name, store, steps=steps, fetch="auto", timing=False)
