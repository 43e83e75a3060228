"""Seeded synthetic inputs for the pre-gated MoE block (shared by the CPU oracle's
tests and the HIP path's tests and benchmark).

This module holds no arithmetic of the method itself: it draws Gaussian weights and
activations of the Switch-Transformer shapes (Table "model_config" of the paper gives the
layer/expert counts; the five workloads below take d_model/d_ff/E/L from there), rounds
them to the storage type, and builds the Zipf-shaped gate bias used by the skewed
workloads.  Every array is a pure function of (workload, tag, block, expert, step), so a
test can regenerate one expert's weights without materialising the whole store.

Storage convention: a "bf16" workload returns float32 arrays whose values are exactly
representable in bfloat16 (rounded to nearest even here, once), plus `to_bf16_bits` to get
the 16-bit patterns.  Both consumers therefore see identical bits.
"""
from __future__ import annotations

import dataclasses
import functools
from concurrent.futures import ThreadPoolExecutor

import numpy as np

BASE_SEED = 23081206 * 10

# tags for the seed sub-streams (fixed integers so that streams never collide)
_TAG_GATE0, _TAG_PREGATE, _TAG_W1, _TAG_W2, _TAG_BIAS, _TAG_X = 1, 2, 3, 4, 5, 6


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    index: int            # position in the configuration list (part of the seed)
    n_blocks: int         # L: MoE blocks in the stack
    d_model: int
    d_ff: int
    n_experts: int
    top_k: int
    tokens: int           # T: tokens per step
    steps: int
    dtype: str            # "f32" or "bf16" (storage of x, gate weights, expert weights)
    zipf_s: float = 0.0   # 0 => no gate bias; else Zipf exponent of expert popularity
    offloaded: bool = True  # experts live in pinned host memory (False: all resident)

    @property
    def seed(self) -> int:
        return BASE_SEED + self.index

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    @property
    def expert_bytes(self) -> int:
        return 2 * self.d_model * self.d_ff * self.elem_bytes

    def replace(self, **kw) -> "Workload":
        return dataclasses.replace(self, **kw)


CONFIGS = {
    # tiny fp32 stack, all experts resident
    "cfg1": Workload("cfg1", 0, 2, 64, 256, 8, 1, 32, 1, "f32", 0.0, False),
    # Switch-Base-8 decode, batch 1, 128 steps, offloaded
    "cfg2": Workload("cfg2", 1, 6, 768, 3072, 8, 1, 1, 128, "bf16", 0.0, True),
    # Switch-Base-64 decode, 16 tokens/step, Zipf(1.1) popularity, offloaded
    "cfg3": Workload("cfg3", 2, 6, 768, 3072, 64, 1, 16, 128, "bf16", 1.1, True),
    # Switch-Base-128 prefill, 8 x 512 tokens, resident (and an offloaded variant)
    "cfg4": Workload("cfg4", 3, 6, 768, 3072, 128, 1, 4096, 1, "bf16", 0.0, False),
    "cfg4_offloaded": Workload("cfg4_offloaded", 3, 6, 768, 3072, 128, 1, 4096, 1, "bf16", 0.0, True),
    # Switch-Large-128 decode, 64 tokens/step, Zipf(1.1), top-1 and top-2, offloaded
    "cfg5": Workload("cfg5", 4, 12, 1024, 4096, 128, 1, 64, 64, "bf16", 1.1, True),
    "cfg5_top2": Workload("cfg5_top2", 4, 12, 1024, 4096, 128, 2, 64, 64, "bf16", 1.1, True),
    # supplementary shape (not one of the five): Switch-Base-8 prefill, ~512 tokens/expert
    "base8_prefill": Workload("base8_prefill", 5, 6, 768, 3072, 8, 1, 4096, 1, "bf16", 0.0, False),
}

# Activated-expert sweep (the paper's micro-benchmark on Switch-Base-64, Sec. VI-D): batch 1 and
# the number of activated experts forced from 1 to all 64.  Every point shares one seed index, so
# the weights are the same and only top_k changes.
SWEEP_K = (1, 2, 4, 8, 16, 32, 64)
for _k in SWEEP_K:
    CONFIGS[f"sweep64_k{_k}"] = Workload(f"sweep64_k{_k}", 6, 6, 768, 3072, 64, _k, 1, 32, "bf16", 0.0, True)


# ----------------------------------------------------------------------------- storage
def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """float32 -> float32 holding the nearest-even bfloat16 value (finite inputs)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    out = ((u + r) >> np.uint32(16)) << np.uint32(16)
    return out.view(np.float32)


def to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """float32 array of bf16-representable values -> uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    return (u >> np.uint32(16)).astype(np.uint16)


def from_bf16_bits(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _store(w: Workload, a: np.ndarray) -> np.ndarray:
    return a if w.dtype == "f32" else round_to_bf16(a)


def _rng(w: Workload, tag: int, a: int = 0, b: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([w.seed, tag, a, b])))


def _normal(w: Workload, tag: int, a: int, b: int, shape, scale: float) -> np.ndarray:
    g = _rng(w, tag, a, b).standard_normal(shape, dtype=np.float32)
    if scale != 1.0:
        g *= np.float32(scale)
    return _store(w, g)


# ----------------------------------------------------------------------------- tensors
def gate0_weight(w: Workload) -> np.ndarray:
    """Conventional gate of block 0: [d_model, E] ~ N(0, 0.02)."""
    return _normal(w, _TAG_GATE0, 0, 0, (w.d_model, w.n_experts), 0.02)


def pregate_weight(w: Workload, block: int) -> np.ndarray:
    """Pre-gate that sits in `block` and routes block+1: [d_model, E] ~ N(0, 0.02)."""
    if not 0 <= block < w.n_blocks - 1:
        raise ValueError("the last block has no pre-gate")
    return _normal(w, _TAG_PREGATE, block, 0, (w.d_model, w.n_experts), 0.02)


def expert_weights(w: Workload, block: int, expert: int):
    """(W1 [d_model, d_ff], W2 [d_ff, d_model]) ~ N(0, 0.02), logical row-major layout."""
    w1 = _normal(w, _TAG_W1, block, expert, (w.d_model, w.d_ff), 0.02)
    w2 = _normal(w, _TAG_W2, block, expert, (w.d_ff, w.d_model), 0.02)
    return w1, w2


def step_input(w: Workload, step: int) -> np.ndarray:
    """Hidden states entering block 0 at a decode step (or the prefill batch): [T, d] ~ N(0,1)."""
    return _normal(w, _TAG_X, step, 0, (w.tokens, w.d_model), 1.0)


def zipf_probabilities(n: int, s: float) -> np.ndarray:
    r = np.arange(1, n + 1, dtype=np.float64)
    q = r ** (-s)
    return q / q.sum()


@functools.lru_cache(maxsize=None)
def zipf_bias_scale(n_experts: int, s: float, sigma_z: float) -> float:
    """Scale c of the bias b = c * ln q that makes the most popular expert win the argmax
    of (b + N(0, sigma_z^2) noise) with probability q_1.

    With Gumbel noise of scale c the argmax would follow q exactly; the unbiased logits here
    are Gaussian, whose tails are lighter, so c is found by bisection on a fixed seeded
    sample (the result is a pure function of the arguments)."""
    q = zipf_probabilities(n_experts, s)
    lq = np.log(q)
    n = 20000
    noise = np.random.Generator(np.random.PCG64(20230812)).standard_normal((n, n_experts)) * sigma_z
    lo, hi = 0.0, 2.0 * sigma_z
    for _ in range(24):
        mid = 0.5 * (lo + hi)
        share = np.count_nonzero((noise + mid * lq).argmax(1) == 0) / n
        if share > q[0]:
            hi = mid
        else:
            lo = mid
    return 0.5 * (lo + hi)


def gate_bias(w: Workload, gate: int):
    """Additive logit bias [E] float32 that makes expert popularity roughly Zipf(s), or None.

    gate = 0 is block 0's conventional gate, gate = 1 + i is the pre-gate in block i.
    b_e = c * ln q_{pi(e)} with q the Zipf pmf, pi a seeded permutation per gate and c from
    zipf_bias_scale for logits of spread sigma_z = 0.02 * sqrt(d_model)."""
    if w.zipf_s <= 0.0:
        return None
    q = zipf_probabilities(w.n_experts, w.zipf_s)
    perm = _rng(w, _TAG_BIAS, gate, 0).permutation(w.n_experts)
    c = zipf_bias_scale(w.n_experts, w.zipf_s, 0.02 * float(np.sqrt(w.d_model)))
    return (c * np.log(q[perm])).astype(np.float32)


def gate_tensors(w: Workload):
    """List over gates g = 0..L-1 of (weight, bias): g = 0 conventional, g >= 1 pre-gate g-1."""
    out = [(gate0_weight(w), gate_bias(w, 0))]
    for i in range(w.n_blocks - 1):
        out.append((pregate_weight(w, i), gate_bias(w, 1 + i)))
    return out


def for_each_expert(w: Workload, fn, threads: int = 8, blocks=None) -> None:
    """Call fn(block, expert, W1, W2) for every expert, generating in a thread pool.

    numpy's generators release the GIL, so this scales over host cores; fn must be
    thread-safe for distinct (block, expert)."""
    blocks = range(w.n_blocks) if blocks is None else blocks
    jobs = [(b, e) for b in blocks for e in range(w.n_experts)]

    def run(be):
        b, e = be
        w1, w2 = expert_weights(w, b, e)
        fn(b, e, w1, w2)

    if threads <= 1:
        for be in jobs:
            run(be)
        return
    with ThreadPoolExecutor(max_workers=threads) as pool:
        list(pool.map(run, jobs))
