"""Plumbing around the C ABI for tests and the benchmark: torch supplies device memory, pinned
host memory and streams; every computation is done by libpgmoe.

Nothing here computes any part of the MoE block.
"""
from __future__ import annotations

import threading

import numpy as np
import torch

import workloads as W

from . import binding as B


def abi_dtype(w: W.Workload) -> int:
    return B.F32 if w.dtype == "f32" else B.BF16


def config_for(w: W.Workload, max_tokens=None, slots_per_gen=0, flags=0, cache_slots=0, cache_policy=0,
               pregate_distance=0) -> B.Config:
    return B.make_config(w.d_model, w.d_ff, w.n_experts, w.top_k, w.n_blocks, max_tokens or w.tokens, abi_dtype(w),
                         slots_per_gen, flags, cache_slots, cache_policy, pregate_distance)


def to_device(a: np.ndarray, dtype: str, device="cuda") -> torch.Tensor:
    """float32 numpy values (bf16-representable when dtype == 'bf16') -> device tensor of the storage type."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    if dtype == "f32":
        return torch.from_numpy(a).to(device)
    bits = W.to_bf16_bits(a).view(np.int16)
    return torch.from_numpy(bits).to(device).view(torch.bfloat16)


def to_numpy64(t: torch.Tensor) -> np.ndarray:
    """Device tensor (f32 / bf16 / int) -> float64 numpy, exact."""
    return t.detach().to("cpu").to(torch.float64).numpy()


class ExpertStore:
    """All experts of all blocks as packed blobs, [L][E][expert_bytes], in pinned host memory
    (the paper's CPU-side expert store) and optionally mirrored in HBM (GPU-only design point)."""

    def __init__(self, w: W.Workload, cfg: B.Config, threads: int = 8, blocks=None, experts=None,
                 get_expert=None, pinned: bool = True):
        self.w, self.cfg = w, cfg
        self.expert_bytes = B.expert_bytes(cfg)
        self.expert_stride = (self.expert_bytes + 255) // 256 * 256
        self.block_stride = self.expert_stride * w.n_experts
        total = self.block_stride * w.n_blocks
        pin = pinned and torch.cuda.is_available()
        self.host = torch.empty(total, dtype=torch.uint8, pin_memory=pin)
        self.device = None
        base = self.host.numpy()
        get = get_expert or (lambda b, e: W.expert_weights(w, b, e))
        lock = threading.Lock()
        self.filled = set()

        def fill(b, e):
            w1, w2 = get(b, e)
            if w.dtype == "bf16":
                w1, w2 = W.to_bf16_bits(w1), W.to_bf16_bits(w2)
            else:
                w1, w2 = np.ascontiguousarray(w1, np.float32), np.ascontiguousarray(w2, np.float32)
            off = b * self.block_stride + e * self.expert_stride
            B.pack_expert(cfg, w1, w2, base[off: off + self.expert_bytes])
            with lock:
                self.filled.add((b, e))

        jobs = [(b, e) for b in (range(w.n_blocks) if blocks is None else blocks)
                for e in (range(w.n_experts) if experts is None else experts)]
        if threads <= 1:
            for b, e in jobs:
                fill(b, e)
        else:
            from concurrent.futures import ThreadPoolExecutor
            with ThreadPoolExecutor(max_workers=threads) as pool:
                list(pool.map(lambda be: fill(*be), jobs))

    def blob(self, b: int, e: int) -> np.ndarray:
        off = b * self.block_stride + e * self.expert_stride
        return self.host.numpy()[off: off + self.expert_bytes]

    def to_hbm(self) -> torch.Tensor:
        if self.device is None:
            self.device = self.host.to("cuda", non_blocking=False)
        return self.device


class Stack:
    """One pre-gated MoE stack on the GPU: context, gate tensors, per-step buffers, two streams."""

    def __init__(self, w: W.Workload, store: ExpertStore, gates=None, max_tokens=None, slots_per_gen=0, flags=0,
                 cache_slots=0, cache_policy=0, pregate_distance=0):
        self.w = w
        self.cfg = config_for(w, max_tokens=max_tokens, slots_per_gen=slots_per_gen, flags=flags,
                              cache_slots=cache_slots, cache_policy=cache_policy, pregate_distance=pregate_distance)
        self.ctx = B.Context(self.cfg)
        self.store = store
        T, d, k, E, L = self.cfg.max_tokens, w.d_model, w.top_k, w.n_experts, w.n_blocks
        tdt = torch.float32 if w.dtype == "f32" else torch.bfloat16
        gates = gates if gates is not None else W.gate_tensors(w)
        self.gate_w = [to_device(gw, w.dtype) for gw, _ in gates]
        self.gate_b = [None if gb is None else torch.from_numpy(np.ascontiguousarray(gb, np.float32)).cuda()
                       for _, gb in gates]
        dev = "cuda"
        self.x_states = torch.zeros((L + 1, T, d), dtype=tdt, device=dev)
        self.y_blocks = torch.zeros((L, T, d), dtype=tdt, device=dev)
        self.topk_idx = torch.zeros((L, T, k), dtype=torch.int32, device=dev)
        self.topk_prob = torch.zeros((L, T, k), dtype=torch.float32, device=dev)
        self.row_of = torch.zeros((L, T * k), dtype=torch.int32, device=dev)
        self.expert_offsets = torch.zeros((L, E + 1), dtype=torch.int32, device=dev)
        self.x_perm = torch.zeros((T * k, d), dtype=tdt, device=dev)
        self.y_perm = torch.zeros((T * k, d), dtype=tdt, device=dev)
        self.workspace = torch.zeros(self.ctx.workspace_bytes, dtype=torch.uint8, device=dev)
        self.compute = torch.cuda.Stream()
        self.copy = torch.cuda.Stream()
        # streams that share a hardware queue would serialise migration and compute without any
        # error: ask the library, and take another copy stream while ours shares one with compute
        self.shared_streams = self.ctx.check_streams(self.compute, self.copy)
        for _ in range(8):
            if not self.shared_streams & B.STREAMS_COMPUTE_COPY:
                break
            self.copy = torch.cuda.Stream()
            self.shared_streams = self.ctx.check_streams(self.compute, self.copy)
        if w.offloaded:
            self.ctx.register_host_experts(store.host, store.expert_stride, store.block_stride)
        else:
            self.ctx.register_resident_experts(store.to_hbm(), store.expert_stride, store.block_stride)
        self.bufs = self.ctx.make_step_buffers(self.gate_w, self.gate_b, self.x_states, self.y_blocks, self.topk_idx,
                                               self.topk_prob, self.row_of, self.expert_offsets, self.x_perm,
                                               self.y_perm, self.workspace)
        torch.cuda.synchronize()

    def set_input(self, x0: np.ndarray):
        self.x_states[0].copy_(to_device(x0, self.w.dtype))
        torch.cuda.synchronize()

    def step(self, T=None):
        """One pass over all blocks (asynchronous on the compute / copy streams)."""
        self.ctx.stack_step(self.bufs, self.cfg.max_tokens if T is None else T, self.compute, self.copy)

    def close(self):
        torch.cuda.synchronize()
        self.ctx.close()
