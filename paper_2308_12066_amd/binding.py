"""Thin ctypes binding of libpgmoe.so: argument marshalling only.

Every step of the path runs inside the library's HIP kernels; torch is used by callers for
device memory and streams.  The functions mirror include/pgmoe.h one to one.  Importing this
module loads the library and raises if it is missing: there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, Structure, byref, c_char_p, c_float, c_int, c_int32, c_int64, c_size_t, c_uint32, c_void_p

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libpgmoe.so")

OK, EINVAL, ENOTPINNED, ENOSLOT, EBADINDEX, EHIP, ENODEVICE, ESTATE = 0, -1, -2, -3, -4, -5, -6, -7
F32, BF16 = 0, 1
STREAMS_COMPUTE_COPY, STREAMS_COMPUTE_OWN, STREAMS_COPY_OWN = 1, 2, 4
FLAG_HOST_ONLY = 1
FLAG_FETCH_MEMCPY = 2
FLAG_FETCH_AUTO = 4
AUTO_COPY_ENGINE_BYTES = 256 << 20
SCHED_PREGATED, SCHED_ON_DEMAND, SCHED_PREFETCH_ALL = 0, 1, 2
CACHE_LRU, CACHE_LFU, CACHE_LIFO = 0, 1, 2
MAX_CACHE_SLOTS = 64
MAX_PREGATE_DISTANCE = 3
MAX_EXPERTS = 256
STATIC_SCRATCH_BYTES = 32 << 20

EXPORTS = [
    "pgmoe_create", "pgmoe_destroy", "pgmoe_last_error", "pgmoe_expert_bytes", "pgmoe_workspace_bytes",
    "pgmoe_pack_expert", "pgmoe_unpack_expert", "pgmoe_pregate_topk", "pgmoe_register_host_experts",
    "pgmoe_register_resident_experts", "pgmoe_fetch_experts", "pgmoe_get_fetch_stats", "pgmoe_unique_experts",
    "pgmoe_permute", "pgmoe_expert_ffn", "pgmoe_combine", "pgmoe_stack_step", "pgmoe_device_flags",
    "pgmoe_ffn_timing_begin", "pgmoe_ffn_timing_end", "pgmoe_slot_address", "pgmoe_fetch_timing", "pgmoe_trace", "pgmoe_get_block_trace", "pgmoe_fetch_all_experts", "pgmoe_set_schedule",
    "pgmoe_ffn_kernel_name", "pgmoe_set_nonmoe_standin", "pgmoe_check_streams", "pgmoe_expert_ffn_static", "pgmoe_migration_engine", "pgmoe_fetch_experts_as_turn",
]


class Config(Structure):
    _fields_ = [("d_model", c_int32), ("d_ff", c_int32), ("n_experts", c_int32), ("top_k", c_int32),
                ("n_blocks", c_int32), ("max_tokens", c_int32), ("dtype", c_int32), ("slots_per_gen", c_int32),
                ("flags", c_uint32), ("cache_slots", c_int32), ("cache_policy", c_int32),
                ("pregate_distance", c_int32)]


class FetchStats(Structure):
    _fields_ = [("n_unique", c_int32), ("n_copied", c_int32), ("bytes_copied", c_int64),
                ("resident_slots", c_int32), ("cache_hits", c_int32), ("fetch_ms", c_float), ("wait_ms", c_float)]


class BlockTrace(Structure):
    _fields_ = [("fetch_ms", c_float), ("stall_ms", c_float), ("compute_ms", c_float), ("fetch_start_ms", c_float),
                ("fetch_end_ms", c_float), ("block_start_ms", c_float), ("block_end_ms", c_float), ("copy_ms", c_float)]


class StepBuffers(Structure):
    _fields_ = [("gate_w", POINTER(c_void_p)), ("gate_b", POINTER(c_void_p)), ("x_states", c_void_p),
                ("y_blocks", c_void_p), ("topk_idx", c_void_p), ("topk_prob", c_void_p), ("row_of", c_void_p),
                ("expert_offsets", c_void_p), ("x_perm", c_void_p), ("y_perm", c_void_p), ("workspace", c_void_p)]


class PgmoeError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"pgmoe error {code}: {text}")
        self.code = code


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2308_12066_amd.build`")
    # One HIP runtime per process: torch ships its own libamdhip64 and looks it up under a
    # different file name than the system one, so if this library came first the process would
    # hold two runtimes and the second to start would see no device.  Loading torch first makes
    # libpgmoe bind to the runtime torch already brought in (same soname).
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    L = ctypes.CDLL(LIB_PATH)
    vp, i = c_void_p, c_int
    L.pgmoe_create.argtypes = [POINTER(vp), POINTER(Config)]
    L.pgmoe_destroy.argtypes = [vp]
    L.pgmoe_last_error.argtypes = [vp]
    L.pgmoe_last_error.restype = c_char_p
    L.pgmoe_expert_bytes.argtypes = [POINTER(Config)]
    L.pgmoe_expert_bytes.restype = c_size_t
    L.pgmoe_workspace_bytes.argtypes = [vp]
    L.pgmoe_workspace_bytes.restype = c_size_t
    L.pgmoe_pack_expert.argtypes = [POINTER(Config), vp, vp, vp]
    L.pgmoe_unpack_expert.argtypes = [POINTER(Config), vp, vp, vp]
    L.pgmoe_pregate_topk.argtypes = [vp, vp, vp, vp, i, vp, vp, vp, vp]
    L.pgmoe_register_host_experts.argtypes = [vp, vp, c_size_t, c_size_t]
    L.pgmoe_register_resident_experts.argtypes = [vp, vp, c_size_t, c_size_t]
    L.pgmoe_fetch_experts.argtypes = [vp, i, vp, i, vp, vp, POINTER(c_int)]
    L.pgmoe_fetch_experts_as_turn.argtypes = [vp, i, vp, i, vp, i, c_float]
    L.pgmoe_get_fetch_stats.argtypes = [vp, i, POINTER(FetchStats)]
    L.pgmoe_migration_engine.argtypes = [vp]
    L.pgmoe_unique_experts.argtypes = [vp, i, i, vp]
    L.pgmoe_permute.argtypes = [vp, vp, vp, i, vp, vp, vp, vp]
    L.pgmoe_expert_ffn.argtypes = [vp, i, vp, vp, i, vp, vp, vp]
    L.pgmoe_expert_ffn_static.argtypes = [vp, i, vp, vp, i, vp, vp]
    L.pgmoe_combine.argtypes = [vp, vp, vp, vp, i, vp, vp, vp, vp]
    L.pgmoe_stack_step.argtypes = [vp, POINTER(StepBuffers), i, vp, vp]
    L.pgmoe_device_flags.argtypes = [vp, POINTER(c_uint32)]
    L.pgmoe_ffn_timing_begin.argtypes = [vp, i]
    L.pgmoe_ffn_kernel_name.argtypes = [vp, i]
    L.pgmoe_ffn_kernel_name.restype = c_char_p
    L.pgmoe_fetch_timing.argtypes = [vp, i]
    L.pgmoe_trace.argtypes = [vp, i]
    L.pgmoe_fetch_all_experts.argtypes = [vp, i, vp, vp]
    L.pgmoe_set_schedule.argtypes = [vp, i]
    L.pgmoe_set_nonmoe_standin.argtypes = [vp, c_float]
    L.pgmoe_check_streams.argtypes = [vp, vp, vp, POINTER(c_int)]
    L.pgmoe_get_block_trace.argtypes = [vp, i, POINTER(BlockTrace)]
    L.pgmoe_slot_address.argtypes = [vp, i, i, POINTER(vp)]
    L.pgmoe_ffn_timing_end.argtypes = [vp, POINTER(c_int), POINTER(c_float), POINTER(c_float)]
    for name in EXPORTS:
        if name not in ("pgmoe_last_error", "pgmoe_expert_bytes", "pgmoe_workspace_bytes", "pgmoe_ffn_kernel_name"):
            getattr(L, name).restype = c_int
    return L


lib = _load()


def _ptr(a):
    """Address of a torch tensor / numpy array / int / None as a void*."""
    if a is None:
        return None
    if isinstance(a, int):
        return c_void_p(a)
    if hasattr(a, "data_ptr"):
        return c_void_p(a.data_ptr())
    if hasattr(a, "ctypes"):
        return c_void_p(a.ctypes.data)
    raise TypeError(f"cannot take the address of {type(a)}")


def _stream(s):
    if s is None:
        return None
    if isinstance(s, int):
        return c_void_p(s)
    return c_void_p(s.cuda_stream)   # torch.cuda.Stream on ROCm carries the hipStream_t here


def last_error(ctx=None) -> str:
    return lib.pgmoe_last_error(ctx).decode()


def make_config(d_model, d_ff, n_experts, top_k, n_blocks, max_tokens, dtype, slots_per_gen=0, flags=0,
                cache_slots=0, cache_policy=0, pregate_distance=0) -> Config:
    return Config(d_model, d_ff, n_experts, top_k, n_blocks, max_tokens, dtype, slots_per_gen, flags, cache_slots,
                  cache_policy, pregate_distance)


def expert_bytes(cfg: Config) -> int:
    return int(lib.pgmoe_expert_bytes(byref(cfg)))


def pack_expert(cfg: Config, w1, w2, blob) -> None:
    rc = lib.pgmoe_pack_expert(byref(cfg), _ptr(w1), _ptr(w2), _ptr(blob))
    if rc:
        raise PgmoeError(rc, last_error())


def unpack_expert(cfg: Config, blob, w1, w2) -> None:
    rc = lib.pgmoe_unpack_expert(byref(cfg), _ptr(blob), _ptr(w1), _ptr(w2))
    if rc:
        raise PgmoeError(rc, last_error())


def unique_experts(idx, n_experts: int):
    import numpy as np
    idx = np.ascontiguousarray(idx, dtype=np.int32).ravel()
    out = np.zeros(max(1, min(n_experts, idx.size)), dtype=np.int32)
    rc = lib.pgmoe_unique_experts(_ptr(idx), idx.size, n_experts, _ptr(out))
    if rc < 0:
        raise PgmoeError(rc, last_error())
    return out[:rc].copy()


class Context:
    """Owns a pgmoe_ctx*.  Methods take tensors (anything with data_ptr()) or raw addresses."""

    def __init__(self, cfg: Config):
        self.cfg = cfg
        self._h = c_void_p()
        rc = lib.pgmoe_create(byref(self._h), byref(cfg))
        if rc:
            raise PgmoeError(rc, last_error())

    def close(self):
        if self._h:
            lib.pgmoe_destroy(self._h)
            self._h = c_void_p()

    def __del__(self):  # pragma: no cover
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc):
        if rc:
            raise PgmoeError(rc, last_error(self._h))

    @property
    def workspace_bytes(self) -> int:
        return int(lib.pgmoe_workspace_bytes(self._h))

    def pregate_topk(self, x, w_gate, bias, T, topk_idx, topk_prob, probs_out=None, stream=None):
        self._check(lib.pgmoe_pregate_topk(self._h, _ptr(x), _ptr(w_gate), _ptr(bias), T, _ptr(topk_idx),
                                           _ptr(topk_prob), _ptr(probs_out), _stream(stream)))

    def register_host_experts(self, host_base, expert_stride, block_stride):
        self._check(lib.pgmoe_register_host_experts(self._h, _ptr(host_base), expert_stride, block_stride))

    def register_resident_experts(self, dev_base, expert_stride, block_stride):
        self._check(lib.pgmoe_register_resident_experts(self._h, _ptr(dev_base), expert_stride, block_stride))

    def fetch_experts(self, block, topk_idx, T, compute_stream, copy_stream) -> int:
        n = c_int(0)
        self._check(lib.pgmoe_fetch_experts(self._h, block, _ptr(topk_idx), T, _stream(compute_stream),
                                            _stream(copy_stream), byref(n)))
        return n.value

    def fetch_experts_as_turn(self, block, topk_idx, T, stream, seq: int, wait_us: float):
        self._check(lib.pgmoe_fetch_experts_as_turn(self._h, block, _ptr(topk_idx), T, _stream(stream), seq, wait_us))

    @property
    def migration_engine(self) -> str:
        rc = lib.pgmoe_migration_engine(self._h)
        self._check(rc if rc < 0 else 0)
        return "copy_engine" if rc == 1 else "pull"

    def fetch_stats(self, block) -> FetchStats:
        st = FetchStats()
        self._check(lib.pgmoe_get_fetch_stats(self._h, block, byref(st)))
        return st

    def permute(self, x, topk_idx, T, x_perm, row_of, expert_offsets, stream=None):
        self._check(lib.pgmoe_permute(self._h, _ptr(x), _ptr(topk_idx), T, _ptr(x_perm), _ptr(row_of),
                                      _ptr(expert_offsets), _stream(stream)))

    def expert_ffn(self, block, x_perm, expert_offsets, n_rows, y_perm, workspace, stream=None):
        self._check(lib.pgmoe_expert_ffn(self._h, block, _ptr(x_perm), _ptr(expert_offsets), n_rows, _ptr(y_perm),
                                         _ptr(workspace), _stream(stream)))

    def expert_ffn_static(self, block, x_perm, expert_offsets, n_rows, y_perm, stream=None):
        self._check(lib.pgmoe_expert_ffn_static(self._h, block, _ptr(x_perm), _ptr(expert_offsets), n_rows, _ptr(y_perm),
                                                _stream(stream)))

    def combine(self, y_perm, row_of, topk_prob, T, y, x_res=None, x_next=None, stream=None):
        self._check(lib.pgmoe_combine(self._h, _ptr(y_perm), _ptr(row_of), _ptr(topk_prob), T, _ptr(y), _ptr(x_res),
                                      _ptr(x_next), _stream(stream)))

    def make_step_buffers(self, gate_w, gate_b, x_states, y_blocks, topk_idx, topk_prob, row_of, expert_offsets,
                          x_perm, y_perm, workspace) -> StepBuffers:
        L = self.cfg.n_blocks
        assert len(gate_w) == L
        gw = (c_void_p * L)(*[g.data_ptr() for g in gate_w])
        gb = None
        if gate_b is not None and any(b is not None for b in gate_b):
            gb = (c_void_p * L)(*[None if b is None else b.data_ptr() for b in gate_b])
        sb = StepBuffers(ctypes.cast(gw, POINTER(c_void_p)), ctypes.cast(gb, POINTER(c_void_p)) if gb else None,
                         _ptr(x_states), _ptr(y_blocks), _ptr(topk_idx), _ptr(topk_prob), _ptr(row_of),
                         _ptr(expert_offsets), _ptr(x_perm), _ptr(y_perm), _ptr(workspace))
        sb._keep = (gw, gb, gate_w, gate_b, x_states, y_blocks, topk_idx, topk_prob, row_of, expert_offsets, x_perm,
                    y_perm, workspace)
        return sb

    def stack_step(self, bufs: StepBuffers, T, compute_stream, copy_stream):
        self._check(lib.pgmoe_stack_step(self._h, byref(bufs), T, _stream(compute_stream), _stream(copy_stream)))

    def device_flags(self) -> int:
        f = c_uint32(0)
        self._check(lib.pgmoe_device_flags(self._h, byref(f)))
        return f.value

    def ffn_kernel_name(self, n_rows: int):
        name = lib.pgmoe_ffn_kernel_name(self._h, n_rows)
        return name.decode() if name is not None else None

    def ffn_timing_begin(self, max_launches: int):
        self._check(lib.pgmoe_ffn_timing_begin(self._h, max_launches))

    def ffn_timing_end(self):
        """-> (timed launches, sum of their event-to-event times in ms, per-pair event overhead in us)."""
        n, ms, oh = c_int(0), c_float(0.0), c_float(0.0)
        self._check(lib.pgmoe_ffn_timing_end(self._h, byref(n), byref(ms), byref(oh)))
        return n.value, ms.value, oh.value * 1e3

    def slot_address(self, block: int, slot: int) -> int:
        p = c_void_p()
        self._check(lib.pgmoe_slot_address(self._h, block, slot, byref(p)))
        return p.value

    def fetch_timing(self, enable: bool):
        self._check(lib.pgmoe_fetch_timing(self._h, 1 if enable else 0))

    def trace(self, enable: bool):
        self._check(lib.pgmoe_trace(self._h, 1 if enable else 0))

    def block_trace(self, block: int) -> BlockTrace:
        t = BlockTrace()
        self._check(lib.pgmoe_get_block_trace(self._h, block, byref(t)))
        return t

    def fetch_all_experts(self, block, compute_stream, copy_stream):
        self._check(lib.pgmoe_fetch_all_experts(self._h, block, _stream(compute_stream), _stream(copy_stream)))

    def set_schedule(self, schedule: int):
        self._check(lib.pgmoe_set_schedule(self._h, schedule))

    def check_streams(self, compute_stream, copy_stream) -> int:
        """Bit mask of the stream pairs that share a hardware queue (STREAMS_*); 0 = all side by side."""
        shared = c_int(0)
        self._check(lib.pgmoe_check_streams(self._h, _stream(compute_stream), _stream(copy_stream), byref(shared)))
        return shared.value

    def set_nonmoe_standin(self, microseconds: float):
        self._check(lib.pgmoe_set_nonmoe_standin(self._h, microseconds))
