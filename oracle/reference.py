"""ctypes front-end of the C oracle plus the stack driver (fp64).  TEST INFRASTRUCTURE ONLY.

The C file evaluates one gate / one routing / one block from the definition; this module
adds the wiring the paper gives for a stack of L pre-gated MoE blocks (Sec. IV-B):

  * block 0 is routed by its own conventional gate applied to the hidden state entering
    block 0, and also runs pre-gate 0 for block 1;
  * block i >= 1 is routed by pre-gate i-1, i.e. by the hidden state that entered block i-1;
  * the last block has no gate of its own and pre-gating never crosses a decoder iteration.

Between blocks the non-MoE layers are out of scope; the stand-in is the residual
x_{i+1} = x_i + y_i.

Nothing here imports or calls the HIP library.
"""
from __future__ import annotations

import ctypes
from typing import Callable, Sequence

import numpy as np

from . import build as _build

F32, BF16, F64 = 0, 1, 2

_lib = None


def bind(path: str):
    """Load an oracle library and declare its entry points (lib() does this for the built one;
    the mutation tests do it for deliberately broken copies)."""
    L = ctypes.CDLL(path)
    dp = ctypes.POINTER(ctypes.c_double)
    ip = ctypes.POINTER(ctypes.c_int32)
    vpp = ctypes.POINTER(ctypes.c_void_p)
    ci = ctypes.c_int
    L.pgo_max_threads.restype = ci
    L.pgo_gate_logits.argtypes = [dp, dp, dp, ci, ci, ci, dp]
    L.pgo_softmax.argtypes = [dp, ci, ci, dp]
    L.pgo_topk.argtypes = [dp, ci, ci, ci, ip, dp, ip]
    L.pgo_route.argtypes = [ip, ci, ci, ci, ip, ip, ip, ip, ip]
    L.pgo_ffn_rows.argtypes = [dp, ci, ci, ci, ctypes.c_void_p, ctypes.c_void_p, ci, dp, ci]
    L.pgo_block.argtypes = [dp, dp, ip, ci, ci, ci, ci, ci, vpp, vpp, ci, dp, ci]
    L.pgo_block.restype = ci
    for f in (L.pgo_gate_logits, L.pgo_softmax, L.pgo_topk, L.pgo_route, L.pgo_ffn_rows):
        f.restype = None
    return L


def lib():
    global _lib
    if _lib is None:
        _lib = bind(_build.build(force=False))
    return _lib


def max_threads() -> int:
    return int(lib().pgo_max_threads())


def _d(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def _dp(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _ip(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def _container(a: np.ndarray):
    """Pick the C container code for a weight array (values are read exactly)."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.float64:
        return a, F64
    if a.dtype == np.float32:
        return a, F32
    if a.dtype == np.uint16:
        return a, BF16
    return np.ascontiguousarray(a, dtype=np.float64), F64


# ------------------------------------------------------------------ single operations
def gate_logits(x, w, bias=None) -> np.ndarray:
    x, w = _d(x), _d(w)
    T, d = x.shape
    d2, E = w.shape
    assert d == d2
    b = None if bias is None else _d(bias)
    z = np.empty((T, E), dtype=np.float64)
    lib().pgo_gate_logits(_dp(x), _dp(w), None if b is None else _dp(b), T, d, E, _dp(z))
    return z


def softmax(z) -> np.ndarray:
    z = _d(z)
    T, E = z.shape
    p = np.empty_like(z)
    lib().pgo_softmax(_dp(z), T, E, _dp(p))
    return p


def topk(z, k: int):
    """-> (idx [T,k] int32, gaps [T,k] float64, nan_flag [T] int32); see pgo_topk."""
    z = _d(z)
    T, E = z.shape
    assert 1 <= k <= E
    idx = np.empty((T, k), dtype=np.int32)
    gaps = np.empty((T, k), dtype=np.float64)
    nan = np.zeros((T,), dtype=np.int32)
    lib().pgo_topk(_dp(z), T, E, k, _ip(idx), _dp(gaps), _ip(nan))
    return idx, gaps, nan


def gate(x, w, bias, k: int):
    """Full gate: -> dict(z, p, idx, prob [T,k] = p at the chosen experts, gaps, nan)."""
    z = gate_logits(x, w, bias)
    p = softmax(np.where(np.isnan(z), -np.inf, z))
    idx, gaps, nan = topk(z, k)
    prob = np.take_along_axis(p, idx.astype(np.int64), axis=1)
    return dict(z=z, p=p, idx=idx, prob=prob, gaps=gaps, nan=nan)


def route(idx, E: int):
    """-> dict(counts [E], offsets [E+1], row_of [T*k], unique (ascending expert ids))."""
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    T, k = idx.shape
    assert idx.size == 0 or (idx.min() >= 0 and idx.max() < E)
    counts = np.zeros((E,), dtype=np.int32)
    offsets = np.zeros((E + 1,), dtype=np.int32)
    row_of = np.zeros((T * k,), dtype=np.int32)
    unique = np.zeros((E,), dtype=np.int32)
    nu = np.zeros((1,), dtype=np.int32)
    lib().pgo_route(_ip(idx), T, k, E, _ip(counts), _ip(offsets), _ip(row_of), _ip(unique), _ip(nu))
    return dict(counts=counts, offsets=offsets, row_of=row_of, unique=unique[: int(nu[0])].copy())


def ffn_rows(x_rows, w1, w2, threads: int = 0) -> np.ndarray:
    """ReLU(x.W1).W2 for rows that all use one expert; W1 [d,f], W2 [f,d]."""
    x = _d(x_rows)
    n, d = x.shape
    w1, dt1 = _container(w1)
    w2, dt2 = _container(w2)
    assert dt1 == dt2 and w1.shape[0] == d and w2.shape == (w1.shape[1], d)
    y = np.empty((n, d), dtype=np.float64)
    lib().pgo_ffn_rows(_dp(x), n, d, w1.shape[1], w1.ctypes.data, w2.ctypes.data, dt1, _dp(y), threads)
    return y


def block(x, p, idx, experts: dict, d_ff: int, threads: int = 0) -> np.ndarray:
    """y[t] = sum_j p[t, idx[t,j]] * FFN_{idx[t,j]}(x[t]);  experts: {e: (W1, W2)}."""
    x, p = _d(x), _d(p)
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    T, d = x.shape
    E = p.shape[1]
    k = idx.shape[1]
    w1p = (ctypes.c_void_p * E)()
    w2p = (ctypes.c_void_p * E)()
    keep, dt = [], None
    for e, (w1, w2) in experts.items():
        w1, d1 = _container(w1)
        w2, d2 = _container(w2)
        assert d1 == d2 and (dt is None or dt == d1)
        assert w1.shape == (d, d_ff) and w2.shape == (d_ff, d)
        dt = d1
        keep.append((w1, w2))
        w1p[e], w2p[e] = w1.ctypes.data, w2.ctypes.data
    y = np.empty((T, d), dtype=np.float64)
    rc = lib().pgo_block(_dp(x), _dp(p), _ip(idx), T, d, d_ff, E, k, w1p, w2p, dt if dt is not None else F64,
                         _dp(y), threads)
    if rc != 0:
        raise ValueError("a selected expert has no weights")
    return y


# ------------------------------------------------------------------ stack of blocks
def routing_source(i: int, wiring: str = "pregated", distance: int = 1) -> int:
    """Index of the hidden state that routes block i.

    "pregated" (Sec. IV-B): x_0 for block 0 (its own conventional gate), x_{i-1} afterwards
    (the pre-gate of block i-1).  With a pre-gate that looks `distance` = N blocks ahead
    (Sec. VI-D, activation level N) block i is routed from x_{i-N}; the first N blocks have no
    block that far behind them and are routed from x_0, the earliest state there is (N = 1
    gives back the rule above, N = 0 the conventional wiring).
    "conventional" (Sec. II-B, the wiring of the paper's comparison systems): every block is
    routed by its own gate on its own input x_i."""
    if wiring == "conventional":
        return i
    if wiring != "pregated":
        raise ValueError(wiring)
    if distance < 0:
        raise ValueError(distance)
    return max(0, i - distance)


def block_from_states(x_route, x_cur, gate_w, gate_b, k: int, get_expert: Callable[[int], tuple],
                      d_ff: int, threads: int = 0):
    """One block given the two hidden states it depends on (used to check a chained GPU run
    block by block on the GPU's own inputs).  -> dict(gate=..., route=..., y=...)."""
    g = gate(x_route, gate_w, gate_b, k)
    r = route(g["idx"], np.asarray(gate_w).shape[1])
    experts = {int(e): get_expert(int(e)) for e in r["unique"]}
    y = block(x_cur, g["p"], g["idx"], experts, d_ff, threads)
    return dict(gate=g, route=r, y=y)


def stack_forward(x0, gates: Sequence[tuple], k: int, get_expert: Callable[[int, int], tuple],
                  d_ff: int, threads: int = 0, wiring: str = "pregated", distance: int = 1):
    """Free-running oracle chain over L = len(gates) blocks.

    gates[i] = (W, bias) of the gate that routes block i: block 0's conventional gate, then the
    pre-gates (gates[i] sits in block max(0, i - distance)); with wiring="conventional"
    gates[i] is block i's own gate.
    get_expert(block, e) -> (W1, W2).  Returns per-block dicts with x_in, gate, route, y,
    and the final hidden state."""
    xs = [_d(x0)]
    out = []
    for i, (gw, gb) in enumerate(gates):
        src = xs[routing_source(i, wiring, distance)]
        res = block_from_states(src, xs[i], gw, gb, k, lambda e, i=i: get_expert(i, e), d_ff, threads)
        res["x_in"] = xs[i]
        out.append(res)
        xs.append(xs[i] + res["y"])
    return out, xs[-1]
