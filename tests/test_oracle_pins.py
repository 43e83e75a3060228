"""Pins for the CPU oracle: every check compares it with something that is not the oracle
itself: a hand-computed case, closed forms, invariants, numpy/scipy library routines, and a
dense brute-force evaluation of every expert followed by masking (written here, in numpy).
"""
import os

import numpy as np
import pytest
import scipy.special

from oracle import reference as R

HERE = os.path.dirname(os.path.abspath(__file__))


def rng(seed):
    return np.random.default_rng(seed)


def make_block(seed, T=13, d=12, f=20, E=6, scale=0.5):
    g = rng(seed)
    x = g.standard_normal((T, d))
    wg = g.standard_normal((d, E)) * scale
    w1 = g.standard_normal((E, d, f)) * scale
    w2 = g.standard_normal((E, f, d)) * scale
    return x, wg, w1, w2


def dense_masked(x_route, x_cur, wg, bias, w1, w2, k):
    """Brute force: every expert on every token, then mask to the top-k (numpy/scipy only)."""
    z = x_route @ wg + (0 if bias is None else bias)
    p = scipy.special.softmax(z, axis=1)
    order = np.argsort(-z, axis=1, kind="stable")          # stable => ties to the lowest index
    mask = np.zeros_like(z)
    np.put_along_axis(mask, order[:, :k], 1.0, axis=1)
    h = np.maximum(np.einsum("td,edf->etf", x_cur, w1), 0.0)
    ye = np.einsum("etf,efd->etd", h, w2)
    y = np.einsum("te,etd->td", mask * p, ye)
    return y, z, p, order[:, :k]


# ----------------------------------------------------------------------- hand case
def test_hand_case_matches_golden_file():
    rows = [l.split() for l in open(os.path.join(HERE, "golden", "hand_case.txt"))
            if l.strip() and not l.startswith("#")]
    x = np.array([[1.0, 0.0], [0.0, 1.0], [1.0, 1.0]])
    wg = np.eye(2)
    experts = {0: (np.array([[1.0, -1.0], [0.0, 2.0]]), np.array([[1.0, 0.0], [3.0, 1.0]])),
               1: (np.array([[2.0, 0.0], [-1.0, 1.0]]), np.array([[0.0, 1.0], [1.0, 1.0]]))}
    g = R.gate(x, wg, None, 1)
    y = R.block(x, g["p"], g["idx"], experts, 2)
    for r in rows:
        t, e, prob, o0, o1 = int(r[0]), int(r[1]), float(r[2]), float(r[3]), float(r[4])
        assert g["idx"][t, 0] == e
        assert abs(g["prob"][t, 0] - prob) < 1e-15
        assert abs(y[t, 0] - o0) < 1e-14 and abs(y[t, 1] - o1) < 1e-14
    assert g["gaps"][2, 0] == 0.0 and abs(g["gaps"][0, 0] - 1.0) < 1e-15


# ----------------------------------------------------------------------- gate pieces
def test_gate_logits_match_numpy_matmul_and_are_not_transposed():
    g = rng(1)
    x, w, b = g.standard_normal((7, 5)), g.standard_normal((5, 3)), g.standard_normal(3)
    np.testing.assert_allclose(R.gate_logits(x, w, b), x @ w + b, rtol=0, atol=1e-13)
    np.testing.assert_allclose(R.gate_logits(x, w), x @ w, rtol=0, atol=1e-13)


def test_softmax_closed_forms():
    z = rng(2).standard_normal((9, 11)) * 3
    p = R.softmax(z)
    np.testing.assert_allclose(p.sum(1), 1.0, atol=1e-12)
    np.testing.assert_allclose(p, scipy.special.softmax(z, axis=1), atol=1e-14)
    np.testing.assert_allclose(R.softmax(z + 123.456), p, atol=1e-12)      # shift invariance
    np.testing.assert_allclose(R.softmax(z + 1e4), p, atol=1e-9)            # no overflow
    two = R.softmax(np.array([[0.3, -0.9]]))
    assert abs(two[0, 0] - 1.0 / (1.0 + np.exp(-1.2))) < 1e-15               # logistic form
    assert np.all(R.softmax(np.zeros((4, 8))) == 1.0 / 8)                    # exact uniform


def test_zero_gate_gives_uniform_probs_and_lowest_indices():
    x = rng(3).standard_normal((5, 4))
    g = R.gate(x, np.zeros((4, 7)), None, 3)
    assert np.all(g["p"] == 1.0 / 7)
    assert np.array_equal(g["idx"], np.tile(np.arange(3, dtype=np.int32), (5, 1)))
    assert np.all(g["gaps"] == 0.0)


def test_topk_order_ties_margin_and_nan():
    z = np.array([[0.1, 0.7, 0.7, -1.0, 0.5],
                  [2.0, np.nan, 3.0, 3.0, -5.0]])
    idx, gaps, nan = R.topk(z, 3)
    assert idx.tolist() == [[1, 2, 4], [2, 3, 0]]
    np.testing.assert_allclose(gaps[0], [0.0, 0.2, 0.4], atol=1e-15)
    np.testing.assert_allclose(gaps[1], [0.0, 1.0, 7.0], atol=1e-15)
    assert nan.tolist() == [0, 1]
    idx_all, gaps_all, _ = R.topk(z[:1], 5)
    assert idx_all.tolist() == [[1, 2, 4, 0, 3]] and np.isinf(gaps_all[0, 4])
    # against numpy's stable sort on random data with many ties
    zz = np.round(rng(4).standard_normal((50, 16)) * 2) / 2
    for k in (1, 2, 5, 16):
        idx, _, _ = R.topk(zz, k)
        assert np.array_equal(idx, np.argsort(-zz, axis=1, kind="stable")[:, :k])


# ----------------------------------------------------------------------- routing
@pytest.mark.parametrize("T,k,E", [(1, 1, 8), (37, 2, 5), (64, 3, 16), (0, 1, 4)])
def test_route_invariants(T, k, E):
    g = rng(5)
    idx = np.stack([g.permutation(E)[:k] for _ in range(T)]).astype(np.int32) if T else np.zeros((0, k), np.int32)
    r = R.route(idx, E)
    n = T * k
    assert r["counts"].sum() == n and r["offsets"][0] == 0 and r["offsets"][E] == n
    assert np.all(np.diff(r["offsets"]) == r["counts"])
    assert np.array_equal(np.sort(r["row_of"]), np.arange(n))                 # a permutation
    assert np.array_equal(r["counts"], np.bincount(idx.ravel(), minlength=E))
    assert np.array_equal(r["unique"], np.unique(idx))
    # numpy's stable sort by expert gives the same grouping
    order = np.argsort(idx.ravel(), kind="stable")
    expect = np.empty(n, dtype=np.int64)
    expect[order] = np.arange(n)
    assert np.array_equal(r["row_of"], expect)
    # rows of one expert hold ascending entry numbers; unpermute(permute(x)) == x
    x = g.standard_normal((T, 3))
    xp = np.empty((n, 3))
    xp[r["row_of"]] = np.repeat(x, k, axis=0)
    assert np.array_equal(xp[r["row_of"]].reshape(T, k, 3)[:, 0], x) if T else True
    for e in range(E):
        ent = order[r["offsets"][e]: r["offsets"][e + 1]]
        assert np.all(np.diff(ent) > 0)
        assert np.all(idx.ravel()[ent] == e)


# ----------------------------------------------------------------------- expert FFN
def test_single_expert_is_a_two_layer_mlp():
    x, _, w1, w2 = make_block(6, E=1)
    wg = rng(6).standard_normal((x.shape[1], 1))
    g = R.gate(x, wg, None, 1)
    assert np.all(g["p"] == 1.0) and np.all(g["idx"] == 0)
    y = R.block(x, g["p"], g["idx"], {0: (w1[0], w2[0])}, w1.shape[2])
    np.testing.assert_allclose(y, np.maximum(x @ w1[0], 0) @ w2[0], atol=1e-12)
    np.testing.assert_allclose(R.ffn_rows(x, w1[0], w2[0]), np.maximum(x @ w1[0], 0) @ w2[0], atol=1e-12)


def test_ffn_relu_really_clips_and_weights_are_not_transposed():
    # a square case (d == f) where using W^T instead of W, or dropping ReLU, changes the answer
    g = rng(7)
    x = g.standard_normal((4, 6))
    w1, w2 = g.standard_normal((6, 6)), g.standard_normal((6, 6))
    y = R.ffn_rows(x, w1, w2)
    np.testing.assert_allclose(y, np.maximum(x @ w1, 0) @ w2, atol=1e-12)
    assert np.abs(y - (x @ w1) @ w2).max() > 1e-3
    assert np.abs(y - np.maximum(x @ w1.T, 0) @ w2).max() > 1e-3
    assert np.abs(y - np.maximum(x @ w1, 0) @ w2.T).max() > 1e-3


def test_ffn_positive_homogeneity_and_zero_w2():
    x, _, w1, w2 = make_block(8, E=1)
    y = R.ffn_rows(x, w1[0], w2[0])
    np.testing.assert_allclose(R.ffn_rows(2.5 * x, w1[0], w2[0]), 2.5 * y, atol=1e-12)
    assert np.abs(R.ffn_rows(-x, w1[0], w2[0]) + y).max() > 1e-3          # not linear
    assert np.all(R.ffn_rows(x, w1[0], np.zeros_like(w2[0])) == 0.0)


def test_weight_containers_read_the_same_values():
    from workloads import round_to_bf16, to_bf16_bits
    g = rng(9)
    x = g.standard_normal((3, 8))
    w1 = round_to_bf16(g.standard_normal((8, 16)).astype(np.float32))
    w2 = round_to_bf16(g.standard_normal((16, 8)).astype(np.float32))
    a = R.ffn_rows(x, w1.astype(np.float64), w2.astype(np.float64))
    b = R.ffn_rows(x, w1, w2)
    c = R.ffn_rows(x, to_bf16_bits(w1), to_bf16_bits(w2))
    assert np.array_equal(a, b) and np.array_equal(a, c)


# ----------------------------------------------------------------------- whole block
@pytest.mark.parametrize("k", [1, 2, 3, 6])
def test_block_equals_dense_brute_force(k):
    x, wg, w1, w2 = make_block(10 + k)
    bias = rng(99).standard_normal(wg.shape[1])
    x_route = rng(98).standard_normal(x.shape)                 # routing source != block input
    g = R.gate(x_route, wg, bias, k)
    experts = {e: (w1[e], w2[e]) for e in range(w1.shape[0])}
    y = R.block(x, g["p"], g["idx"], experts, w1.shape[2])
    y_ref, z_ref, p_ref, idx_ref = dense_masked(x_route, x, wg, bias, w1, w2, k)
    np.testing.assert_allclose(g["z"], z_ref, atol=1e-13)
    np.testing.assert_allclose(g["p"], p_ref, atol=1e-14)
    assert np.array_equal(g["idx"], idx_ref)
    np.testing.assert_allclose(y, y_ref, atol=1e-12)
    # combine weights are the raw softmax values: their sum is the selected softmax mass
    np.testing.assert_allclose(g["prob"].sum(1), np.take_along_axis(p_ref, idx_ref, 1).sum(1), atol=1e-14)
    if k < wg.shape[1]:
        assert np.all(g["prob"].sum(1) < 1.0 - 1e-6)           # i.e. NOT renormalised


def test_all_experts_selected_is_the_soft_mixture():
    x, wg, w1, w2 = make_block(20, E=4)
    g = R.gate(x, wg, None, 4)
    y = R.block(x, g["p"], g["idx"], {e: (w1[e], w2[e]) for e in range(4)}, w1.shape[2])
    p = scipy.special.softmax(x @ wg, axis=1)
    mix = sum(p[:, [e]] * (np.maximum(x @ w1[e], 0) @ w2[e]) for e in range(4))
    np.testing.assert_allclose(y, mix, atol=1e-12)
    same = {e: (w1[0], w2[0]) for e in range(4)}               # identical experts: sum p = 1
    y1 = R.block(x, g["p"], g["idx"], same, w1.shape[2])
    np.testing.assert_allclose(y1, np.maximum(x @ w1[0], 0) @ w2[0], atol=1e-12)


def test_token_permutation_equivariance():
    x, wg, w1, w2 = make_block(21)
    experts = {e: (w1[e], w2[e]) for e in range(w1.shape[0])}
    perm = rng(22).permutation(x.shape[0])
    g = R.gate(x, wg, None, 2)
    y = R.block(x, g["p"], g["idx"], experts, w1.shape[2])
    gp = R.gate(x[perm], wg, None, 2)
    yp = R.block(x[perm], gp["p"], gp["idx"], experts, w1.shape[2])
    np.testing.assert_allclose(yp, y[perm], atol=1e-13)


def test_missing_expert_is_an_error():
    x, wg, w1, w2 = make_block(23)
    g = R.gate(x, wg, None, 1)
    with pytest.raises(ValueError):
        R.block(x, g["p"], g["idx"], {}, w1.shape[2])


# ----------------------------------------------------------------------- stack wiring
def _numpy_stack(x0, gates, w1, w2, k, conventional=False, table=None):
    """The pre-gated (or conventional) wiring written out by hand with explicit indices (numpy only).
    table: for every block, the index of the hidden state that routes it, spelled out."""
    L = len(gates)
    xs = [x0]
    ys, idxs = [], []
    for i in range(L):
        src = xs[i] if conventional else (xs[0] if i == 0 else xs[i - 1])
        if table is not None:
            src = xs[table[i]]
        y, _, _, idx = dense_masked(src, xs[i], gates[i][0], gates[i][1], w1[i], w2[i], k)
        ys.append(y)
        idxs.append(idx)
        xs.append(xs[i] + y)
    return ys, idxs, xs


@pytest.mark.parametrize("k", [1, 2])
def test_stack_wiring_matches_explicit_numpy_chain(k):
    g = rng(30)
    L, T, d, f, E = 4, 9, 10, 14, 5
    x0 = g.standard_normal((T, d))
    gates = [(g.standard_normal((d, E)), g.standard_normal(E) * 0.3) for _ in range(L)]
    w1 = g.standard_normal((L, E, d, f)) * 0.4
    w2 = g.standard_normal((L, E, f, d)) * 0.4
    out, x_last = R.stack_forward(x0, gates, k, lambda b, e: (w1[b, e], w2[b, e]), f)
    ys, idxs, xs = _numpy_stack(x0, gates, w1, w2, k)
    for i in range(L):
        assert np.array_equal(out[i]["gate"]["idx"], idxs[i]), f"routing of block {i}"
        np.testing.assert_allclose(out[i]["y"], ys[i], atol=1e-11)
        np.testing.assert_allclose(out[i]["x_in"], xs[i], atol=1e-11)
    np.testing.assert_allclose(x_last, xs[-1], atol=1e-11)
    # the wiring matters on this data: routing block i>=1 from its own input would differ
    alt = [np.argsort(-(xs[i] @ gates[i][0] + gates[i][1]), axis=1, kind="stable")[:, :k] for i in range(1, L)]
    assert any(not np.array_equal(a, idxs[i + 1]) for i, a in enumerate(alt))


def test_conventional_wiring_matches_explicit_numpy_chain():
    g = rng(33)
    L, T, d, f, E, k = 3, 7, 8, 12, 4, 2
    x0 = g.standard_normal((T, d))
    gates = [(g.standard_normal((d, E)), None) for _ in range(L)]
    w1 = g.standard_normal((L, E, d, f)) * 0.4
    w2 = g.standard_normal((L, E, f, d)) * 0.4
    out, x_last = R.stack_forward(x0, gates, k, lambda b, e: (w1[b, e], w2[b, e]), f, wiring="conventional")
    ys, idxs, xs = _numpy_stack(x0, gates, w1, w2, k, conventional=True)
    for i in range(L):
        assert np.array_equal(out[i]["gate"]["idx"], idxs[i])
        np.testing.assert_allclose(out[i]["y"], ys[i], atol=1e-11)
    np.testing.assert_allclose(x_last, xs[-1], atol=1e-11)
    pre, _ = R.stack_forward(x0, gates, k, lambda b, e: (w1[b, e], w2[b, e]), f)
    assert any(not np.array_equal(pre[i]["gate"]["idx"], idxs[i]) for i in range(1, L))   # the wirings differ


@pytest.mark.parametrize("distance,table", [(2, [0, 0, 0, 1, 2, 3]), (3, [0, 0, 0, 0, 1, 2]), (1, [0, 0, 1, 2, 3, 4]),
                                            (0, [0, 1, 2, 3, 4, 5])])
def test_pregate_distance_wiring_matches_a_spelled_out_table(distance, table):
    # Sec. VI-D, activation level N: the gate evaluated N blocks earlier routes the block; the
    # expected source of every block is written out by hand above, not computed.
    g = rng(37 + distance)
    L, T, d, f, E, k = 6, 7, 8, 10, 5, 2
    x0 = g.standard_normal((T, d))
    gates = [(g.standard_normal((d, E)), g.standard_normal(E) * 0.2) for _ in range(L)]
    w1 = g.standard_normal((L, E, d, f)) * 0.4
    w2 = g.standard_normal((L, E, f, d)) * 0.4
    assert [R.routing_source(i, "pregated", distance) for i in range(L)] == table
    out, x_last = R.stack_forward(x0, gates, k, lambda b, e: (w1[b, e], w2[b, e]), f, distance=distance)
    ys, idxs, xs = _numpy_stack(x0, gates, w1, w2, k, table=table)
    for i in range(L):
        assert np.array_equal(out[i]["gate"]["idx"], idxs[i]), f"routing of block {i}"
        np.testing.assert_allclose(out[i]["y"], ys[i], atol=1e-10)
    np.testing.assert_allclose(x_last, xs[-1], atol=1e-10)
    if distance != 1:   # and it is a different computation from the default wiring on this data
        base, _ = R.stack_forward(x0, gates, k, lambda b, e: (w1[b, e], w2[b, e]), f)
        assert any(not np.array_equal(base[i]["gate"]["idx"], idxs[i]) for i in range(L))


def test_pregate_reduces_to_conventional_gate_when_block_is_identity():
    # W2 = 0 in block 0 => x_1 = x_0, so block 1 routed by pre-gate 0 (on x_0) must equal a
    # conventional gate with the same weights applied to block 1's own input.
    g = rng(31)
    T, d, f, E = 8, 6, 10, 4
    x0 = g.standard_normal((T, d))
    gates = [(g.standard_normal((d, E)), None), (g.standard_normal((d, E)), None)]
    w1 = g.standard_normal((2, E, d, f))
    w2 = g.standard_normal((2, E, f, d))
    w2[0] = 0.0
    out, _ = R.stack_forward(x0, gates, 1, lambda b, e: (w1[b, e], w2[b, e]), f)
    assert np.all(out[0]["y"] == 0.0) and np.array_equal(out[1]["x_in"], x0)
    conv = R.gate(out[1]["x_in"], gates[1][0], None, 1)
    assert np.array_equal(conv["idx"], out[1]["gate"]["idx"])
    y_conv = R.block(out[1]["x_in"], conv["p"], conv["idx"], {e: (w1[1, e], w2[1, e]) for e in range(E)}, f)
    np.testing.assert_allclose(out[1]["y"], y_conv, atol=1e-13)


def test_fetch_set_is_the_unique_selected_experts():
    g = rng(32)
    idx = g.integers(0, 64, size=(16, 1)).astype(np.int32)
    r = R.route(idx, 64)
    assert np.array_equal(r["unique"], np.unique(idx))
    assert len(r["unique"]) <= 16


# ----------------------------------------------------------------------- cache policy model
def test_cache_policy_model_on_hand_traced_sequences():
    """The reference model of the expert cache against sequences traced by hand."""
    from oracle.cache_policy import ExpertCache, LRU, LFU, LIFO
    # LRU, 2 slots: 1,2 fill; 1 hits; 3 evicts 2 (1 was used later); 2 evicts 1? no: 3 then 2 -> victim is 1
    c = ExpertCache(2, LRU)
    assert c.fetch([1])["copies"] == [(1, "cache", 0)]
    assert c.fetch([2])["copies"] == [(2, "cache", 1)]
    r = c.fetch([1]); assert r["hits"] == 1 and r["copies"] == []
    assert c.fetch([3])["copies"] == [(3, "cache", 1)]          # 2 is least recently used
    assert c.fetch([2])["copies"] == [(2, "cache", 0)]          # now 1 is
    # LFU, 2 slots: 1 used three times, 2 once -> 3 evicts 2; then 4 evicts 3 (count 1, older than nothing else)
    c = ExpertCache(2, LFU)
    c.fetch([1]); c.fetch([1]); c.fetch([1]); c.fetch([2])
    assert c.fetch([3])["copies"] == [(3, "cache", 1)]
    assert c.fetch([4])["copies"] == [(4, "cache", 1)]
    assert c.fetch([1])["hits"] == 1
    # LIFO, 3 slots: 5,6,7 fill in order; 8 evicts 7 (last in); 9 evicts 8
    c = ExpertCache(3, LIFO)
    assert [x[2] for x in c.fetch([5, 6, 7])["copies"]] == [0, 1, 2]
    assert c.fetch([8])["copies"] == [(8, "cache", 2)]
    assert c.fetch([9])["copies"] == [(9, "cache", 2)]
    assert c.fetch([5, 6])["hits"] == 2
    # a fetch never evicts what it uses itself; what does not fit goes to the ordinary slots
    c = ExpertCache(2, LRU)
    r = c.fetch([4, 1, 3])
    assert r["copies"] == [(1, "cache", 0), (3, "cache", 1), (4, "gen", 0)] and r["unique"] == 3
    r = c.fetch([1, 2, 3])
    assert r["hits"] == 2 and r["copies"] == [(2, "gen", 0)]
