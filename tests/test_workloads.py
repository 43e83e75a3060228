"""The seeded input generators: determinism, storage rounding, and the Zipf recipe."""
import numpy as np
import pytest
import torch

import workloads as W


def test_streams_are_deterministic_and_distinct():
    w = W.CONFIGS["cfg1"]
    a1, a2 = W.expert_weights(w, 0, 3)
    b1, b2 = W.expert_weights(w, 0, 3)
    assert np.array_equal(a1, b1) and np.array_equal(a2, b2)
    c1, _ = W.expert_weights(w, 1, 3)
    assert not np.array_equal(a1, c1)
    assert a1.shape == (64, 256) and a2.shape == (256, 64) and a1.dtype == np.float32
    assert not np.array_equal(W.step_input(w, 0), W.step_input(w, 1))
    assert abs(float(a1.std()) - 0.02) < 0.002 and abs(float(W.step_input(w, 0).std()) - 1.0) < 0.05


def test_bf16_rounding_matches_torch_and_round_trips():
    g = np.random.default_rng(0)
    a = (g.standard_normal(100000) * np.exp(g.uniform(-20, 20, 100000))).astype(np.float32)
    a[:4] = [0.0, -0.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8]     # exact ties: to even
    r = W.round_to_bf16(a)
    t = torch.from_numpy(a).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(r.view(np.uint32), t.view(np.uint32))
    assert np.array_equal(W.from_bf16_bits(W.to_bf16_bits(r)), r)
    assert np.array_equal(W.round_to_bf16(r), r)


def test_bf16_workloads_hold_bf16_values():
    w = W.CONFIGS["cfg2"]
    for a in (W.gate0_weight(w), W.pregate_weight(w, 0), W.step_input(w, 5)):
        assert np.array_equal(W.round_to_bf16(a), a)
    assert w.expert_bytes == 9437184 and W.CONFIGS["cfg5"].expert_bytes == 16777216
    assert W.CONFIGS["cfg1"].expert_bytes == 131072


def test_zipf_bias_makes_the_hottest_expert_about_q1():
    # the recipe promises argmax frequencies roughly Zipf(1.1): the hottest expert's share is
    # within 25 % (relative) of q_1, checked on Gaussian logits of the stated spread.
    for name, q1 in (("cfg3", 0.250), ("cfg5", 0.226)):
        w = W.CONFIGS[name]
        b = W.gate_bias(w, 1)
        q = W.zipf_probabilities(w.n_experts, w.zipf_s)
        assert abs(q[0] - q1) < 2e-3
        g = np.random.default_rng(1)
        z = g.standard_normal((20000, w.n_experts)) * (0.02 * np.sqrt(w.d_model)) + b
        share = np.bincount(z.argmax(1), minlength=w.n_experts) / 20000.0
        assert int(share.argmax()) == int(b.argmax())
        assert abs(share.max() - q[0]) / q[0] < 0.25
    assert W.gate_bias(W.CONFIGS["cfg4"], 0) is None


@pytest.mark.parametrize("name,L,d,f,E,k,T,steps,dtype,offloaded,expert_bytes,store_gb", [
    ("cfg1", 2, 64, 256, 8, 1, 32, 1, "f32", False, 131072, None),
    ("cfg2", 6, 768, 3072, 8, 1, 1, 128, "bf16", True, 9437184, 0.45),
    ("cfg3", 6, 768, 3072, 64, 1, 16, 128, "bf16", True, 9437184, 3.62),
    ("cfg4", 6, 768, 3072, 128, 1, 4096, 1, "bf16", False, 9437184, 7.25),
    ("cfg4_offloaded", 6, 768, 3072, 128, 1, 4096, 1, "bf16", True, 9437184, 7.25),
    ("cfg5", 12, 1024, 4096, 128, 1, 64, 64, "bf16", True, 16777216, 25.77),
    ("cfg5_top2", 12, 1024, 4096, 128, 2, 64, 64, "bf16", True, 16777216, 25.77),
])
def test_configurations_have_the_shapes_and_sizes_of_the_switch_models(name, L, d, f, E, k, T, steps, dtype, offloaded,
                                                                     expert_bytes, store_gb):
    """The five benchmark configurations: shapes as listed for the Switch-Base / Switch-Large
    variants (Sec. V, model table), expert bytes 2*d*f*sizeof(weight), expert store L*E*bytes."""
    w = W.CONFIGS[name]
    assert (w.n_blocks, w.d_model, w.d_ff, w.n_experts, w.top_k, w.tokens, w.steps, w.dtype, w.offloaded) == \
           (L, d, f, E, k, T, steps, dtype, offloaded)
    assert w.expert_bytes == expert_bytes
    if store_gb is not None:
        assert abs(w.n_blocks * w.n_experts * w.expert_bytes / 1e9 - store_gb) < 0.006
    assert 4 * w.d_model * w.d_ff == {64: 65536, 768: 9437184, 1024: 16777216}[d]      # FFN flops per token and expert


def test_gate_list_has_one_conventional_gate_and_L_minus_1_pregates():
    w = W.CONFIGS["cfg2"]
    gates = W.gate_tensors(w)
    assert len(gates) == w.n_blocks
    assert np.array_equal(gates[0][0], W.gate0_weight(w))
    assert np.array_equal(gates[3][0], W.pregate_weight(w, 2))


def test_activated_expert_sweep_points_share_weights_and_differ_only_in_top_k():
    pts = [W.CONFIGS[f"sweep64_k{k}"] for k in W.SWEEP_K]
    assert [p.top_k for p in pts] == [1, 2, 4, 8, 16, 32, 64]
    a, b = pts[0], pts[-1]
    assert (a.d_model, a.d_ff, a.n_experts, a.tokens, a.index) == (768, 3072, 64, 1, b.index) and b.top_k == b.n_experts
    assert np.array_equal(W.pregate_weight(a, 0), W.pregate_weight(b, 0))
    assert np.array_equal(W.step_input(a, 3), W.step_input(b, 3))


def test_bench_refuses_more_than_one_gpu():
    """This build is one GPU's share of the path: bench.py says so instead of launching ranks."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "ONE GPU" in r.stderr and r.stdout.strip() == ""
