"""Do the pins really pin the oracle?  Each case plants ONE plausible mistake in a copy of the
oracle's C source (a dropped term, a wrong index, a transposed operand, a wrong tie rule ...),
builds it, puts it in the oracle's place and runs the pin tests of test_oracle_pins.py: at
least one of them has to fail.  Everything here runs on the CPU; nothing touches the HIP path."""
import os
import subprocess

import pytest

from oracle import reference as R

import test_oracle_pins as P

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(os.path.dirname(HERE), "oracle", "pgmoe_oracle.c")

# (name, text in the source, what a careless author might have written instead)
MUTANTS = [
    ("relu_dropped", "if (!(h[j] > 0.0)) h[j] = 0.0;", ";"),
    ("relu_sign", "if (!(h[j] > 0.0)) h[j] = 0.0;", "if (h[j] > 0.0) h[j] = 0.0;"),
    ("w1_transposed", "load_elem(w1, (size_t)i * f + j, dt)", "load_elem(w1, (size_t)j * d + i, dt)"),
    ("w2_transposed", "load_elem(w2, (size_t)j * d + c, dt)", "load_elem(w2, (size_t)c * f + j, dt)"),
    ("combine_prob_by_rank", "const double pe = p[(size_t)t * E + e];", "const double pe = p[(size_t)t * E + j];"),
    ("combine_keeps_last_expert", "yt[c] += pe * ye[c];", "yt[c] = pe * ye[c];"),
    ("combine_unweighted", "yt[c] += pe * ye[c];", "yt[c] += ye[c];"),
    ("gate_w_transposed", "w[(size_t)i * E + e]", "w[(size_t)e * d + i]"),
    ("gate_bias_dropped", "z[(size_t)t * E + e] = s + (bias ? bias[e] : 0.0);", "z[(size_t)t * E + e] = s;"),
    ("gate_bias_sign", "z[(size_t)t * E + e] = s + (bias ? bias[e] : 0.0);", "z[(size_t)t * E + e] = s - (bias ? bias[e] : 0.0);"),
    ("softmax_not_normalised", "for (int e = 0; e < E; ++e) pt[e] /= s;", ";"),
    ("softmax_exp_sign", "pt[e] = exp(zt[e] - m);", "pt[e] = exp(m - zt[e]);"),
    ("topk_ties_to_highest", "(best < 0 || v[e] > v[best])", "(best < 0 || v[e] >= v[best])"),
    ("topk_smallest", "(best < 0 || v[e] > v[best])", "(best < 0 || v[e] < v[best])"),
    ("topk_nan_not_lowest", "if (isnan(a)) { a = -INFINITY; saw_nan = 1; }", "if (isnan(a)) { a = INFINITY; saw_nan = 1; }"),
    ("topk_gap_off_by_one", "gaps[(size_t)t * k + (j - 1)] = (best >= 0) ? prev - v[best] : INFINITY;",
     "gaps[(size_t)t * k + (j - 1)] = (best >= 0) ? v[best] - prev : INFINITY;"),
    ("route_offsets_inclusive", "offsets[e + 1] = offsets[e] + counts[e];", "offsets[e + 1] = offsets[e] + counts[e] + (e == 0);"),
    ("route_not_stable", "row_of[n] = offsets[e] + seen[e];", "row_of[n] = offsets[e] + counts[e] - 1 - seen[e];"),
    ("route_unique_keeps_idle", "if (counts[e] > 0) unique[u++] = e;", "unique[u++] = e;"),
    ("bf16_low_half", "(uint32_t)((const uint16_t *)base)[i] << 16", "(uint32_t)((const uint16_t *)base)[i]"),
]


def detectors():
    """The pin tests, as argument-free callables."""
    calls = [
        P.test_hand_case_matches_golden_file,
        P.test_gate_logits_match_numpy_matmul_and_are_not_transposed,
        P.test_softmax_closed_forms,
        P.test_zero_gate_gives_uniform_probs_and_lowest_indices,
        P.test_topk_order_ties_margin_and_nan,
        lambda: P.test_route_invariants(37, 2, 5),
        P.test_single_expert_is_a_two_layer_mlp,
        P.test_ffn_relu_really_clips_and_weights_are_not_transposed,
        P.test_ffn_positive_homogeneity_and_zero_w2,
        P.test_weight_containers_read_the_same_values,
        lambda: P.test_block_equals_dense_brute_force(1),
        lambda: P.test_block_equals_dense_brute_force(2),
        P.test_all_experts_selected_is_the_soft_mixture,
        P.test_token_permutation_equivariance,
        lambda: P.test_stack_wiring_matches_explicit_numpy_chain(2),
        P.test_fetch_set_is_the_unique_selected_experts,
    ]
    return calls


def failing_detectors():
    out = []
    for call in detectors():
        try:
            call()
        except AssertionError:
            out.append(getattr(call, "__name__", "lambda"))
        except Exception as exc:   # a crash inside a pin (e.g. an index out of range) also exposes the mistake
            out.append(f"{getattr(call, '__name__', 'lambda')}:{type(exc).__name__}")
    return out


def test_the_unmodified_oracle_passes_every_detector(monkeypatch):
    monkeypatch.setattr(R, "_lib", None)
    assert failing_detectors() == []


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_a_planted_mistake_is_caught(tmp_path, monkeypatch, name, old, new):
    text = open(SRC).read()
    assert text.count(old) >= 1, f"{name}: the source no longer has the line this mutant edits"
    src = tmp_path / f"oracle_{name}.c"
    src.write_text(text.replace(old, new))
    so = tmp_path / f"liboracle_{name}.so"
    subprocess.run(["gcc", "-O1", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-w", "-o", str(so), str(src), "-lm"], check=True)
    monkeypatch.setattr(R, "_lib", R.bind(str(so)))
    caught = failing_detectors()
    assert caught, f"mutant {name} passes every pin: the pins do not cover this mistake"
