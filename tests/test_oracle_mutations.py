"""The pins must be able to fail: each plausible mistake below is planted in a copy of the oracle's C
source (on the CPU, in a temporary directory), the copy is loaded in place of the real one, and at
least one of the pin tests has to reject it."""
import ctypes
import os
import subprocess

import pytest

import oracle
import test_oracle_alias as t_alias
import test_oracle_philox as t_philox
import test_oracle_score as t_score
import test_oracle_sequential as t_seq
import test_oracle_sgns as t_sgns
import test_oracle_shared as t_shared
import test_oracle_walks as t_walks

SRC = os.path.join(os.path.dirname(oracle.__file__), "ne_oracle.c")

# (name, text to find, replacement, pins that must catch it)
MUTATIONS = [
    ("negative label sign", "const double g = (j == 0) ? 1.0 - sigmoid(s) : -sigmoid(s);",
     "const double g = (j == 0) ? 1.0 - sigmoid(s) : sigmoid(s);",
     [t_sgns.test_update_equals_torch_autograd, t_sgns.test_update_equals_finite_difference_gradient]),
    ("context update without the learning rate", "dc[i] += lr * g * (double)x[i];", "dc[i] += g * (double)x[i];",
     [t_sgns.test_update_equals_torch_autograd, t_sgns.test_first_batch_from_zero_context_closed_form]),
    ("source gradient built from the source row", "dx[i] += lr * g * (double)c[i];", "dx[i] += lr * g * (double)x[i];",
     [t_sgns.test_update_equals_torch_autograd]),
    ("duplicates overwrite instead of adding", "dc[i] += lr * g * (double)x[i];", "dc[i] = lr * g * (double)x[i];",
     [t_sgns.test_update_equals_finite_difference_gradient, t_sgns.test_update_equals_torch_autograd]),
    ("loss term of a negative with the wrong sign", "total += (j == 0) ? softplus(-s) : softplus(s);",
     "total += softplus(-s);", [t_sgns.test_loss_closed_forms]),
    ("Vose residual", "p[l] = (p[l] + p[s]) - 1.0;", "p[l] = p[l] - p[s];", [lambda: t_alias.test_alias_identity(1000, 5)]),
    ("weight exponent", "p[i] = sqrt(deg) * sqrt(sqrt(deg));", "p[i] = sqrt(deg);", [lambda: t_alias.test_alias_identity(1000, 5)]),
    ("threshold word", "return (r[2] < thr_q[slot]) ? slot : (int64_t)alias[slot];",
     "return (r[3] < thr_q[slot]) ? slot : (int64_t)alias[slot];", [t_alias.test_alias_draw_mapping_matches_big_integers]),
    ("slot word order", "((unsigned __int128)r[0] << 32) | (unsigned __int128)r[1]",
     "((unsigned __int128)r[1] << 32) | (unsigned __int128)r[0]", [t_alias.test_alias_draw_mapping_matches_big_integers]),
    ("k not in the counter", "(uint32_t)k, STREAM_NEGATIVE };", "0u, STREAM_NEGATIVE };",
     [t_alias.test_alias_draw_mapping_matches_big_integers, t_alias.test_alias_frequencies_1e7_draws]),
    ("Philox multipliers swapped", "const uint64_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;",
     "const uint64_t M0 = 0xCD9E8D57u, M1 = 0xD2511F53u;", [t_philox.test_philox_matches_bigint]),
    ("Philox round wiring", "uint32_t n0 = hi1 ^ c1 ^ k0;", "uint32_t n0 = hi0 ^ c1 ^ k0;", [t_philox.test_philox_matches_bigint]),
    ("Philox key schedule", "k0 += W0; k1 += W1;", "k0 += W1; k1 += W0;", [t_philox.test_philox_matches_bigint]),
    ("init mantissa bits", "(double)(r[col % 4] >> 9) + 0.5) * (1.0 / 8388608.0)", "(double)(r[col % 4] >> 8) + 0.5) * (1.0 / 16777216.0)",
     [t_sgns.test_init_tables]),
    ("init word index", "uint32_t)(col / 4), STREAM_INIT };", "uint32_t)(col / 2), STREAM_INIT };", [t_sgns.test_init_tables]),
    ("shared coefficients not rounded", "if (bf16_inputs) G = (double)bf16_rne((float)G);", ";",
     [t_shared.test_shared_with_bf16_rounding_matches_torch_bfloat16]),
    ("shared negatives unweighted", "double G = -neg_scale * sigmoid(S);", "double G = -sigmoid(S);",
     [t_shared.test_shared_equals_autograd_without_rounding]),
    ("bf16 rounding truncates", "u += 0x7FFFu + ((u >> 16) & 1u);", "u += 0u;",
     [t_shared.test_shared_with_bf16_rounding_matches_torch_bfloat16]),
    ("sequential mode reuses stale source row", "for (int32_t i = 0; i < d; ++i) x[i] = (float)(xs[i] + dx[i]);",
     "for (int32_t i = 0; i < d; ++i) x[i] = (float)(xs[i] + 0.5 * dx[i]);", [t_seq.test_sequential_equals_batches_of_one]),
    ("pair score reads the wrong second table", "const float* S = second_from_context ? C : X;",
     "const float* S = second_from_context ? X : C;", [t_score.test_score_hand_values_and_table_choice]),
    ("pair score indexes the second node by the first", "const float* b = S + (int64_t)pairs[2 * i + 1] * d;",
     "const float* b = S + (int64_t)pairs[2 * i] * d;", [t_score.test_score_agrees_with_the_positive_loss_term]),
    ("walk window one too narrow", "for (int32_t j = 1; j <= window; ++j) {", "for (int32_t j = 1; j < window; ++j) {",
     [t_walks.test_sample_count_of_full_walks]),
    ("walk sample direction reversed", "pairs_out[2 * n] = w[i];\n                pairs_out[2 * n + 1] = w[i + j];",
     "pairs_out[2 * n] = w[i + j];\n                pairs_out[2 * n + 1] = w[i];", [t_walks.test_worked_example]),
    ("walk sample index without the offset", "* (int64_t)window + (j - 1);", "* (int64_t)window;",
     [t_walks.test_worked_example]),
]


@pytest.mark.parametrize("name,find,repl,pins", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_pins_reject_planted_mistake(name, find, repl, pins, tmp_path):
    text = open(SRC).read()
    assert text.count(find) >= 1, f"mutation target not found: {find}"
    mutated = tmp_path / "ne_oracle_mut.c"
    mutated.write_text(text.replace(find, repl, 1))
    so = tmp_path / "libmut.so"
    subprocess.run(["gcc", "-O1", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off", "-o", str(so), str(mutated), "-lm"],
                   check=True, capture_output=True)
    oracle._load()
    real = oracle._lib
    oracle._lib = oracle._bind(ctypes.CDLL(str(so)))
    try:
        caught = False
        for pin in pins:
            try:
                pin()
            except AssertionError:
                caught = True
                break
        assert caught, f"no pin noticed: {name}"
    finally:
        oracle._lib = real
