"""Are the pins sharp?  Each case plants one plausible mistake in a copy of the oracle's source (a dropped
term, a wrong sign or index, a transposed operand, a missing factor), runs the pin tests against the
mutant on the CPU, and requires at least one of the named pins to fail.  The real oracle is untouched."""
import os
import types

import pytest

import test_oracle_pins as pins

ORACLE = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle", "peagle_oracle.py")

# (what is planted, text to find, replacement, pins expected to catch it: (name, args) ...)
MUTATIONS = [
    ("depth-0 keys visible strictly before the anchor", "depth0 = (e == 0) & (j <= i)", "depth0 = (e == 0) & (j < i)",
     [("test_mask_matches_dependency_rules", (16, 4)), ("test_mask_closed_form_counts", (16, 4))]),
    ("chain keys of deeper depths visible", "chain = (e >= 1) & (e <= d) & (j == i)", "chain = (e >= 1) & (j == i)",
     [("test_mask_matches_dependency_rules", (16, 4))]),
    ("chain keys of other anchors visible", "chain = (e >= 1) & (e <= d) & (j == i)", "chain = (e >= 1) & (e <= d) & (j <= i)",
     [("test_mask_closed_form_counts", (16, 4))]),
    ("wrong KV head of a query head", "return h // (Hq // Hkv)", "return h % Hkv",
     [("test_library_autograd_with_independent_mask", (12, 3, 4, 2, 8))]),
    ("scale left out of the scores (forward)", "S = scale * (q[rb, h, :] @ k[cols, g, :].T)", "S = (q[rb, h, :] @ k[cols, g, :].T)",
     [("test_depth0_rows_are_plain_causal_attention", ())]),
    ("dQ without the softmax scale", "dQ[sl, h, :] = scale * (dS @ Kc)", "dQ[sl, h, :] = (dS @ Kc)",
     [("test_finite_differences", ())]),
    ("dK from the unscaled, untransposed score gradient", "dK[cols, g, :] += scale * (dS.T @ q[rb, h, :])",
     "dK[cols, g, :] += scale * (dS.T @ do[rb, h, :])", [("test_finite_differences", ())]),
    ("Delta dropped from dS", "dS = P * (dP - delta)", "dS = P * dP", [("test_finite_differences", ())]),
    ("dV from the probabilities of the wrong orientation", "dV[cols, g, :] += P.T @ dOh", "dV[cols, g, :] += P.T @ q[rb, h, :]",
     [("test_finite_differences", ())]),
    ("segment keys without the cumulative depth-0 context", "n0 = np.arange(0, b_hi)", "n0 = np.arange(b_lo, b_hi)",
     [("test_partitioned_equals_unpartitioned", ([0, 5, 16],))]),
    ("deeper depths do not inherit their segment", "A[g][p] = segment_holding(head)", "A[g][p] = segment_holding(p)",
     [("test_partition_worked_example_from_paper", ())]),
    ("rotation turned the wrong way for gradients", "    if inverse:\n        s = -s\n", "    if inverse:\n        s = s\n",
     [("test_rope_step_gradients_against_finite_differences", ()), ("test_rope_is_an_isometry_with_the_transpose_as_inverse", ())]),
    ("interleaved instead of half-split feature pairs",
     "x1, x2 = x[..., :D // 2], x[..., D // 2:]\n    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)",
     "x1, x2 = x[..., 0::2], x[..., 1::2]\n    return np.stack([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1).reshape(x.shape)",
     [("test_rope_hand_computed_vector_and_frequencies", ())]),
    ("frequency exponent without the factor two", "** (-2.0 * j / D)", "** (-1.0 * j / D)",
     [("test_rope_hand_computed_vector_and_frequencies", ())]),
    ("position ids without the depth", "return i + d\n", "return i\n",
     [("test_position_ids_follow_the_rows_named_in_the_paper_example", ())]),
    ("positions do not restart per packed sequence", "return ta - first[ts] + td", "return ta + td",
     [("test_position_ids_follow_the_rows_named_in_the_paper_example", ())]),
    ("shared-vector gradient summed over every stored position", 'r["dK"][L:].sum(axis=0), "dV_shared"', 'r["dK"].sum(axis=0), "dV_shared"',
     [("test_shared_chain_vectors_gradients_against_finite_differences", ())]),
    ("drafting rows see every new key", "M[d, n + e] = visible(n, d, n, e)", "M[d, n + e] = True",
     [("test_draft_decode_against_library_attention_and_closed_forms", ())]),
]


def _mutant(find, replace):
    src = open(ORACLE).read()
    assert src.count(find) >= 1, f"mutation target not found: {find!r}"
    mod = types.ModuleType("peagle_oracle_mutant")
    exec(compile(src.replace(find, replace), "peagle_oracle_mutant", "exec"), mod.__dict__)
    return mod


@pytest.mark.parametrize("what,find,replace,catchers", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_a_planted_mistake_fails_a_pin(monkeypatch, what, find, replace, catchers):
    monkeypatch.setattr(pins, "orc", _mutant(find, replace))
    caught = []
    for name, args in catchers:
        try:
            getattr(pins, name)(*args)
        except AssertionError:      # only a failed comparison counts; any other exception propagates
            caught.append(name)
    assert caught, f"no pin noticed: {what}"


def test_the_unmutated_oracle_passes_the_same_pins():
    for _, _, _, catchers in MUTATIONS:
        for name, args in catchers:
            getattr(pins, name)(*args)
