"""Do the pins bite?  Plant one plausible mistake at a time in a copy of the
oracle's C source (on the CPU, in a temp dir), build it, and require that at
least one pin of the regular suite fails for it.  A mutant that survives means
the pins leave that mistake undetected.
"""
import os
import subprocess

import pytest

import oracle as oracle_pkg
import test_oracle_backward as B
import test_oracle_bias_and_inputs as G
import test_oracle_forward as F

SRC = os.path.join(os.path.dirname(oracle_pkg.__file__), "fwa_oracle.c")

# (name, text to find, replacement, occurrence index or None for all)
MUTANTS = [
    ("score_scale_dropped", "double sij = scale * dot;", "double sij = dot;", None),
    ("bias_transposed", "sij += bias[((size_t)h * L + i) * L + j];", "sij += bias[((size_t)h * L + j) * L + i];", None),
    ("bias_head_ignored", "sij += bias[((size_t)h * L + i) * L + j];", "sij += bias[((size_t)0 * L + i) * L + j];", None),
    ("mask_window_off_by_one", "(n % nW)", "((n + 1) % nW)", None),
    ("mask_dropped", "if (mask) sij +=", "if (0) sij +=", None),
    ("head_offset_wrong", "const double *kn = k + (size_t)n * L * C + (size_t)h * d;",
     "const double *kn = k + (size_t)n * L * C;", 0),
    ("row_max_not_subtracted", "exp(s[(size_t)i * L + j] - m)", "exp(s[(size_t)i * L + j])", None),
    ("normalisation_dropped", "for (int j = 0; j < L; ++j) p[(size_t)i * L + j] /= z;", "", None),
    ("pv_uses_p_transposed", "acc += p[(size_t)i * L + j] * vn[(size_t)j * C + c];",
     "acc += p[(size_t)j * L + i] * vn[(size_t)j * C + c];", None),
    ("dv_uses_p_untransposed", "acc += p[(size_t)i * L + j] * gn[(size_t)i * C + c];",
     "acc += p[(size_t)j * L + i] * gn[(size_t)i * C + c];", None),
    ("dp_operands_swapped", "acc += gn[(size_t)i * C + c] * vn[(size_t)j * C + c];",
     "acc += gn[(size_t)j * C + c] * vn[(size_t)i * C + c];", None),
    ("ds_sign", "(dp[(size_t)i * L + j] - delta)", "(dp[(size_t)i * L + j] + delta)", None),
    ("ds_delta_without_p", "delta += p[(size_t)i * L + l] * dp[(size_t)i * L + l];",
     "delta += dp[(size_t)i * L + l];", None),
    ("dq_scale_dropped", "dqn[(size_t)i * C + c] = scale * acc;", "dqn[(size_t)i * C + c] = acc;", None),
    ("dk_scale_dropped", "dkn[(size_t)j * C + c] = scale * acc;", "dkn[(size_t)j * C + c] = acc;", None),
    ("dq_uses_ds_transposed", "acc += ds[(size_t)i * L + j] * kn[(size_t)j * C + c];",
     "acc += ds[(size_t)j * L + i] * kn[(size_t)j * C + c];", None),
    ("dk_uses_ds_untransposed", "acc += ds[(size_t)i * L + j] * qn[(size_t)i * C + c];",
     "acc += ds[(size_t)j * L + i] * qn[(size_t)i * C + c];", None),
    ("dbias_scaled", "acc[e] += ds[e];", "acc[e] += scale * ds[e];", None),
    ("dbias_head_ignored", "partial + ((size_t)tid * heads + h) * LL", "partial + ((size_t)tid * heads) * LL", None),
    ("gather_offset_sign", "int dy = i / k - j / k + k - 1;", "int dy = j / k - i / k + k - 1;", None),
    ("label_mask_inverted", "labels[w * L + i] == labels[w * L + j] ? 0.0 : value",
     "labels[w * L + i] == labels[w * L + j] ? value : 0.0", None),
    ("label_mask_window_ignored", "labels[w * L + i] == labels[w * L + j]", "labels[i] == labels[j]", None),
    ("label_mask_value_hardwired", "labels[w * L + j] ? 0.0 : value", "labels[w * L + j] ? 0.0 : -100.0", None),
    ("gather_xy_swapped", "table[(size_t)h * T + dy * (2 * k - 1) + dx]", "table[(size_t)h * T + dx * (2 * k - 1) + dy]", None),
]


def _pins(o):
    """A fast subset of the regular pins, each bound to the oracle `o`."""
    yield lambda: F.test_brute_force_tiny(o, 3, 5, 4, 2, 3, True)
    yield lambda: F.test_brute_force_tiny(o, 4, 3, 2, 2, 2, False)
    yield lambda: F.test_L2_is_logistic(o)
    yield lambda: F.test_equal_keys_give_uniform_weights(o)
    yield lambda: F.test_constant_added_to_a_score_row_has_no_effect(o)
    yield lambda: F.test_feature_chunk_identity(o)
    yield lambda: F.test_heads_are_independent_channel_slices(o)
    yield lambda: F.test_joint_key_value_permutation_leaves_output_unchanged(o)
    yield lambda: B.test_central_differences(o, 3, 5, 4, 2, 3, True)
    yield lambda: B.test_central_differences(o, 4, 3, 2, 3, 2, True)
    yield lambda: B.test_dv_equals_p_transpose_do(o)
    yield lambda: B.test_dq_dk_scale_with_scale_only_through_chain_rule(o)
    yield lambda: G.test_gather_k2_written_out_by_hand(o)
    yield lambda: G.test_gather_depends_only_on_relative_offset(o, 3)
    yield lambda: G.test_scatter_is_the_adjoint_of_gather(o, 2)
    yield lambda: G.test_mask_from_labels_written_out_by_hand(o)


def _mutate(src, find, repl, occurrence):
    assert find in src, f"mutation site not found: {find!r}"
    if occurrence is None:
        return src.replace(find, repl)
    parts = src.split(find)
    return find.join(parts[:occurrence + 1]) + repl + find.join(parts[occurrence + 1:])


def test_unmutated_source_passes_the_subset(oracle):
    for pin in _pins(oracle):
        pin()


@pytest.mark.parametrize("name,find,repl,occ", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_mutant_is_caught(tmp_path, name, find, repl, occ):
    src = _mutate(open(SRC).read(), find, repl, occ)
    c = tmp_path / f"{name}.c"
    so = tmp_path / f"lib{name}.so"
    c.write_text(src)
    subprocess.run(["gcc", "-O1", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-w", "-o", str(so), str(c), "-lm"],
                   check=True)
    mutant = oracle_pkg.Oracle(str(so))
    caught = False
    for pin in _pins(mutant):
        try:
            pin()
        except (AssertionError, ValueError, FloatingPointError):
            caught = True
            break
    assert caught, f"no pin noticed the planted mistake '{name}'"
