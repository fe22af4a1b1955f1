"""Are the oracle's pins strong enough?  Each case plants ONE plausible mistake in a copy of the
oracle's source (a dropped term, a wrong sign or index, a transposed operand, a swapped argument),
builds it on the CPU and runs the pins of tests/test_oracle_pins.py and tests/test_oracle_ops.py
against the broken build: at least one of them has to fail.  A mutant that survives every pin means
the oracle could contain that mistake unnoticed."""
import os
import subprocess
import tempfile

import pytest

import test_oracle_ops as ops
import test_oracle_pins as pins

HERE = os.path.dirname(os.path.abspath(__file__))
SOURCE = os.path.join(os.path.dirname(HERE), "oracle", "sga_oracle.cpp")

# (name, text in the oracle's source, what it is replaced by)
MUTANTS = [
    ("sddmm reads the other operand backwards",
     "acc += X[(i * H + h) * D + d] * Y[(j * H + h) * D + d];",
     "acc += X[(i * H + h) * D + d] * Y[(j * H + h) * D + (D - 1 - d)];"),
    ("sddmm uses the destination row for both operands",
     "acc += X[(i * H + h) * D + d] * Y[(j * H + h) * D + d];",
     "acc += X[(i * H + h) * D + d] * Y[(i * H + h) * D + d];"),
    ("softmax forgets the scale in the weights",
     "U[e * H + h] = std::exp(scale * Z[e * H + h] - m) / sum;",
     "U[e * H + h] = std::exp(Z[e * H + h] - m / scale) / sum;"),
    ("lse drops the subtracted maximum",
     "lse[i * H + h] = m + std::log(sum);",
     "lse[i * H + h] = std::log(sum);"),
    ("no maximum is subtracted (overflow at large scores)",
     "double m = scale * Z[b * H + h];\n            for (int64_t e = b; e < t; ++e) m = std::fmax(m, scale * Z[e * H + h]);",
     "double m = 0.0;"),
    ("empty row reports lse = 0",
     "lse[i * H + h] = -std::numeric_limits<double>::infinity();",
     "lse[i * H + h] = 0.0;"),
    ("spmm takes head 0's weight for every head",
     "Y[(i * H + h) * D + d] += W[e * H + h] * X[(j * H + h) * D + d];",
     "Y[(i * H + h) * D + d] += W[e * H + 0] * X[(j * H + h) * D + d];"),
    ("spmm gathers the destination's own row",
     "Y[(i * H + h) * D + d] += W[e * H + h] * X[(j * H + h) * D + d];",
     "Y[(i * H + h) * D + d] += W[e * H + h] * X[(i * H + h) * D + d];"),
    ("serial transposed spmm gathers by source instead of destination",
     "for (int64_t k = 0; k < n_src * H * D; ++k) Y[k] = 0.0;\n    for (int64_t i = 0; i < n_dst; ++i)\n        for (int64_t e = indptr[i]; e < indptr[i + 1]; ++e) {\n            const int64_t j = indices[e];\n            for (int h = 0; h < H; ++h)\n                for (int d = 0; d < D; ++d)\n                    Y[(j * H + h) * D + d] += W[e * H + h] * X[(i * H + h) * D + d];",
     "for (int64_t k = 0; k < n_src * H * D; ++k) Y[k] = 0.0;\n    for (int64_t i = 0; i < n_dst; ++i)\n        for (int64_t e = indptr[i]; e < indptr[i + 1]; ++e) {\n            const int64_t j = indices[e];\n            for (int h = 0; h < H; ++h)\n                for (int d = 0; d < D; ++d)\n                    Y[(j * H + h) * D + d] += W[e * H + h] * X[(i * H + h) * D + (D - 1 - d)];"),
    ("grouped transposed spmm pairs every entry with the group's first destination",
     "const int64_t e = eid[(size_t)p], i = row[(size_t)p];",
     "const int64_t e = eid[(size_t)p], i = row[(size_t)start[(size_t)j]];"),
    ("grouped transposed spmm loses the last entry of a group",
     "for (int64_t p = start[(size_t)j]; p < start[(size_t)j + 1]; ++p) {\n            const int64_t e = eid",
     "for (int64_t p = start[(size_t)j]; p + 1 < start[(size_t)j + 1]; ++p) {\n            const int64_t e = eid"),
    ("softmax backward adds the row term instead of subtracting it",
     "dZ[e * H + h] = scale * U[e * H + h] * (dU[e * H + h] - dot);",
     "dZ[e * H + h] = scale * U[e * H + h] * (dU[e * H + h] + dot);"),
    ("softmax backward forgets the scale",
     "dZ[e * H + h] = scale * U[e * H + h] * (dU[e * H + h] - dot);",
     "dZ[e * H + h] = U[e * H + h] * (dU[e * H + h] - dot);"),
    ("softmax backward forgets the row term",
     "dZ[e * H + h] = scale * U[e * H + h] * (dU[e * H + h] - dot);",
     "dZ[e * H + h] = scale * U[e * H + h] * dU[e * H + h];"),
    ("dV is built from dZ instead of the weights",
     "spmm_t(n_dst, n_src, indptr, indices, H, D, U.data(), dY, dV);",
     "spmm_t(n_dst, n_src, indptr, indices, H, D, dZ.data(), dY, dV);"),
    ("dU pairs dY with K instead of V",
     "sga_sddmm(n_dst, indptr, indices, H, D, dY, V, dU.data());",
     "sga_sddmm(n_dst, indptr, indices, H, D, dY, K, dU.data());"),
    ("dQ gathers V instead of K",
     "sga_spmm(n_dst, indptr, indices, H, D, dZ.data(), K, dQ);",
     "sga_spmm(n_dst, indptr, indices, H, D, dZ.data(), V, dQ);"),
    ("dK uses the weights instead of dZ",
     "spmm_t(n_dst, n_src, indptr, indices, H, D, dZ.data(), Q, dK);",
     "spmm_t(n_dst, n_src, indptr, indices, H, D, U.data(), Q, dK);"),
]


def run_pins(oracle, gen):
    """Names of the pins that fail (AssertionError) against the currently loaded oracle build."""
    def forward_cases():
        for case in pins.test_forward_matches_dense_brute_force.pytestmark[0].args[1]:
            pins.test_forward_matches_dense_brute_force(oracle, gen, case)

    def autograd_cases():
        for case in pins.test_backward_matches_autograd_of_dense_form.pytestmark[0].args[1]:
            pins.test_backward_matches_autograd_of_dense_form(oracle, gen, case)

    checks = {
        "hand-worked example": lambda: pins.test_hand_worked_example(oracle),
        "dense brute force": forward_cases,
        "complete graph = SDPA": lambda: pins.test_complete_graph_is_textbook_attention(oracle),
        "closed forms": lambda: pins.test_closed_forms(oracle, gen),
        "forward invariances": lambda: pins.test_forward_invariances(oracle, gen),
        "large scores": lambda: pins.test_large_scores_are_stable(oracle, gen),
        "autograd of the dense form": autograd_cases,
        "finite differences": lambda: pins.test_backward_matches_finite_differences(oracle, gen),
        "backward invariants": lambda: pins.test_backward_invariants(oracle, gen),
        "operator definitions": ops.test_operator_functions_match_numpy_definitions,
        "merge of two entry sets": ops.test_merge_of_two_entry_sets_is_attention_over_their_union,
    }
    failed = []
    for name, check in checks.items():
        try:
            check()
        except AssertionError:
            failed.append(name)
    return failed


def test_the_unmodified_oracle_passes_every_pin(oracle, gen):
    assert run_pins(oracle, gen) == []


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(oracle, gen, name, old, new):
    text = open(SOURCE).read()
    assert text.count(old) == 1, f"the text to replace must occur exactly once in the oracle's source ({name})"
    with tempfile.TemporaryDirectory() as tmp:
        src, lib = os.path.join(tmp, "mutant.cpp"), os.path.join(tmp, "mutant.so")
        open(src, "w").write(text.replace(old, new))
        subprocess.check_call(["g++", "-O1", "-std=c++17", "-fopenmp", "-fPIC", "-shared", "-o", lib, src])
        good = oracle._load()
        oracle._lib = oracle._open(lib)
        try:
            with __import__("numpy").errstate(all="ignore"):
                failed = run_pins(oracle, gen)
        finally:
            oracle._lib = good
    print(f"  '{name}' fails: {', '.join(failed) if failed else 'NOTHING'}")
    assert failed, f"no pin notices the mistake: {name}"
