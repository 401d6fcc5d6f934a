"""The oracle's pins must catch plausible mistakes.

Each case plants one mistake in a copy of the oracle's C source (on the CPU, in a temporary
directory), builds it, swaps it in for the real library and re-runs the pins of
tests/test_oracle.py: at least one pin has to fail for every mutant, and all pins pass again on
the untouched source."""
import ctypes
import os
import subprocess
import tempfile

import pytest

import oracle
import test_oracle as pins

SRC_DIR = os.path.dirname(os.path.abspath(oracle.__file__))

PIN_FUNCS = [
    lambda: [pins.test_exact_matches_library_attention(*a) for a in
             [(1, 1, 1, 37, 8, False), (2, 4, 2, 50, 16, True), (1, 8, 2, 129, 64, True)]],
    pins.test_exact_brute_force_python_loops,
    pins.test_closed_forms_zero_queries_and_constant_values,
    pins.test_one_column_per_group_is_exact,
    lambda: pins.test_duplicated_columns_make_the_approximation_exact(2),
    pins.test_worked_example_fig4_eq2,
    pins.test_residual_identity_eq2_eq3,
    pins.test_keys_are_fused_not_values,
    pins.test_gray_table_properties,
    pins.test_sort_worked_example_fig5,
    pins.test_sort_is_ascending_stable_permutation,
    pins.test_projection_signs_and_bit_order,
    pins.test_lsh_invariances,
    pins.test_hyperplane_generator_statistics,
    pins.test_blocks_are_independent_and_single_block_is_global,
    pins.test_permutation_tables_are_valid_and_sorted,
    lambda: [pins.test_exact_with_other_key_count_matches_library_attention(*a) for a in
             [(1, 1, 1, 1, 37, 8, True), (2, 4, 2, 20, 50, 16, True), (1, 6, 3, 64, 33, 32, False)]],
    pins.test_exact_with_other_key_count_scalar_loops,
    lambda: [pins.test_last_queries_of_a_square_problem(c) for c in (False, True)],
    pins.test_worked_example_fig4_right_side,
    pins.test_mirrored_form_is_the_transpose_of_the_form_with_roles_exchanged,
    pins.test_mirrored_form_residual_identity_and_block_tables,
    pins.test_mirrored_form_exact_cases,
]

# (name, text in the oracle source, replacement)
MUTANTS = [
    ("sort descending", "hash[idx[j]] > hash[ci]", "hash[idx[j]] < hash[ci]"),
    ("unstable ties", "hash[idx[j]] > hash[ci]", "hash[idx[j]] >= hash[ci]"),
    ("sample the group's last column", "acc += (double)qi[perm[j * G]] * kfn[j];", "acc += (double)qi[perm[j * G + G - 1]] * kfn[j];"),
    ("fusion drops a member", "for (int g = 0; g < G; ++g) acc += (double)kn[perm[j * G + g]];",
     "for (int g = 0; g + 1 < G || g == 0; ++g) acc += (double)kn[perm[j * G + g]];"),
    ("fusion ignores the permutation", "acc += (double)kn[perm[j * G + g]];", "acc += (double)kn[j * G + g];"),
    ("plane 0 in the lowest bit", "code |= bit << (n_planes - 1 - pl);", "code |= bit << pl;"),
    ("zero counts as positive", "(acc > 0.0f) ? 1u : 0u", "(acc >= 0.0f) ? 1u : 0u"),
    ("negative projections set the bit", "(acc > 0.0f) ? 1u : 0u", "(acc < 0.0f) ? 1u : 0u"),
    ("causal mask off by one", "int n_vis = causal ? i + shift + 1 : Nk; /* shift", "int n_vis = causal ? (i + shift > 0 ? i + shift : 1) : Nk; /* shift"),
    ("causal mask ignores the extra keys", "int n_vis = causal ? i + shift + 1 : Nk; /* shift", "int n_vis = causal ? i + 1 : Nk; /* shift"),
    ("approximation's causal mask ignores the extra keys", "int n_keys = causal ? r0 + rows + shift : Nk;", "int n_keys = causal ? r0 + rows : Nk; shift = 0;"),
    ("keys addressed with the query count", "const float *kh = k + ((size_t)b * p->Hkv + h / rep) * Nk * d;\n        const float *vh", "const float *kh = k + ((size_t)b * p->Hkv + h / rep) * N * d;\n        const float *vh"),
    ("mirrored form samples the group's last key column", "acc += qf[j] * (double)kn[perm[j * G]];", "acc += qf[j] * (double)kn[perm[j * G + G - 1]];"),
    ("mirrored form drops a query column from the fusion", "for (int g = 0; g < G; ++g) acc += (double)qi[perm[j * G + g]];", "for (int g = 0; g + 1 < G || g == 0; ++g) acc += (double)qi[perm[j * G + g]];"),
    ("mirrored form uses the first K block's grouping everywhere", "const uint8_t *perm = perm_k + (size_t)(n0 / Bc) * d;", "const uint8_t *perm = perm_k;"),
    ("mirrored form hashes the wrong rows of K", "lsh_block(kh, d, n0, rows, R, Bc,", "lsh_block(kh, d, 0, rows, R, Bc,"),
    ("scale applied twice", "s[n] = scale * acc;", "s[n] = scale * scale * acc;"),
    ("GQA head mapping by modulo", "kh = k + ((size_t)b * p->Hkv + h / rep) * Nk * d;\n        const float *vh", "kh = k + ((size_t)b * p->Hkv + h % p->Hkv) * Nk * d;\n        const float *vh"),
    ("Gray rank replaced by Gray code", "for (uint32_t g = code; g; g >>= 1) rank ^= g;", "rank = code ^ (code >> 1);"),
    ("projection matrix read transposed", "R[(size_t)pl * Br + r], acc);", "R[(size_t)r * n_planes + pl], acc);"),
    ("projection walks the block's rows backwards", "R[(size_t)pl * Br + r], acc);", "R[(size_t)pl * Br + (rows - 1 - r)], acc);"),
    ("softmax denominator misses a term", "for (int n = 0; n < n_vis; ++n) {\n    s[n] = exp(s[n] - m);", "for (int n = 0; n < n_vis; ++n) {\n    if (n == 1) { s[n] = exp(s[n] - m); continue; }\n    s[n] = exp(s[n] - m);"),
    ("values transposed with keys in P.V", "const float *vr = vh + (size_t)n * d;", "const float *vr = vh + (size_t)(n_vis - 1 - n) * d;"),
    ("hyperplane fields not centred", "(float)(sum - 2L * 65535L) / 65536.0f", "(float)(sum) / 65536.0f"),
]


def _build(source_text, workdir, tag):
    c_path = os.path.join(workdir, f"oracle_{tag}.c")
    so_path = os.path.join(workdir, f"oracle_{tag}.so")
    with open(c_path, "w") as f:
        f.write(source_text)
    subprocess.run(["gcc", "-std=c11", "-O1", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off", "-mfma",
                    "-I", SRC_DIR, "-o", so_path, c_path, "-lm"], check=True)
    lib = ctypes.CDLL(so_path)
    lib.oracle_gray_hash.restype = ctypes.c_uint32
    lib.oracle_gray_hash.argtypes = [ctypes.c_uint32, ctypes.c_int, ctypes.c_int]
    return lib


def _failing_pins():
    failed = []
    for i, fn in enumerate(PIN_FUNCS):
        try:
            fn()
        except (AssertionError, ValueError):
            failed.append(i)
    return failed


@pytest.fixture(scope="module")
def source():
    return open(os.path.join(SRC_DIR, "distr_attn_oracle.c")).read()


def test_untouched_source_passes_every_pin(source, monkeypatch):
    with tempfile.TemporaryDirectory() as tmp:
        monkeypatch.setattr(oracle, "_lib", _build(source, tmp, "clean"))
        assert _failing_pins() == []


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_pins_catch_a_planted_mistake(source, monkeypatch, name, old, new):
    assert source.count(old) >= 1, f"mutation site for '{name}' not found in the oracle source"
    with tempfile.TemporaryDirectory() as tmp:
        monkeypatch.setattr(oracle, "_lib", _build(source.replace(old, new), tmp, "mutant"))
        assert _failing_pins(), f"no pin noticed: {name}"
