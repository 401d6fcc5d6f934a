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
import test_oracle_bwd as bwd_pins

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


BWD_SRC = os.path.join(SRC_DIR, "distr_attn_oracle_bwd.c")


def _build(source_text, workdir, tag, bwd_text=None):
    c_path = os.path.join(workdir, f"oracle_{tag}.c")
    so_path = os.path.join(workdir, f"oracle_{tag}.so")
    with open(c_path, "w") as f:
        f.write(source_text)
    bwd_path = BWD_SRC
    if bwd_text is not None:
        bwd_path = os.path.join(workdir, f"oracle_bwd_{tag}.c")
        with open(bwd_path, "w") as f:
            f.write(bwd_text)
    subprocess.run(["gcc", "-std=c11", "-O1", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off", "-mfma",
                    "-I", SRC_DIR, "-o", so_path, c_path, bwd_path, "-lm"], check=True)
    lib = ctypes.CDLL(so_path)
    lib.oracle_gray_hash.restype = ctypes.c_uint32
    lib.oracle_gray_hash.argtypes = [ctypes.c_uint32, ctypes.c_int, ctypes.c_int]
    return lib


def _failing_pins(funcs=None):
    failed = []
    for i, fn in enumerate(PIN_FUNCS if funcs is None else funcs):
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


# The backward pass and the row statistics (distr_attn_oracle_bwd.c) against their own pins.
BWD_PIN_FUNCS = [
    lambda: [bwd_pins.test_distr_backward_matches_automatic_differentiation(kw) for kw in bwd_pins.CASES],
    lambda: [bwd_pins.test_exact_backward_matches_library_attention(kw) for kw in
             (dict(), dict(causal=True), dict(H=6, Hkv=2, N=13, Nk=31, causal=True))],
    lambda: [bwd_pins.test_backward_is_the_finite_difference_of_the_forward(c) for c in (False, True)],
    bwd_pins.test_structure_of_the_gradient,
    lambda: [bwd_pins.test_row_statistics(kw) for kw in (dict(), dict(causal=True, N=20, Nk=29), dict(H=4, Hkv=2, causal=True))],
]

BWD_MUTANTS = [
    ("row term D dropped from dS", "const double ds = s[n] * (dp - D);", "const double ds = s[n] * dp;"),
    ("dV weighted by dS instead of P", "dvh[(size_t)n * d + c] += s[n] * (double)doi[c];", "dvh[(size_t)n * d + c] += s[n] * (dp - D) * (double)doi[c];"),
    ("dQ lands on the group's last member", "dqh[(size_t)i * d + perm[j * G]] = p->scale * dqr[j];", "dqh[(size_t)i * d + perm[j * G + G - 1]] = p->scale * dqr[j];"),
    ("dQ spread over every member of the group", "for (int j = 0; j < ng; ++j) dqh[(size_t)i * d + perm[j * G]] = p->scale * dqr[j];",
     "for (int j = 0; j < ng; ++j) for (int g = 0; g < G; ++g) dqh[(size_t)i * d + perm[j * G + g]] = p->scale * dqr[j];"),
    ("dK only to the group's first member", "for (int g = 0; g < G; ++g)\n                  dkh[", "for (int g = 0; g < 1; ++g)\n                  dkh["),
    ("dK without the scale", "+= p->scale * dkf[(size_t)n * ng + j];", "+= dkf[(size_t)n * ng + j];"),
    ("dK_f taken with the unsampled column", "dkf[(size_t)n * ng + j] += ds * (double)qi[perm[j * G]];", "dkf[(size_t)n * ng + j] += ds * (double)qi[perm[j * G + G - 1]];"),
    ("gradient forgets the other query heads of a kv head", "for (int h = hk * rep; h < (hk + 1) * rep; ++h) {", "for (int h = hk * rep; h < hk * rep + 1; ++h) {"),
    ("causal shift dropped in the backward", "const int n_vis = p->causal ? i + shift + 1 : Nk;\n              const float *qi", "const int n_vis = p->causal ? i + 1 : Nk;\n              const float *qi"),
    ("row statistics without the maximum added back", "lse[(size_t)bh * N + i] = m + log(sum);", "lse[(size_t)bh * N + i] = log(sum);"),
    ("row statistics of the exact scores for the approximation", "const uint8_t *perm = distr ? table + ((size_t)bh * Tq + i / Br) * d : NULL;", "const uint8_t *perm = NULL;"),
]


@pytest.fixture(scope="module")
def bwd_source():
    return open(BWD_SRC).read()


def test_untouched_backward_source_passes_its_pins(source, bwd_source, monkeypatch):
    with tempfile.TemporaryDirectory() as tmp:
        monkeypatch.setattr(oracle, "_lib", _build(source, tmp, "clean", bwd_source))
        assert _failing_pins(BWD_PIN_FUNCS) == []


@pytest.mark.parametrize("name,old,new", BWD_MUTANTS, ids=[m[0] for m in BWD_MUTANTS])
def test_backward_pins_catch_a_planted_mistake(source, bwd_source, monkeypatch, name, old, new):
    assert bwd_source.count(old) == 1, f"mutation site for '{name}' not found (or not unique) in the backward source"
    with tempfile.TemporaryDirectory() as tmp:
        monkeypatch.setattr(oracle, "_lib", _build(source, tmp, "mutant", bwd_source.replace(old, new)))
        assert _failing_pins(BWD_PIN_FUNCS), f"no pin noticed: {name}"
