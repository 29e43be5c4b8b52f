"""Do the pins of the oracle notice a plausible mistake?  Each case plants ONE mistake in a copy of
``oracle/da_oracle.c`` (a wrong sign, a dropped term, a wrong index, a reversed order ...), builds it,
and runs ``tests/test_oracle_pins.py`` against that copy in a child process: the run must fail.
Everything here happens on the CPU."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "da_oracle.c")

# (name, text in da_oracle.c, replacement, which occurrence)
MUTATIONS = [
    ("heat_subtracts", "rn[d] = rn[d] + c[d];", "rn[d] = rn[d] - c[d];", 0),
    ("cool_adds", "xn[d] = xn[d] - c[d];", "xn[d] = xn[d] + c[d];", 0),
    ("argmin_ties_to_highest_index", "if (k == 0 || s < best) {", "if (k == 0 || s <= best) {", 0),
    ("distance_drops_first_coordinate",
     "for (int d = 0; d < D; ++d) {\n                double t = x[d] - c[d];",
     "for (int d = 1; d < D; ++d) {\n                double t = x[d] - c[d];", 0),
    ("mean_divides_by_count_plus_one", "/ (double)cnt[k];", "/ (double)(cnt[k] + 1);", 0),
    ("update_reads_first_code_column", "int k = codes[n * M + m];", "int k = codes[n * M + 0];", 0),
    ("empty_cluster_overwritten", "if (cnt[k] > 0) {", "if (cnt[k] >= 0) {", 0),
    ("error_is_a_sum", "return N > 0 ? total / (double)N : 0.0;", "return total;", 0),
    ("stage_without_final_assign",
     "    da_assign(r, C, N, D, M, K, m, codes, NULL, NULL, NULL);\n    da_cool(r, codes, C, N, D, M, K, m);               /* r holds",
     "    da_cool(r, codes, C, N, D, M, K, m);               /* r holds", 0),
    ("sweep_runs_backwards",
     "for (int m = 0; m < M; ++m) {\n        double E = da_anneal_stage(m,",
     "for (int m = M - 1; m >= 0; --m) {\n        double E = da_anneal_stage(m,", 0),
    ("beam_ties_to_highest_path", "if (a->l != b->l) return a->l < b->l ? -1 : 1;",
     "if (a->l != b->l) return a->l > b->l ? -1 : 1;", 0),
    ("beam_error_adds_the_codeword", "const double t = (double)x[d] - a[d] - c[d];",
     "const double t = (double)x[d] - a[d] + c[d];", 0),
    ("beam_answer_is_the_last_path", "memcpy(codes + (size_t)n * M, pre + (size_t)n * Lc * M, (size_t)M);",
     "memcpy(codes + (size_t)n * M, pre + ((size_t)n * Lc + (Lc - 1)) * M, (size_t)M);", 0),
    ("encode_skips_the_residue_update",
     "        da_assign(r, C, N, D, M, K, m, codes, NULL, NULL, NULL);\n        da_cool(r, codes, C, N, D, M, K, m);\n    }\n}",
     "        da_assign(r, C, N, D, M, K, m, codes, NULL, NULL, NULL);\n    }\n}", 0),
    # online learning (Sec. 3.4) and the improved k-means (Sec. 3.2)
    ("online_counts_not_kept", "            cm[k] += 1;", "            cm[k] = 1;", 0),
    ("online_without_second_assign",
     "        da_assign(r, C, n, D, M, K, m, codes, NULL, NULL, NULL);\n        da_cool(r, codes, C, n, D, M, K, m);\n    }\n    return da_quant_error(r, n, D);",
     "        da_cool(r, codes, C, n, D, M, K, m);\n    }\n    return da_quant_error(r, n, D);", 0),
    ("rotation_transposed", "(transpose ? R[(size_t)j * D + i] : R[(size_t)i * D + j])",
     "(transpose ? R[(size_t)i * D + j] : R[(size_t)j * D + i])", 0),
    ("prefix_assignment_uses_all_coordinates", "for (int d = 0; d < dact; ++d) {", "for (int d = 0; d < D; ++d) {", 0),
    ("prefix_mean_over_the_prefix_only",
     "for (int d = 0; d < D; ++d) Cp[(size_t)k * D + d] = S[(size_t)k * D + d] / (double)cnt[k];",
     "for (int d = 0; d < dims[i]; ++d) Cp[(size_t)k * D + d] = S[(size_t)k * D + d] / (double)cnt[k];", 0),
    ("dictionary_not_rotated_back", "    da_rotate(Cp, K, D, R, 1, Cm);", "    da_rotate(Cp, K, D, R, 0, Cm);", 0),
    ("reconstruction_skips_the_last_dictionary",
     "        for (int m = 0; m < M; ++m) {\n            const double *c = C + ((size_t)m * K + codes[n * M + m]) * D;",
     "        for (int m = 0; m + 1 < M; ++m) {\n            const double *c = C + ((size_t)m * K + codes[n * M + m]) * D;", 0),
]


def _run_pins(env):
    return subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"),
                           "-x", "-q", "-p", "no:cacheprovider"],
                          cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)


def test_pins_pass_on_a_faithful_copy(tmp_path):
    """The harness itself: an unchanged copy, built and loaded through the same switch, passes."""
    dst = tmp_path / "da_oracle_copy.c"
    dst.write_text(open(SRC).read())
    p = _run_pins(dict(os.environ, DA_ORACLE_SRC=str(dst)))
    assert p.returncode == 0, p.stdout[-2000:] + p.stderr[-2000:]


@pytest.mark.parametrize("name,old,new,which", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_pins_catch_a_planted_mistake(tmp_path, name, old, new, which):
    text = open(SRC).read()
    assert text.count(old) >= which + 1, "the passage to mutate is gone: update the mutation table"
    pos = -1
    for _ in range(which + 1):
        pos = text.index(old, pos + 1)
    mutant = text[:pos] + new + text[pos + len(old):]
    dst = tmp_path / ("da_oracle_%s.c" % name)
    dst.write_text(mutant)
    p = _run_pins(dict(os.environ, DA_ORACLE_SRC=str(dst)))
    assert p.returncode == 1, "no pin noticed the planted mistake '%s'\n%s" % (name, p.stdout[-1500:] + p.stderr[-1500:])
    assert " failed" in p.stdout, p.stdout[-1500:]


# ---- the NumPy half of the oracle (schedule, principal axes, dictionary order, code statistics) ------------
PY_MUTATIONS = [
    ("schedule_rounds_down", "d = int(np.ceil(D ** (i / I) - 1e-9))", "d = int(np.floor(D ** (i / I) - 1e-9))"),
    ("axes_least_variance_first", 'order = np.argsort(-w, kind="stable")', 'order = np.argsort(w, kind="stable")'),
    ("variance_without_the_mean", "((C - C.mean(axis=1, keepdims=True)) ** 2)", "((C) ** 2)"),
    ("order_ascending", "key=lambda j: (-v[j], j)", "key=lambda j: (v[j], j)"),
    ("entropy_in_nats", "return float(-(p * np.log2(p)).sum())", "return float(-(p * np.log(p)).sum())"),
    ("information_adds_the_joint_entropy", "+ entropy_bits(J.sum(0)) - entropy_bits(J)",
     "+ entropy_bits(J.sum(0)) + entropy_bits(J)"),
    ("joint_histogram_of_one_column", "(codes[:, a].astype(np.int64), codes[:, b].astype(np.int64))",
     "(codes[:, a].astype(np.int64), codes[:, a].astype(np.int64))"),
]


def _run_pins_with_package(tmp_path, init_text):
    pkg = tmp_path / "oracle"
    pkg.mkdir()
    (pkg / "__init__.py").write_text(init_text)
    (pkg / "da_oracle.c").write_text(open(SRC).read())
    # the copied package is imported first, so every later "import oracle" of the child gets it
    code = ("import sys; sys.path.insert(0, %r); import oracle; assert oracle.__file__.startswith(%r); "
            "import pytest; sys.exit(pytest.main([%r, '-x', '-q', '-p', 'no:cacheprovider']))"
            % (str(tmp_path), str(tmp_path), os.path.join(ROOT, "tests", "test_oracle_pins.py")))
    env = {k: v for k, v in os.environ.items() if k != "DA_ORACLE_SRC"}
    return subprocess.run([sys.executable, "-c", code], cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)


def test_pins_pass_on_a_faithful_copy_of_the_package(tmp_path):
    p = _run_pins_with_package(tmp_path, open(os.path.join(ROOT, "oracle", "__init__.py")).read())
    assert p.returncode == 0, p.stdout[-2000:] + p.stderr[-2000:]


@pytest.mark.parametrize("name,old,new", PY_MUTATIONS, ids=[m[0] for m in PY_MUTATIONS])
def test_pins_catch_a_planted_mistake_in_the_numpy_half(tmp_path, name, old, new):
    text = open(os.path.join(ROOT, "oracle", "__init__.py")).read()
    assert text.count(old) == 1, "the passage to mutate is gone: update the mutation table"
    p = _run_pins_with_package(tmp_path, text.replace(old, new))
    assert p.returncode == 1, "no pin noticed the planted mistake '%s'\n%s" % (name, p.stdout[-1500:] + p.stderr[-1500:])
    assert " failed" in p.stdout, p.stdout[-1500:]
