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
    assert p.returncode != 0, "no pin noticed the planted mistake '%s'" % name
    assert "failed" in p.stdout or "error" in p.stdout.lower(), p.stdout[-1500:]
