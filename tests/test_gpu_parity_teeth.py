"""Would the GPU parity tests notice a wrong result?  The HIP path is left alone; the mistake is planted
in the ORACLE (a copy of ``oracle/da_oracle.c`` with one change, built on the CPU), and a slice of
``tests/test_gpu_parity.py`` is run against that copy in a child process: the comparison must fail.
An unchanged copy, run the same way, must pass."""
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "da_oracle.c")

# (name, text in da_oracle.c, replacement, -k expression selecting the parity tests that must object)
CASES = [
    ("heat_subtracts", "rn[d] = rn[d] + c[d];", "rn[d] = rn[d] - c[d];", "test_heat_and_cool_step and tiny"),
    ("distance_drops_first_coordinate",
     "for (int d = 0; d < D; ++d) {\n                double t = x[d] - c[d];",
     "for (int d = 1; d < D; ++d) {\n                double t = x[d] - c[d];", "test_assign_step and tiny"),
    ("mean_divides_by_count_plus_one", "/ (double)cnt[k];", "/ (double)(cnt[k] + 1);", "test_update_step and tiny"),
    ("error_is_a_sum", "return N > 0 ? total / (double)N : 0.0;", "return total;", "test_quant_error and tiny"),
    ("cool_adds", "xn[d] = xn[d] - c[d];", "xn[d] = xn[d] + c[d];", "test_encode and tiny"),
    ("argmin_prefers_the_second_best", "codes[n * M + m] = (uint8_t)ibest;",
     "codes[n * M + m] = (uint8_t)(isecond >= 0 ? isecond : ibest);", "test_lockstep_sweeps and tiny"),
]


def _run(tmp_path, text, expr):
    dst = tmp_path / "da_oracle_copy.c"
    dst.write_text(text)
    return subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_gpu_parity.py"),
                           "-m", "gpu", "-x", "-q", "-p", "no:cacheprovider", "-k", expr],
                          cwd=ROOT, env=dict(os.environ, DA_ORACLE_SRC=str(dst)),
                          capture_output=True, text=True, timeout=600)


def test_parity_slice_passes_against_a_faithful_copy(tmp_path):
    expr = " or ".join("(%s)" % c[3] for c in CASES)
    p = _run(tmp_path, open(SRC).read(), expr)
    assert p.returncode == 0, p.stdout[-2000:] + p.stderr[-2000:]
    assert " passed" in p.stdout


@pytest.mark.parametrize("name,old,new,expr", CASES, ids=[c[0] for c in CASES])
def test_parity_objects_to_a_mistake_planted_in_the_oracle(tmp_path, name, old, new, expr):
    text = open(SRC).read()
    assert text.count(old) >= 1, "the passage to mutate is gone: update the table"
    p = _run(tmp_path, text.replace(old, new, 1), expr)
    assert p.returncode == 1, "the parity tests did not object to '%s'\n%s" % (name, p.stdout[-1500:] + p.stderr[-1500:])
    assert " failed" in p.stdout, p.stdout[-1500:]
