"""Would the GPU parity tests notice a wrong result?  The HIP path is left alone; the mistake is planted
in the ORACLE (a copy of ``oracle/da_oracle.c`` with one change, built on the CPU and loaded as a second
instance of the oracle module), and the matching test of ``tests/test_gpu_parity.py`` is called with that
instance in place of the oracle: its comparison must fail.  With an unchanged copy, loaded the same way, the
same calls must pass."""
import contextlib
import importlib.util
import os
import sys

import pytest

import test_gpu_beam as beam
import test_gpu_parity as parity
import test_gpu_pca as pca

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "da_oracle.c")

# (name, text in da_oracle.c, replacement, the GPU test that must object: a name in test_gpu_parity.py, run on
# its "tiny" case, or (module, name, arguments before the oracle))
CASES = [
    ("heat_subtracts", "rn[d] = rn[d] + c[d];", "rn[d] = rn[d] - c[d];", "test_heat_and_cool_step"),
    ("distance_drops_first_coordinate",
     "for (int d = 0; d < D; ++d) {\n                double t = x[d] - c[d];",
     "for (int d = 1; d < D; ++d) {\n                double t = x[d] - c[d];", "test_assign_step"),
    ("mean_divides_by_count_plus_one", "/ (double)cnt[k];", "/ (double)(cnt[k] + 1);", "test_update_step"),
    ("error_is_a_sum", "return N > 0 ? total / (double)N : 0.0;", "return total;", "test_quant_error"),
    ("cool_adds", "xn[d] = xn[d] - c[d];", "xn[d] = xn[d] + c[d];", "test_encode"),
    ("argmin_prefers_the_second_best", "codes[n * M + m] = (uint8_t)ibest;",
     "codes[n * M + m] = (uint8_t)(isecond >= 0 ? isecond : ibest);", "test_lockstep_sweeps"),
    # multi-path encoding (Sec. 3.3) and the rotation of the improved k-means (Sec. 3.2)
    ("beam_error_adds_the_codeword", "const double t = (double)x[d] - a[d] - c[d];",
     "const double t = (double)x[d] - a[d] + c[d];", (beam, "test_beam_step_locked", ("tiny", 3))),
    ("beam_answer_is_the_last_path", "memcpy(codes + (size_t)n * M, pre + (size_t)n * Lc * M, (size_t)M);",
     "memcpy(codes + (size_t)n * M, pre + ((size_t)n * Lc + (Lc - 1)) * M, (size_t)M);",
     (beam, "test_encode_beam_against_oracle", ("tiny", 5))),
    ("rotation_transposed", "(transpose ? R[(size_t)j * D + i] : R[(size_t)i * D + j])",
     "(transpose ? R[(size_t)i * D + j] : R[(size_t)j * D + i])", (pca, "test_rotate", ("tiny",))),
]


def _call(test, oracle):
    if isinstance(test, str):
        return getattr(parity, test)("tiny", oracle)
    module, name, args = test
    return getattr(module, name)(*args, oracle)


def _oracle_from(tmp_path, name, text):
    """A second instance of the oracle module, built from `text` (the module reads DA_ORACLE_SRC when it is
    executed and keeps its own library handle)."""
    src = tmp_path / ("da_oracle_%s.c" % name)
    src.write_text(text)
    spec = importlib.util.spec_from_file_location("oracle_copy_" + name, os.path.join(ROOT, "oracle", "__init__.py"))
    mod = importlib.util.module_from_spec(spec)
    os.environ["DA_ORACLE_SRC"] = str(src)
    try:
        spec.loader.exec_module(mod)
    finally:
        del os.environ["DA_ORACLE_SRC"]
    mod.build(force=True)
    return mod


@contextlib.contextmanager
def _fresh_parity_state():
    """The parity module caches oracle states per case: what a planted mistake computes must neither come from
    that cache nor stay in it."""
    saved, saved_contraction = parity._cache, [m._CONTRACTION for m in (parity, beam, pca)]
    parity._cache = {}
    parity._CONTRACTION = beam._CONTRACTION = pca._CONTRACTION = 0
    try:
        yield
    finally:
        parity._cache = saved
        parity._CONTRACTION, beam._CONTRACTION, pca._CONTRACTION = saved_contraction


def test_parity_slice_passes_against_a_faithful_copy(tmp_path):
    copy = _oracle_from(tmp_path, "faithful", open(SRC).read())
    with _fresh_parity_state():
        for case in CASES:
            _call(case[3], copy)


@pytest.mark.parametrize("name,old,new,test", CASES, ids=[c[0] for c in CASES])
def test_parity_objects_to_a_mistake_planted_in_the_oracle(tmp_path, name, old, new, test):
    text = open(SRC).read()
    assert text.count(old) >= 1, "the passage to mutate is gone: update the table"
    wrong = _oracle_from(tmp_path, name, text.replace(old, new, 1))
    with _fresh_parity_state():
        with pytest.raises(AssertionError):
            _call(test, wrong)
    sys.modules.pop("oracle_copy_" + name, None)
