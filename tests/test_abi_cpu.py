"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, and rejects bad arguments before touching HIP."""
import ctypes
import os
import re
import subprocess
import sys

import pytest

from paper_1509_05194_amd import hclae

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "hclae.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(hclae_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = hclae.lib()
    names = _declared()
    assert set(names) == set(hclae.EXPORTS), (names, hclae.EXPORTS)
    for n in names:
        assert hasattr(L, n), n


@pytest.mark.parametrize("args,ok", [
    ((10, 16, 4, 16), True), ((0, 4, 1, 1), True), ((1 << 31, 16, 4, 16), False),
    ((-1, 16, 4, 16), False), ((10, 0, 4, 16), False), ((10, 18, 4, 16), False),
    ((10, 4100, 4, 16), False), ((10, 16, 0, 16), False), ((10, 16, 257, 16), False),
    ((10, 16, 4, 0), False), ((10, 16, 4, 257), False), ((10, 960, 16, 256), True),
])
def test_check_shape(args, ok):
    assert (hclae.check_shape(*args) == hclae.OK) == ok


def test_create_rejects_bad_shapes_before_hip():
    L = hclae.lib()
    h = ctypes.c_void_p()
    assert L.hclae_create(None, 10, 16, 4, 16, None) == hclae.EINVAL
    for bad in [(0, 16, 4, 16), (10, 15, 4, 16), (10, 16, 4, 300), (10, 16, 0, 16)]:
        assert L.hclae_create(ctypes.byref(h), *bad, None) == hclae.EINVAL
        assert not h.value
        assert b"shape" in L.hclae_last_error(None)


def test_null_ctx_is_einval():
    L = hclae.lib()
    out = ctypes.c_double()
    assert L.hclae_quant_error(None, None, 0, 16, ctypes.byref(out)) == hclae.EINVAL
    assert L.hclae_encode(None, None, 1, 16, None, 4, 16, None, None) == hclae.EINVAL
    assert L.hclae_anneal_stage(None, 0, 1, 16, None, 4, 16, None, None, 1, None, None) == hclae.EINVAL
    assert L.hclae_sweep(None, None, 1, 16, None, 4, 16, None, None, 1, 0, None, None) == hclae.EINVAL
    assert L.hclae_anneal(None, 1, 16, None, 4, 16, None, None, 1, 2, None, None) == hclae.EINVAL
    assert L.hclae_heat(None, 0, 1, 16, None, 4, 16, None, None) == hclae.EINVAL
    assert L.hclae_cool(None, 0, 1, 16, None, 4, 16, None, None) == hclae.EINVAL
    assert L.hclae_assign(None, 0, 1, 16, None, None, 4, 16, None, None) == hclae.EINVAL
    assert L.hclae_update(None, 0, 1, 16, None, None, 4, 16, None, None) == hclae.EINVAL
    assert L.hclae_destroy(None) == hclae.EINVAL


def test_no_device_fails_loudly():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(hclae.HclaeError) as e:
        hclae.Context(100, 16, 4, 16, stream=0)
    assert e.value.code == hclae.EHIP


def test_product_path_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_1509_05194_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h")):
                src = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in src.lower().replace("the cpu oracle's tests", ""), f


def test_null_ctx_is_einval_for_the_settings():
    L = hclae.lib()
    assert L.hclae_set_pruning(None, 1) == hclae.EINVAL
    assert L.hclae_set_contraction(None, 0) == hclae.EINVAL
    assert L.hclae_set_beam_width(None, 10) == hclae.EINVAL


def test_bench_refuses_more_than_one_gpu():
    """The build runs on one GPU: bench.py says so and exits before it touches a device."""
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert p.returncode != 0
    assert "ONE GPU" in p.stderr
