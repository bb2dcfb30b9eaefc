"""Host-side checks that need no GPU: the library loads, exports the declared ABI and rejects bad arguments."""
import ctypes as C
import os
import re

import pytest

import paper_2210_15748_amd as dz

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "dessert.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dessert_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    l = dz.lib()
    names = declared_symbols()
    assert len(names) >= 14
    for n in names:
        assert hasattr(l, n), n
    assert sorted(dz.EXPORTS) == names
    assert dz.version().startswith("dessert-gfx950")


def test_create_rejects_bad_configs_before_touching_a_device():
    l = dz.lib()
    h = C.c_void_p()

    def status(**kw):
        base = dict(d=128, L=32, C=7, dtype=0, proj_kind=0, device=0, seed=1, proj_dev=None, stream=None)
        base.update(kw)
        cfg = dz.Config(**base)
        return l.dessert_create(C.byref(cfg), C.byref(h))

    assert status(C=17) == dz.EINVAL and "C must be" in dz.last_error()
    assert status(C=0) == dz.EINVAL
    assert status(L=30) == dz.EINVAL and "multiple of 4" in dz.last_error()
    assert status(L=132) == dz.EINVAL
    assert status(d=0) == dz.EINVAL
    assert status(dtype=3) == dz.EINVAL
    assert status(proj_kind=1) == dz.EINVAL and "Gaussian" in dz.last_error()
    assert l.dessert_create(None, C.byref(h)) == dz.EINVAL
    assert h.value is None


def test_null_handles_are_rejected():
    l = dz.lib()
    assert l.dessert_hash(None, None, 1, None) == dz.EINVAL
    assert l.dessert_build_index(None, None, 0, None, 0, None, None) == dz.EINVAL
    assert l.dessert_search(None, None, None, 1, None, None, 5, None, 0, None, None) == dz.EINVAL
    assert l.dessert_search(None, None, None, 1, None, None, 0, None, 0, None, None) == dz.EINVAL   # k = 0
    assert "k must be" in dz.last_error()
    assert l.dessert_scores(None, None, None, 1, None, None, None, 0, None) == dz.EINVAL
    assert l.dessert_set_algo(None, 0, 0) == dz.EINVAL
    assert l.dessert_code_bytes(None, 10) == 0
    l.dessert_destroy(None)


def test_no_gpu_means_loud_failure_not_a_fallback():
    import torch
    if torch.cuda.is_available():
        pytest.skip("GPU present")
    with pytest.raises(dz.DessertError) as e:
        cfg = dz.Config(d=128, L=32, C=7, dtype=0, proj_kind=0, device=0, seed=1, proj_dev=None, stream=None)
        h = C.c_void_p()
        dz._check(dz.lib().dessert_create(C.byref(cfg), C.byref(h)))
    assert e.value.status == dz.EHIP
    assert "no CPU path" in str(e.value)


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2210_15748_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower().replace("no fallback", ""), (dirpath, f)


def test_bench_refuses_more_than_one_gpu_with_a_message():
    """Nothing here uses a second GPU: the benchmark says so instead of running a single-GPU job under another label."""
    import pathlib
    import subprocess
    import sys
    bench = pathlib.Path(__file__).resolve().parent.parent / "bench.py"
    r = subprocess.run([sys.executable, str(bench), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in (r.stdout + r.stderr)
