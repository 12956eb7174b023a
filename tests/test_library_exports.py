"""CPU-side checks of the boundary: the HIP library loads and exports every symbol
that include/qgbdt.h declares (no compute call is made here)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "qgbdt.h")).read()
    return sorted(set(re.findall(r"QGBDT_API\s+[\w\s\*]+?\b(qgbdt_\w+)\s*\(", text)))


def test_header_declares_the_six_calls_of_the_path():
    names = _declared()
    for n in ("qgbdt_quantize_gradients", "qgbdt_build_histograms", "qgbdt_subtract_histograms",
              "qgbdt_find_best_splits", "qgbdt_refit_leaves", "qgbdt_grow_tree", "qgbdt_partition_rows"):
        assert n in names


def test_library_exports_every_declared_symbol():
    from paper_2207_09682_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2207_09682_amd import build
        build.build()
    lib = ctypes.CDLL(binding.LIB_PATH)
    for n in _declared():
        assert hasattr(lib, n), n
    assert sorted(binding.EXPORTS) == _declared()


def test_binding_refuses_to_run_without_gpu():
    import torch
    from paper_2207_09682_amd import Context
    if torch.cuda.is_available():
        pytest.skip("GPU present")
    with pytest.raises(RuntimeError):
        Context(100, 4, 16)


def test_product_does_not_import_oracle():
    pkg = os.path.join(ROOT, "paper_2207_09682_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text and "qgbdt_ref_" not in text, f
    otext = open(os.path.join(ROOT, "oracle", "__init__.py")).read() + open(os.path.join(ROOT, "oracle", "qgbdt_oracle.c")).read()
    assert "paper_2207_09682_amd" not in otext and "libqgbdt.so" not in otext
