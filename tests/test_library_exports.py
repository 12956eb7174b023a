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


def test_workspace_bytes_follows_from_the_shape_alone():
    # host-only call: no context, no GPU.  Sections are 256-byte aligned, optional ones add what they hold.
    from paper_2207_09682_amd import Context
    from paper_2207_09682_amd import binding as b
    N, F, nb, L = 1_000_000, 28, 255, 255
    base = Context.workspace_bytes_for(N, F, nb, L, flags=0)
    assert base % 256 == 0
    # three row-id lists, three gradient lists, packed and fp32 gradients, flags, a pool of 3L+1 histograms
    floor = N * (3 * 4 + 3 * 2 + 2 + 8 + 1) + (3 * L + 1) * F * nb * 8
    assert floor < base < floor + (512 << 20)
    bind = Context.workspace_bytes_for(N, F, nb, L, flags=b.WS_BIND)
    assert N * F <= bind - base <= N * F + 1024
    rows = Context.workspace_bytes_for(N, F, nb, L, flags=b.WS_ROW_COPIES)
    assert 3 * N * F <= rows - base <= 3 * N * F + 1024
    boost = Context.workspace_bytes_for(N, F, nb, L, flags=b.WS_BOOST)
    assert 8 * N <= boost - base <= 8 * N + 1024
    allf = Context.workspace_bytes_for(N, F, nb, L)
    assert allf - base == (bind - base) + (rows - base) + (boost - base)
    # shapes that cannot keep leaf-ordered rows ignore that flag
    assert Context.workspace_bytes_for(N, 200, nb, L, flags=b.WS_ROW_COPIES) == Context.workspace_bytes_for(N, 200, nb, L, flags=0)
    # 16-bit bins double the copy of a bound matrix
    d16 = Context.workspace_bytes_for(N, 40, 600, L, 2, flags=b.WS_BIND) - Context.workspace_bytes_for(N, 40, 600, L, 2, flags=0)
    assert 2 * N * 40 <= d16 <= 2 * N * 40 + 1024
    for bad in (dict(n_rows=0), dict(n_bins=1), dict(n_bins=300), dict(max_leaves=0), dict(max_leaves=5000)):
        kw = dict(n_rows=N, n_features=F, n_bins=nb, max_leaves=L)
        kw.update(bad)
        with pytest.raises(b.QgbdtError):
            Context.workspace_bytes_for(**kw)
    with pytest.raises(b.QgbdtError):
        Context.workspace_bytes_for(N, F, nb, L, flags=64)
