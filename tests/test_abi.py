"""CPU-only checks of the boundary: the library loads and exports every symbol
the header declares; the binding refuses to run without a GPU (no fallback)."""

import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "artopk.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(artopk_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_are_exported():
    import paper_2312_02493_amd as pkg

    names = _declared_symbols()
    assert {"artopk_variance", "artopk_select_topk", "artopk_gather_sum", "artopk_scatter_residual",
            "artopk_step", "artopk_create", "artopk_destroy"} <= set(names)
    lib = pkg.load_library()
    for name in names:
        assert hasattr(lib, name), name
    assert sorted(pkg.exported_symbols()) == names
    assert lib.artopk_version() >= 100


def test_no_cpu_fallback():
    import torch
    import paper_2312_02493_amd as pkg

    if torch.cuda.is_available():
        pytest.skip("GPU present")
    with pytest.raises(RuntimeError):
        pkg.Context(2, 1024, 16)


def test_product_does_not_import_oracle():
    pkg_dir = os.path.join(ROOT, "paper_2312_02493_amd")
    for dirpath, _, files in os.walk(pkg_dir):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                src = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in src.lower(), f
