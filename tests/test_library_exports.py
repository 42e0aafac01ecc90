"""CPU-side checks of the boundary: the built library loads and exports every symbol that
include/som.h declares; the binding refuses host tensors and has no fallback."""
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "som.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(som_[a-z_0-9]+)\s*\(", text)))


def test_header_declares_the_expected_entry_points():
    names = declared_symbols()
    for must in ("som_init", "som_train_epoch_dense", "som_train_epoch_csr", "som_train", "som_umatrix"):
        assert must in names


def test_library_exports_every_declared_symbol():
    from paper_1305_1422_amd import capi
    lib = capi.load()
    for name in declared_symbols():
        assert hasattr(lib, name), f"libsom.so does not export {name}"
    assert sorted(capi.EXPORTS) == declared_symbols()


def test_binding_refuses_host_tensors():
    torch = pytest.importorskip("torch")
    from paper_1305_1422_amd import capi
    with pytest.raises(TypeError):
        capi._ptr(torch.zeros(3), torch.float32, "x")


def test_product_path_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_1305_1422_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h")):
                src = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in src.replace("no CPU fallback", ""), f"{f} mentions the oracle"
