"""The C-ABI library loads and exports every entry point the header declares; host
argument checks work without a GPU (no compute is launched here)."""
import ctypes as C
import os

import pytest

from paper_2305_00645_amd import gtree


def test_library_exports_every_declared_symbol():
    L = gtree.load()
    syms = gtree.declared_symbols()
    assert len(syms) >= 20
    missing = [s for s in syms if not hasattr(L, s)]
    assert not missing, missing


def test_error_strings_and_null_checks():
    L = gtree.load()
    assert L.gt_strerror(0) == b"ok"
    assert b"order" in L.gt_strerror(gtree.GT_ESTATE)
    h = C.c_void_p()
    assert L.gt_ctx_create(C.byref(h), None) == gtree.GT_EINVAL
    assert L.gt_ctx_destroy(None) == gtree.GT_EINVAL
    assert L.gt_train_level(None, None, 0) == gtree.GT_EINVAL
    assert L.gt_infer_batch(None, None, None, 0, 0, None) == gtree.GT_EINVAL
    assert L.gt_train_export_size(None, 0) == 0


def test_product_does_not_import_oracle():
    """The product path never routes through the CPU oracle."""
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    for dirpath, _, files in os.walk(os.path.join(root, "paper_2305_00645_amd")):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower() or f == "gtree.py" and "import oracle" not in text, f
    text = open(os.path.join(root, "paper_2305_00645_amd", "gtree.py")).read()
    assert "import oracle" not in text and "from oracle" not in text
