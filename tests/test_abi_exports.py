"""The built C-ABI library loads and exports every symbol include/als.h declares (no compute calls)."""
import os
import re

import paper_1808_03843_amd as P

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_header_symbols_are_exported():
    header = open(os.path.join(ROOT, "include", "als.h")).read()
    declared = set(re.findall(r"\b(als_[a-z_0-9]+)\s*\(", header))
    assert declared == set(P.EXPORTS), declared ^ set(P.EXPORTS)
    lib = P.load_library()
    for name in declared:
        assert getattr(lib, name) is not None


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_1808_03843_amd")
    for dirpath, _, files in os.walk(pkg):
        for fn in files:
            if fn.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, fn)).read()
                assert "import oracle" not in text and "from oracle" not in text and "als_oracle" not in text
