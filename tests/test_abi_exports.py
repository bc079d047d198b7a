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


def test_bench_refuses_more_than_one_gpu():
    """One GPU only: asking for more must end with a message, before anything touches a device."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "one GPU" in (r.stderr + r.stdout)
