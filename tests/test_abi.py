"""CPU-only: the C-ABI library loads, exports what include/commrand.h declares, and validates arguments."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "commrand.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(cr_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_function():
    from paper_2504_18082_amd import binding as B
    lib = B.lib()
    names = declared_functions()
    assert len(names) >= 15
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(B.EXPORTS) == names
    assert B.cr_version().startswith("commrand")


def test_mix_count_from_percent():
    from paper_2504_18082_amd import binding as B
    import math
    # k percent of the communities present in the training set, rounded to nearest, at least one (Section 5, evaluated schemes)
    for k, c in ((0, 50), (12.5, 50), (25, 50), (50, 50), (100, 50), (12.5, 3), (50, 1), (12.5, 497)):
        assert B.cr_mix_count_from_percent(k, c) == min(c, max(1, math.floor(k * c / 100.0 + 0.5)))
    assert B.cr_mix_count_from_percent(12.5, 50) == 6
