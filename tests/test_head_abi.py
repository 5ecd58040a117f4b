"""The library exports every function include/gllm_head.h declares (no GPU needed)."""
import os
import re

from paper_2504_14775_amd import binding as B
from paper_2504_14775_amd import head as HD

HEADER = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include", "gllm_head.h")


def test_library_exports_every_function_the_header_declares():
    text = re.sub(r"/\*.*?\*/", "", open(HEADER).read(), flags=re.S)
    declared = sorted(set(re.findall(r"\b(gllm_[a-z0-9_]+)\s*\(", text)))
    lib = B.load_library()
    for n in declared:
        assert hasattr(lib, n), n
    assert set(declared) == set(HD.EXPORTS)
