"""CPU-side checks of the boundary: the shared library loads, exports every function the header
declares, rejects calls without a context, and the product package is independent of the oracle."""
import ctypes
import os
import re
import subprocess
import sys

import pytest
import torch

from paper_1712_02912_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADERS = sorted(os.path.join(ROOT, "include", f) for f in os.listdir(os.path.join(ROOT, "include")) if f.endswith(".h"))


def declared_functions():
    names = []
    for header in HEADERS:
        text = open(header).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names += re.findall(r"^(?:int|const char \*|void|size_t)\s*\*?(\w+)\s*\(", text, flags=re.M)
    return names


def test_header_declares_the_named_entry_points():
    names = declared_functions()
    for required in ("pq_build_luts", "pq_quantize_luts", "pq_adc_scan_topk", "ivf_adc_search"):
        assert required in names
    assert len(names) == len(set(names))


def test_library_exports_every_declared_function():
    lib = ctypes.CDLL(binding.LIB_PATH)
    for name in declared_functions():
        assert hasattr(lib, name), f"{name} is declared in include/*.h but not exported"


def test_binding_lists_exactly_the_declared_functions():
    assert sorted(binding.EXPORTS) == sorted(declared_functions())


def test_version_string():
    lib = ctypes.CDLL(binding.LIB_PATH)
    lib.pq_version.restype = ctypes.c_char_p
    assert lib.pq_version().decode().startswith("pqadc")


def test_calls_without_context_are_rejected():
    lib = ctypes.CDLL(binding.LIB_PATH)
    null = ctypes.c_void_p()
    assert lib.pq_destroy(null) in (0, -1)
    assert lib.pq_set_profiling(null, 1) == -1
    assert lib.pq_build_luts(null, null, null, 1, 8, 1, 16, null) == -1
    assert lib.pq_quantize_luts(null, null, 1, 16, 16, null, null, null, null) == -1
    assert lib.pq_adc_scan_topk(null, null, ctypes.c_int64(0), 0, null, 0, 1, 8, 256, 1, null, null) == -1
    assert lib.ivf_adc_search(null, null, null, 8, 256, 0, null, 1, 1, 1, null, null) == -1


@pytest.mark.skipif(torch.cuda.is_available(), reason="checks the behaviour on a machine without a GPU")
def test_create_fails_loudly_without_a_gpu():
    lib = ctypes.CDLL(binding.LIB_PATH)
    ctx = ctypes.c_void_p()
    assert lib.pq_create(ctypes.byref(ctx), 0, None) < 0
    assert not ctx.value
    with pytest.raises(Exception):
        binding.Context(0)


def test_product_package_does_not_touch_the_oracle():
    pkg = os.path.join(ROOT, "paper_1712_02912_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"^\s*(from|import)\s+oracle|pq_oracle|liborc", text, flags=re.M), f
    code = "import sys; import paper_1712_02912_amd, paper_1712_02912_amd.binding; " \
           "sys.exit(1 if any(m.startswith('oracle') for m in sys.modules) else 0)"
    assert subprocess.run([sys.executable, "-c", code], cwd=ROOT).returncode == 0


def test_oracle_does_not_touch_the_product_package():
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c", ".h")):
            text = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_1712_02912_amd" not in text and "libpqadc" not in text, f
