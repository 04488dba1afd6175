"""Host-side checks that need no GPU: the C-ABI library loads and exports every
symbol the public headers declare (msgemm.h: the library; msgemm_measure.h: the
comparison kernel and the yardsticks), and the binding mirrors the headers."""
import ctypes
import os
import re

import pytest

from paper_2310_06178_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
INCLUDE = os.path.join(ROOT, "include")
HEADERS = sorted(f for f in os.listdir(INCLUDE) if f.endswith(".h"))


def declared_functions(headers=None):
    names = set()
    for h in headers or HEADERS:
        text = open(os.path.join(INCLUDE, h)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(msgemm_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_header_declares_the_three_named_entry_points():
    assert HEADERS == ["msgemm.h", "msgemm_measure.h"]
    names = declared_functions(["msgemm.h"])
    for must in ("msgemm_plan", "msgemm_build_lut", "msgemm_run"):
        assert must in names
    # the library's own header holds no measurement aid
    assert not [n for n in names if n.startswith("msgemm_calib_") or n == "msgemm_dequant_mfma_run"]


def test_library_exports_every_declared_symbol():
    if not os.path.exists(binding.LIB_PATH):
        pytest.fail("libmsgemm.so has not been built (python -m paper_2310_06178_amd.build)")
    lib = ctypes.CDLL(binding.LIB_PATH)
    for name in declared_functions():
        assert hasattr(lib, name), f"{name} is declared under include/ but not exported"


def test_binding_mirrors_header():
    names = declared_functions()
    assert sorted(binding.EXPORTS) == names
    for name in names:
        if name in ("msgemm_status_string", "msgemm_last_hip_error", "msgemm_version"):
            continue
        assert hasattr(binding, name)


def test_status_strings_and_version_without_gpu():
    assert binding.status_string(0) == "ok"
    assert "invalid" in binding.status_string(binding.ERR_INVALID_ARG)
    assert binding.version().count(".") == 1
    assert "unknown" in binding.status_string(-99)


def test_product_path_does_not_touch_the_oracle():
    pkg = os.path.join(ROOT, "paper_2310_06178_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text, f
                assert "msgemm_oracle" not in text, f
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c", ".h")):
            text = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_2310_06178_amd" not in text and "libmsgemm.so" not in text, f
