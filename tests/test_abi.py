"""CPU-side checks of the boundary: the library loads, exports what include/aj.h declares, and
refuses bad configurations before touching a GPU."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "aj.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(aj_[a-z_]+)\s*\(", text)))


def test_header_declares_the_three_calls():
    names = declared_functions()
    for n in ("aj_create", "aj_verify", "aj_destroy"):
        assert n in names


def test_library_exports_every_declared_symbol():
    import paper_2504_20039_amd as aj
    lib = ctypes.CDLL(aj.library_path())
    for n in declared_functions():
        assert hasattr(lib, n), f"libaj.so does not export {n}"
    assert set(declared_functions()) == set(aj.exported_symbols())


def test_header_compiles_as_c():
    import subprocess
    src = '#include "aj.h"\nint main(void){aj_config c; (void)c; return AJ_OK;}\n'
    r = subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"),
                        "-x", "c", "-", "-fsyntax-only"], input=src, text=True, capture_output=True)
    assert r.returncode == 0, r.stderr


def test_bad_configurations_are_refused_without_a_gpu():
    import paper_2504_20039_amd as aj
    good = dict(B=1, K=8, d_t=256, d_d=128, V=1024, dtype=aj.AJ_BF16)
    for bad in (dict(K=0), dict(K=1024), dict(V=0), dict(d_t=0), dict(d_t=100), dict(d_d=4), dict(B=-1),
                dict(dtype=7), dict(feat_offset=2), dict(kernel=9), dict(d_d=-8)):
        with pytest.raises(aj.AjError) as e:
            aj.aj_create(**{**good, **bad})
        assert e.value.status == -1
    assert "invalid" in aj.aj_strerror(-1)
    assert aj.aj_strerror(0) == "ok"


def test_product_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2504_20039_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower().replace("no cpu fallback", ""), f
    text = open(os.path.join(ROOT, "oracle", "__init__.py")).read() + open(os.path.join(ROOT, "oracle", "aj_oracle.c")).read()
    assert "paper_2504_20039_amd" not in text and "libaj.so" not in text
