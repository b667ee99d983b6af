"""The product and its checker stay apart, and the product has no fallback.

The oracle is test infrastructure: nothing under the package may import, include, link or
open it, and nothing under oracle/ may use the package.  Without the built HIP library the
binding must refuse to work instead of computing anything some other way.
"""
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PKG = os.path.join(ROOT, "paper_2302_02599_amd")
ORACLE = os.path.join(ROOT, "oracle")


def sources(top, suffixes):
    for base, _, files in os.walk(top):
        if "__pycache__" in base:
            continue
        for name in files:
            if name.endswith(suffixes):
                yield os.path.join(base, name)


def test_the_package_never_names_the_oracle():
    pat = re.compile(r"\boracle\b|ckpt_oracle|libckpt_oracle", re.I)
    for path in list(sources(PKG, (".py", ".hip", ".cpp", ".h"))) + list(sources(os.path.join(ROOT, "include"), (".h",))):
        text = open(path, encoding="utf-8").read()
        hits = [ln for ln in text.splitlines() if pat.search(ln)]
        assert not hits, f"{path}: {hits[:3]}"


def test_the_oracle_never_names_the_package():
    pat = re.compile(r"paper_2302_02599_amd|libckpt_dp|ckpt_dp\.h|ckpt_roofs")
    for path in sources(ORACLE, (".py", ".c", ".h")):
        text = open(path, encoding="utf-8").read()
        hits = [ln for ln in text.splitlines() if pat.search(ln)]
        assert not hits, f"{path}: {hits[:3]}"


def test_the_two_sides_share_no_header_or_source_file():
    pkg_names = {os.path.basename(p) for p in sources(PKG, (".hip", ".cpp", ".h", ".c"))}
    pkg_names |= {os.path.basename(p) for p in sources(os.path.join(ROOT, "include"), (".h",))}
    oracle_names = {os.path.basename(p) for p in sources(ORACLE, (".c", ".h", ".cpp"))}
    assert not (pkg_names & oracle_names)
    for path in sources(ORACLE, (".c", ".h")):
        for inc in re.findall(r'#include\s+"([^"]+)"', open(path, encoding="utf-8").read()):
            assert os.path.basename(inc) not in pkg_names, (path, inc)


def test_without_the_built_library_the_binding_refuses(monkeypatch, tmp_path):
    import paper_2302_02599_amd.binding as binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_LIB_PATH", str(tmp_path / "libckpt_dp.so"))
    with pytest.raises(ImportError, match="no fallback"):
        binding.load_library()
    with pytest.raises(ImportError):
        binding.ckpt_row_pitch(10)
