"""The product path and the oracle stay apart, and the product fails loudly without its library."""
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PKG = os.path.join(ROOT, "paper_2407_13726_amd")


def _sources(top, exts):
    for d, _, files in os.walk(top):
        if "_build" in d or "__pycache__" in d:
            continue
        for f in files:
            if f.endswith(exts):
                yield os.path.join(d, f)


def test_binding_raises_when_the_library_is_missing(monkeypatch, tmp_path):
    from paper_2407_13726_amd import dastac

    monkeypatch.setattr(dastac, "_lib", None)
    monkeypatch.setattr(dastac, "LIB_PATH", str(tmp_path / "libdastac_hip.so"))
    with pytest.raises(RuntimeError):
        dastac.lib()
    with pytest.raises(RuntimeError):
        dastac.tri_count(4)  # every entry point goes through lib(): there is no CPU fallback


def test_package_never_touches_the_oracle():
    for path in _sources(PKG, (".py", ".hip", ".h")):
        text = open(path).read()
        assert not re.search(r"^\s*(import|from)\s+oracle\b", text, re.M), path
        assert "dastac_oracle" not in text, path


def test_oracle_includes_nothing_of_the_package():
    for path in _sources(os.path.join(ROOT, "oracle"), (".c", ".h", ".py")):
        text = open(path).read()
        assert "paper_2407_13726_amd" not in text and "csrc" not in text and "index_poly" not in text, path
        for inc in re.findall(r'#include\s+"([^"]+)"', text):
            assert False, "%s includes %s" % (path, inc)
