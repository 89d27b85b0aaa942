"""The oracle and the HIP path share nothing, and the product path has no fallback (CPU only, static checks)."""
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PKG = os.path.join(ROOT, "paper_2602_11812_amd")


def _sources(top, exts):
    out = []
    for base, dirs, files in os.walk(top):
        dirs[:] = [d for d in dirs if d not in ("__pycache__", "_build")]
        out += [os.path.join(base, f) for f in files if f.endswith(exts)]
    return sorted(out)


def test_product_sources_never_reach_for_the_oracle():
    """Nothing under the package (Python or HIP/C++) or the public headers imports, includes or names oracle/."""
    files = _sources(PKG, (".py", ".hip", ".h", ".cpp")) + _sources(os.path.join(ROOT, "include"), (".h",))
    assert len(files) > 15
    for f in files:
        text = open(f).read()
        assert not re.search(r"^\s*(import|from)\s+oracle\b", text, flags=re.M), f
        assert "egtp_oracle" not in text and "oracle/" not in text, f


def test_oracle_sources_never_reach_for_the_product():
    """The oracle imports neither the package nor torch, and includes none of the product's headers."""
    files = _sources(os.path.join(ROOT, "oracle"), (".py", ".c", ".h"))
    assert len(files) >= 3
    for f in files:
        text = open(f).read()
        assert "paper_2602_11812_amd" not in text, f
        assert not re.search(r"^\s*(import|from)\s+torch\b", text, flags=re.M), f
        assert not re.search(r'#include\s+"(\.\./)*(include|paper_)', text), f
        assert "egtp.h" not in text and "kernels.h" not in text, f


def test_only_tests_smoke_and_the_cpu_baseline_import_the_oracle():
    """Top-level files: bench.py imports the oracle inside its cpu_baseline leg only, __graft_entry__ inside
    build() / smoke() only -- never at module level, so importing either does not pull the oracle in."""
    for name in ("bench.py", "__graft_entry__.py"):
        text = open(os.path.join(ROOT, name)).read()
        assert not re.search(r"^(import|from)\s+oracle\b", text, flags=re.M), name      # no module-level import
        assert re.search(r"^\s+import oracle\b", text, flags=re.M), name                 # but a local one exists


def test_binding_fails_loudly_without_the_library(monkeypatch, tmp_path):
    from paper_2602_11812_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "libegtp.so"))
    with pytest.raises(RuntimeError, match="no fallback"):
        binding.load_library()
    with pytest.raises(RuntimeError):
        binding.egtp_static_scratch_bytes()            # any entry point goes through the same loader
