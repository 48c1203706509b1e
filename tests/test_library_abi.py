"""CPU-side checks of the C-ABI library: it loads, exports every declared symbol, and its
host-only entry points behave (no GPU needed, no kernels run)."""
import os
import re

from paper_2011_09017_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "cmpz.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(cmp_[a-z_]+)\s*\(", text)))


def test_library_loads_and_exports_every_declared_symbol():
    L = binding.lib()
    names = declared_symbols()
    assert len(names) >= 10
    for n in names:
        assert hasattr(L, n), n
    assert sorted(binding.EXPORTS) == names


def test_host_only_entry_points():
    cfg = binding.cmp_default_config()
    assert (cfg.radius, cfg.chunk, cfg.sub, cfg.guard_shift) == (512, 4096, 128, 7)
    for code in (0, -1, -2, -3, -4, -5, 1):
        assert binding.cmp_strerror(code) != "unknown code"
    assert binding.cmp_strerror(99) == "unknown code"
    assert binding.cmp_bound(None, (1, 1, 2, 2)) == 0


def test_product_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2011_09017_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                src = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in src.lower() or f == "workloads.py", f
