"""The GPU library and the CPU oracle stay apart: neither imports, includes or
links the other, and the package has no CPU fallback to route through."""
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def sources(top, exts):
    for base, _, files in os.walk(os.path.join(ROOT, top)):
        if "__pycache__" in base:
            continue
        for f in files:
            if f.endswith(exts):
                yield os.path.join(base, f)


def test_package_never_touches_the_oracle():
    for path in sources("paper_2009_03816_amd", (".py", ".hip", ".h", ".cpp")):
        text = open(path).read()
        assert not re.search(r"^\s*(from|import)\s+oracle\b", text, re.M), path
        assert "pso_ps_oracle" not in text and "oracle/" not in text, path
    header = open(os.path.join(ROOT, "include", "pso_ps.h")).read()
    assert "oracle" not in header.lower()


def test_oracle_never_touches_the_package_or_hip():
    for path in sources("oracle", (".py", ".cpp", ".h")):
        text = open(path).read()
        assert "paper_2009_03816_amd" not in text, path
        assert "hip/hip_runtime" not in text and "libpso_ps.so" not in text, path
        assert not re.search(r'#include\s+"(pso_ps|tile_order)\.h"', text), path


def test_only_the_allowed_entry_points_load_the_oracle():
    allowed = {os.path.join(ROOT, "bench.py"), os.path.join(ROOT, "__graft_entry__.py")}
    for name in os.listdir(ROOT):
        path = os.path.join(ROOT, name)
        if name.endswith(".py") and path not in allowed:
            assert "oracle" not in open(path).read(), path
    bench = open(os.path.join(ROOT, "bench.py")).read()
    body = bench[bench.index("def cpu_baseline"):bench.index("def main")]
    assert "from oracle import" in body and "from oracle import" not in bench.replace(body, "")
