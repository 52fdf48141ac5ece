"""The product path must stand on its own: nothing under the package may import, load or call the
CPU oracle (or the benchmark's baselines), and the package must refuse to work without its HIP library."""
import os
import re
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PKG = os.path.join(ROOT, "paper_2101_07956_amd")


def _sources():
    for base, _, files in os.walk(PKG):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h", ".cpp", ".c")):
                yield os.path.join(base, f)


def test_package_never_touches_the_oracle():
    for path in _sources():
        text = open(path).read()
        assert not re.search(r"^\s*(import|from)\s+oracle\b", text, re.M), path
        assert "liboracle" not in text and "gather_oracle" not in text, path
        if os.path.basename(path) not in ("baseline_cpu_centric.hip", "build.py", "tune.py"):
            assert "libud_baseline" not in text and "udb_" not in text, path


def test_oracle_never_touches_the_package():
    for base, _, files in os.walk(os.path.join(ROOT, "oracle")):
        for f in files:
            if f.endswith((".py", ".c", ".h")):
                text = open(os.path.join(base, f)).read()
                assert "paper_2101_07956_amd" not in text and "libud" not in text, f
                assert not re.search(r"#\s*include\s*<hip|import\s+torch|hipcc", text), f


def test_missing_library_fails_loudly(tmp_path):
    # the binding, placed where no libud.so exists, must refuse to import: there is no fallback path
    (tmp_path / "binding.py").write_text(open(os.path.join(PKG, "binding.py")).read())
    r = subprocess.run([sys.executable, "-c", "import binding"], cwd=tmp_path, capture_output=True, text=True)
    assert r.returncode != 0
    assert "ImportError" in r.stderr and "no fallback" in r.stderr.lower()
