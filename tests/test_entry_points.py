"""Command-line and entry-point behaviour that needs no GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_refuses_more_than_one_gpu():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True,
                         text=True, timeout=300)
    assert res.returncode != 0
    assert "ONE GPU" in res.stderr + res.stdout
    assert not any(line.startswith("{") for line in res.stdout.splitlines())      # no result line


def test_graft_entry_exposes_build_and_smoke():
    sys.path.insert(0, ROOT)
    import __graft_entry__ as entry
    assert callable(entry.build) and callable(entry.smoke)


def test_product_package_does_not_import_the_oracle():
    """The library side may never reach into the test oracle (or the other way round)."""
    pkg = os.path.join(ROOT, "paper_2004_14020_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".cpp", ".hpp", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text, f
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith(".py"):
            text = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_2004_14020_amd" not in text, f
