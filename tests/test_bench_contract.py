"""Host-side checks of the measurement contract (no GPU): one GPU only, and the product never reaches the oracle."""
import os
import re
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "ONE GPU" in (r.stdout + r.stderr)


def test_product_path_never_imports_the_oracle():
    """The oracle is test infrastructure: only tests/, the smoke entry and bench.py's cpu_baseline may touch it."""
    pkg = os.path.join(ROOT, "paper_2503_02356_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"\boracle\b", text), os.path.join(dirpath, f)
    for name in ("bench_sweep.py", "bench_longtail.py", "bench_memory.py", "bench_offload.py"):
        assert not re.search(r"\boracle\b", open(os.path.join(ROOT, name)).read()), name
    bench = open(os.path.join(ROOT, "bench.py")).read()
    uses = [m.start() for m in re.finditer(r"from oracle|import oracle", bench)]
    start, end = bench.index("def cpu_baseline"), bench.index("def measure")
    assert uses and all(start < u < end for u in uses)


def test_binding_fails_loudly_without_the_library(tmp_path):
    code = ("import sys; sys.path.insert(0, %r)\n"
            "from paper_2503_02356_amd import binding as B\n"
            "B.LIB_PATH = %r\n"
            "try:\n    B.lib()\nexcept Exception as e:\n    print('raised', type(e).__name__); sys.exit(0)\n"
            "sys.exit(1)\n") % (ROOT, str(tmp_path / "missing.so"))
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True)
    assert r.returncode == 0 and "raised" in r.stdout, r.stdout + r.stderr
