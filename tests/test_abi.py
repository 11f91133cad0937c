"""The C-ABI library loads and exports every entry point include/thia.h declares (no GPU needed)."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    src = open(os.path.join(ROOT, "include", "thia.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(thia_[a-z_0-9]+)\s*\(", src)))


def test_library_exports_every_declared_symbol():
    from paper_2102_08481_amd import EXPORTS, LIB_PATH
    if not os.path.exists(LIB_PATH):
        from paper_2102_08481_amd import build
        build.build()
    names = declared_functions()
    assert "thia_load_model" in names and "thia_detect_chunk" in names and "thia_run_plan" in names
    L = ctypes.CDLL(LIB_PATH)
    for n in names:
        assert hasattr(L, n), f"{n} is declared in thia.h but not exported"
    assert sorted(EXPORTS) == names          # the binding covers exactly the header


def test_header_is_plain_c():
    import subprocess
    r = subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-fsyntax-only", "-x", "c", os.path.join(ROOT, "include", "thia.h")],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr


def test_product_package_never_imports_the_oracle():
    pkg = os.path.join(ROOT, "paper_2102_08481_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                txt = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in txt and "from oracle" not in txt and "thia_oracle" not in txt, f


def test_bench_refuses_more_than_one_gpu():
    """One GPU per run: the benchmark says so and exits before touching a device."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout.strip() == ""
