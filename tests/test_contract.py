"""Host-side contract of the entry scripts (no GPU needed): one GPU only, no fallback when the library is missing, and
the product package never reaches into the oracle."""
import os
import re
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_refuses_more_than_one_gpu_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "--gpus 2 is not supported" in r.stderr and "one GPU" in r.stderr
    assert r.stdout.strip() == ""                       # no JSON line that could be mistaken for a measurement


def test_binding_raises_when_the_library_is_missing():
    code = ("import paper_2511_11729_amd.binding as b\n"
            "b.LIB_PATH = '/nonexistent/libharli.so'\n"
            "try:\n    b.lib()\nexcept RuntimeError as e:\n    print('RAISED', e)\n")
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, cwd=ROOT, timeout=120)
    assert r.returncode == 0 and "RAISED" in r.stdout and "no CPU fallback" in r.stdout


def test_product_package_and_benchmark_paths_do_not_import_the_oracle():
    pat = re.compile(r"^\s*(from|import)\s+oracle\b", re.M)
    pkg = os.path.join(ROOT, "paper_2511_11729_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith(".py"):
                assert not pat.search(open(os.path.join(dirpath, f)).read()), f
    # bench.py may use the oracle for its cpu_baseline leg only: one import, inside that block
    src = open(os.path.join(ROOT, "bench.py")).read()
    hits = [m.start() for m in pat.finditer(src)]
    assert len(hits) == 1 and "no_cpu_baseline" in src[max(0, hits[0] - 400): hits[0]]
