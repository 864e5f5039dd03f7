"""The product and the CPU oracle stay apart: neither names, imports or loads the other, and the input
generators hold none of the method's arithmetic (no GPU needed)."""
import glob
import os
import re
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _files(*patterns):
    out = []
    for p in patterns:
        out += glob.glob(os.path.join(ROOT, p), recursive=True)
    return [f for f in out if os.path.isfile(f) and not f.endswith((".so", ".pyc"))]


def test_product_sources_never_mention_the_oracle():
    for f in _files("paper_2412_02252_amd/**/*", "include/*"):
        text = open(f, errors="replace").read().lower()
        assert "oracle" not in text, f


def test_oracle_sources_never_mention_the_product():
    for f in _files("oracle/*.py", "oracle/*.c", "oracle/*.h"):
        text = open(f, errors="replace").read()
        for word in ("paper_2412_02252_amd", "libpod.so", "pod.h", "csrc", "hip/"):
            assert word not in text, (f, word)


def test_importing_the_product_loads_no_oracle_module_and_vice_versa():
    code = ("import sys, {0}; bad = [m for m in sys.modules if m == '{1}' or m.startswith('{1}.')]; "
            "print(bad); sys.exit(1 if bad else 0)")
    for mod, other in (("paper_2412_02252_amd", "oracle"), ("oracle.pod_oracle", "paper_2412_02252_amd"),
                       ("oracle.pod_grouping", "paper_2412_02252_amd"),
                       ("oracle.pod_select", "paper_2412_02252_amd")):
        r = subprocess.run([sys.executable, "-c", code.format(mod, other)], cwd=ROOT, capture_output=True, text=True)
        assert r.returncode == 0, (mod, r.stdout, r.stderr)


def test_input_generators_hold_no_attention_arithmetic_and_import_neither_side():
    text = open(os.path.join(ROOT, "pod_inputs", "gen.py")).read()
    assert not re.search(r"^\s*(from|import)\s+(oracle|paper_2412_02252_amd)", text, re.M)
    for word in ("softmax", "exp(", "exp2", "matmul", "einsum", "bmm("):
        assert word not in text, word


def test_only_tests_smoke_and_the_bench_baseline_use_the_oracle():
    allowed = {"bench.py", "__graft_entry__.py"}
    for f in _files("*.py", "pod_inputs/*.py", "paper_2412_02252_amd/**/*.py"):
        rel = os.path.relpath(f, ROOT)
        if rel in allowed:
            continue
        assert not re.search(r"^\s*(from|import)\s+oracle", open(f).read(), re.M), rel
    bench = open(os.path.join(ROOT, "bench.py")).read()
    # in the bench the oracle is imported inside the cpu_baseline leg only
    assert len(re.findall(r"^\s*from oracle import", bench, re.M)) == 1
    assert re.search(r"if not a\.no_cpu:\n\s+from oracle import pod_oracle", bench)
