"""The oracle under AddressSanitizer and UndefinedBehaviorSanitizer: oracle/pod_oracle.c is built with
-fsanitize=address,undefined (host code only, gcc) and the pin tests run against that build in a child process.
A read or write outside an array, a signed overflow or a misaligned access anywhere the pins reach aborts the
child.  CPU only."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "pod_oracle.c")


def _runtime(name):
    path = subprocess.run(["gcc", f"-print-file-name={name}"], capture_output=True, text=True, check=True).stdout.strip()
    return path if os.path.isabs(path) and os.path.exists(path) else None


def test_pins_pass_on_a_sanitized_build_of_the_oracle(tmp_path):
    asan = _runtime("libasan.so")
    assert asan, "gcc's AddressSanitizer runtime is part of this image"
    lib = str(tmp_path / "pod_oracle_san.so")
    subprocess.run(["gcc", "-O1", "-g", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-fno-omit-frame-pointer",
                    "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", SRC, "-o", lib, "-lm"], check=True)
    # the interpreter itself is not instrumented: the runtime is loaded in front of it, the interpreter's own
    # allocations at exit are not the oracle's business (no leak report), the oracle's handles are freed by the pins
    preload = ":".join(x for x in (asan, os.environ.get("LD_PRELOAD", "")) if x)
    env = dict(os.environ, POD_ORACLE_LIB=lib, LD_PRELOAD=preload, ASAN_OPTIONS="detect_leaks=0:abort_on_error=1",
               UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1", OMP_NUM_THREADS="4")
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_oracle_pins.py")], cwd=ROOT, env=env, capture_output=True, text=True)
    assert r.returncode == 0, (r.stdout[-1500:], r.stderr[-1500:])
    assert "passed" in r.stdout


def test_the_sanitized_build_does_catch_an_overrun(tmp_path):
    """The set-up above is live: a copy of the oracle whose attention loop reads one key past the sequence must
    abort under the same build and environment."""
    asan = _runtime("libasan.so")
    text = open(SRC).read()
    old = "for (long j = 0; j <= i; ++j) {"
    assert text.count(old) >= 1
    bad = text.replace(old, "for (long j = 0; j <= i + 1; ++j) {", 1)
    src = str(tmp_path / "overrun.c")
    open(src, "w").write(bad)
    lib = str(tmp_path / "overrun.so")
    subprocess.run(["gcc", "-O1", "-g", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-fsanitize=address,undefined",
                    "-fno-sanitize-recover=undefined", src, "-o", lib, "-lm"], check=True)
    preload = ":".join(x for x in (asan, os.environ.get("LD_PRELOAD", "")) if x)
    env = dict(os.environ, POD_ORACLE_LIB=lib, LD_PRELOAD=preload, ASAN_OPTIONS="detect_leaks=0:abort_on_error=1",
               OMP_NUM_THREADS="1")
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-s", "-p", "no:cacheprovider",   # -s: the report goes to the real stderr
                        os.path.join(ROOT, "tests", "test_oracle_pins.py")], cwd=ROOT, env=env, capture_output=True, text=True)
    assert r.returncode != 0 and "AddressSanitizer" in (r.stdout + r.stderr), (r.returncode, r.stderr[-800:])
