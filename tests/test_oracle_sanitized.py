"""Host sanitizer pass over the CPU oracle: the oracle's own pins run once more against a build of
oracle/salad_oracle.c with AddressSanitizer and UndefinedBehaviorSanitizer (no GPU code involved)."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_pins_under_address_and_ub_sanitizers():
    asan = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    assert os.path.isabs(asan) and os.path.exists(asan), "gcc's libasan.so not found"
    env = dict(os.environ)
    env["SALAD_ORACLE_SANITIZE"] = "1"
    env["LD_PRELOAD"] = asan + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")     # added in front, nothing removed
    # the interpreter itself is not instrumented: its allocations are not leaks of the oracle
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    env["OMP_NUM_THREADS"] = "4"
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_oracle_mask.py"), os.path.join(ROOT, "tests", "test_oracle_attention.py")],
                       capture_output=True, text=True, env=env, cwd=ROOT, timeout=1500)
    text = r.stdout + r.stderr
    assert "AddressSanitizer" not in text and "runtime error:" not in text, text[-4000:]
    assert r.returncode == 0, text[-4000:]
    assert " passed" in r.stdout
    lib = os.path.join(ROOT, "oracle", "libsalad_oracle_asan.so")
    assert os.path.exists(lib)
    # the sanitized library is what those tests loaded: it carries the ASan runtime's symbols
    nm = subprocess.run(["nm", "-D", lib], capture_output=True, text=True).stdout
    assert "__asan_init" in nm and "__ubsan_handle" in nm
