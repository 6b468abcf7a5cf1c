"""The CPU code under AddressSanitizer + UndefinedBehaviorSanitizer (no GPU): the C oracle, and the
host logic of the library (block accounting, prefix index with its LRU and reference counts, argument
checks, workspace sizing) built for the host only.  Each runs the existing CPU tests of that code in a
child process that starts with the matching sanitizer runtime preloaded (gcc's for the oracle, the
HIP compiler's for the library: the two cannot share a process); a report from either sanitizer ends
the child with an error."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
T = os.path.join(ROOT, "tests")


def run_tests(files, env_extra):
    env = dict(os.environ)
    env.update(env_extra)
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1"       # (the interpreter itself never frees everything)
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *[os.path.join(T, f) for f in files]]
    r = subprocess.run(cmd, cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    tail = (r.stdout + r.stderr)[-4000:]
    assert r.returncode == 0, tail
    assert " passed" in r.stdout and "failed" not in r.stdout, tail
    return r.stdout


def test_oracle_under_asan_and_ubsan():
    libasan = subprocess.run(["gcc", "-print-file-name=libasan.so"], check=True, capture_output=True,
                             text=True).stdout.strip()
    assert os.path.isabs(libasan) and os.path.exists(libasan), libasan
    run_tests(["test_oracle_step.py", "test_oracle_stages.py", "test_oracle_q4.py", "test_oracle_sampling.py"],
              {"LD_PRELOAD": libasan, "ORACLE_SANITIZE": "1"})
    # the instrumented build is the one that ran
    import oracle.reference as R
    san = os.path.join(os.path.dirname(R.__file__), "_build", "san", "liboracle_f64.so")
    syms = subprocess.run(["nm", "-D", san], check=True, capture_output=True, text=True).stdout
    assert "__asan_init" in syms and "__ubsan_handle" in syms


def test_library_host_code_under_asan_and_ubsan():
    from paper_2601_19139_amd import build
    lib = build.build_host_sanitizer_library()
    syms = subprocess.run(["nm", "-D", lib], check=True, capture_output=True, text=True).stdout
    assert "__asan_init" in syms and "__ubsan_handle" in syms
    run_tests(["test_prefix_index.py", "test_abi_host.py"],
              {"LD_PRELOAD": build.asan_runtime(), "DECODEKIT_LIBRARY": lib})
