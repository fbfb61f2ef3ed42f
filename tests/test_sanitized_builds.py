"""Memory and undefined-behaviour checks of the host code (CPU only).

The oracle (plain C) and the host side of the library (argument checks, launch logic, the graph
partitioner) are built a second time with AddressSanitizer and UndefinedBehaviorSanitizer and the
CPU tests that exercise them are run again, in a child process that has the sanitizer runtime
preloaded. A planted one-past-the-end write shows that the set-up reports what it is there to find.
"""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run_child(cmd, runtime, extra_env, cwd=ROOT):
    env = dict(os.environ)
    env.update(extra_env)
    # the sanitizer runtime has to come first; whatever is preloaded already stays
    env["LD_PRELOAD"] = runtime + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0:exitcode=86"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:exitcode=87:print_stacktrace=1"
    return subprocess.run(cmd, cwd=cwd, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True,
                          timeout=900)


def gcc_asan_runtime():
    return subprocess.check_output(["gcc", "-print-file-name=libasan.so"], text=True).strip()


def test_planted_overflow_is_reported(tmp_path):
    src = tmp_path / "planted.c"
    src.write_text("#include <stdlib.h>\n"
                   "int planted(int n) { volatile char* p = malloc(n); p[n] = 1; int r = p[0]; free((void*)p); return r; }\n")
    lib = tmp_path / "libplanted.so"
    subprocess.check_call(["gcc", "-O1", "-g", "-fsanitize=address,undefined", "-shared", "-fPIC", "-o", str(lib), str(src)])
    r = run_child([sys.executable, "-c", f"import ctypes; ctypes.CDLL({str(lib)!r}).planted(16)"], gcc_asan_runtime(), {})
    assert r.returncode != 0 and "heap-buffer-overflow" in r.stdout, r.stdout[-2000:]


def test_oracle_pins_pass_under_asan_and_ubsan():
    r = run_child([sys.executable, "-m", "pytest", "tests/test_oracle_pins.py", "-x", "-q", "-p", "no:cacheprovider"],
                  gcc_asan_runtime(), {"CDF_ORACLE_SANITIZE": "1"})
    assert r.returncode == 0, r.stdout[-4000:]
    assert " passed" in r.stdout and "ERROR: AddressSanitizer" not in r.stdout and "runtime error" not in r.stdout
    assert os.path.exists(os.path.join(ROOT, "oracle", "libcdf_oracle_san.so"))


def test_library_host_code_passes_under_asan_and_ubsan():
    from paper_2408_00232_amd import build
    srcs = [os.path.join(build.CSRC, f) for f in os.listdir(build.CSRC)] + [os.path.join(ROOT, "include", "cdf.h")]
    if not os.path.exists(build.LIB_SANITIZED) or \
            os.path.getmtime(build.LIB_SANITIZED) < max(os.path.getmtime(s) for s in srcs):
        build.build_lib(verbose=False, sanitize_host=True)
    check = ("import paper_2408_00232_amd.binding as B, sys; "
             "assert B.LIB_PATH.endswith('libcdf_san.so'); B.load(); sys.exit(0)")
    r = run_child([sys.executable, "-c", check], build.asan_runtime(), {"CDF_LIB_SANITIZE": "1"})
    assert r.returncode == 0, r.stdout[-2000:]
    r = run_child([sys.executable, "-m", "pytest", "tests/test_partitioner.py", "tests/test_library_exports.py", "-x", "-q",
                   "-p", "no:cacheprovider"], build.asan_runtime(), {"CDF_LIB_SANITIZE": "1"})
    assert r.returncode == 0, r.stdout[-4000:]
    assert " passed" in r.stdout and "ERROR: AddressSanitizer" not in r.stdout and "runtime error" not in r.stdout
