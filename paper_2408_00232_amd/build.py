"""Builds libcdf.so (HIP, gfx950 only) in-tree with hipcc."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libcdf.so")
SOURCES = ["cdf_cache.hip", "cdf_quant.hip", "cdf_spmm.hip", "cdf_gemm.hip", "cdf_layer.hip", "cdf_train.hip",
           "cdf_partition.hip", "cdf_gemm_bf16.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I" + os.path.join(ROOT, "include"), "-I" + CSRC, "-Wall", "-Wno-unused-function"]


def sources_sha() -> str:
    """Short hash of the library's sources (kernels, shared header, C header): profiles record it so
    that a counter summary can be told apart from one taken on other kernels."""
    import hashlib
    h = hashlib.sha256()
    files = sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith((".hip", ".h")))
    for path in files + [os.path.join(ROOT, "include", "cdf.h")]:
        h.update(os.path.basename(path).encode())
        h.update(open(path, "rb").read())
    return h.hexdigest()[:16]


LIB_SANITIZED = os.path.join(HERE, "libcdf_san.so")
SANITIZE_FLAGS = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                  "-Xarch_host", "-fno-sanitize-recover=undefined", "-g"]


def build_lib(verbose: bool = True, sanitize_host: bool = False) -> str:
    """Compile every source to an object (in parallel), then link the shared library.
    sanitize_host: a second library, libcdf_san.so, whose HOST code (argument checks, launch logic, the
    partitioner) is instrumented with AddressSanitizer and UndefinedBehaviorSanitizer; device code is
    unchanged. A process that loads it needs clang's ASan runtime preloaded (asan_runtime())."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    bdir = os.path.join(HERE, "_build", "san" if sanitize_host else "")
    lib_path = LIB_SANITIZED if sanitize_host else LIB
    flags = FLAGS + (SANITIZE_FLAGS if sanitize_host else [])
    os.makedirs(bdir, exist_ok=True)
    procs = []
    objs = []
    for s in SOURCES:
        obj = os.path.join(bdir, s.replace(".hip", ".o"))
        objs.append(obj)
        cmd = [hipcc, "-c", os.path.join(CSRC, s), "-o", obj] + flags
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((s, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    failed = False
    for s, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if out.strip() and verbose:
            print(out)
        if p.returncode != 0:
            failed = True
            print(f"hipcc failed on {s}", file=sys.stderr)
    if failed:
        raise RuntimeError("libcdf build failed")
    cmd = [hipcc, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", lib_path] + objs
    if sanitize_host:
        cmd += ["-fsanitize=address", "-fsanitize=undefined", "-shared-libsan", "-fno-gpu-sanitize"]
    subprocess.check_call(cmd)
    return lib_path


def asan_runtime() -> str:
    """Path of the ASan runtime of the compiler hipcc drives (to be preloaded by a process that loads
    libcdf_san.so)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    out = subprocess.check_output([hipcc, "-print-file-name=libclang_rt.asan-x86_64.so"], text=True).strip()
    return out


if __name__ == "__main__":
    print(build_lib())
