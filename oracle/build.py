"""Compile the C oracle with gcc.  Test infrastructure; building it is not using it.

`python -m oracle.build` rebuilds the library.  `python -m oracle.build --sanitize-check` builds the
oracle and libtoma's host code with AddressSanitizer and UndefinedBehaviorSanitizer (host code only:
there is no GPU sanitizer here) and runs the CPU test suite on those builds in a child process."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "toma_oracle.c")
LIB = os.path.join(HERE, "libtoma_oracle.so")
LIB_SAN = os.path.join(HERE, "libtoma_oracle_san.so")
# The sanitizer builds of the oracle and of libtoma's host side live in one process, so both use one
# runtime: the ROCm toolchain's clang and its shared AddressSanitizer library (which carries the
# UndefinedBehaviorSanitizer handlers too).
CLANG = "/opt/rocm/lib/llvm/bin/clang"
SAN_FLAGS = ["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
             "-shared-libsan"]


def sanitized():
    """True when this process was asked (TOMA_SANITIZE=1) to load the sanitizer builds."""
    return os.environ.get("TOMA_SANITIZE", "0") == "1"


def build(force=False, sanitize=None):
    sanitize = sanitized() if sanitize is None else sanitize
    lib = LIB_SAN if sanitize else LIB
    if not force and os.path.exists(lib) and os.path.getmtime(lib) >= os.path.getmtime(SRC):
        return lib
    if sanitize:
        omp_dir = os.path.dirname(subprocess.run([CLANG, "-print-file-name=libomp.so"], check=True, capture_output=True,
                                                 text=True).stdout.strip())
        cmd = [CLANG, *SAN_FLAGS, "-fopenmp", "-fPIC", "-shared", "-fvisibility=hidden", "-Wall", "-Wextra",
               "-o", lib, SRC, "-lm", "-Wl,-rpath," + omp_dir]
    else:
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-fvisibility=hidden", "-Wall", "-Wextra",
               "-o", lib, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return lib


def sanitize_check():
    """Sanitizer builds of the oracle and of libtoma's host side, then `pytest -m "not gpu"` on them."""
    root = os.path.dirname(HERE)
    sys.path.insert(0, root)
    from paper_2509_10918_amd import build as toma_build
    build(force=True, sanitize=True)
    toma_build.build(sanitize=True)
    asan = subprocess.run([CLANG, "-print-file-name=libclang_rt.asan-x86_64.so"], check=True, capture_output=True,
                          text=True).stdout.strip()
    env = dict(os.environ)
    env["TOMA_SANITIZE"] = "1"
    # the interpreter itself is not instrumented: the runtime has to be loaded first, and what CPython
    # leaves allocated at exit is not a leak of ours
    env["LD_PRELOAD"] = asan + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    return subprocess.run([sys.executable, "-m", "pytest", os.path.join(root, "tests"), "-x", "-q", "-m", "not gpu"],
                          env=env, cwd=root).returncode


if __name__ == "__main__":
    if "--sanitize-check" in sys.argv:
        sys.exit(sanitize_check())
    print(build(force=True, sanitize="--sanitize" in sys.argv))
