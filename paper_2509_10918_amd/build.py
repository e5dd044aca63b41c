"""Compile libtoma (HIP, gfx950 only) in-tree with hipcc."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libtoma.so")
SOURCES = ["toma_api.hip", "toma_select.hip", "toma_gram_i8.hip", "toma_merge.hip", "toma_attend.hip", "toma_pinv.hip", "toma_fused.hip", "toma_profile.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall", "-Wno-unused-parameter", "-Wno-inline-asm"]


LIB_SAN = os.path.join(HERE, "libtoma_san.so")
# host code only (there is no GPU sanitizer here): each option directly after -Xarch_host
SAN_FLAGS = ["-g", "-fno-omit-frame-pointer", "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined"]


def build(verbose=False, extra=(), sanitize=False):
    """sanitize: AddressSanitizer + UndefinedBehaviorSanitizer on the host side, into libtoma_san.so
    (loaded instead of libtoma.so by a process started with TOMA_SANITIZE=1; CPU checks only)."""
    objs = []
    procs = []
    if sanitize:
        extra = (*extra, *SAN_FLAGS)
    for src in SOURCES:
        obj = os.path.join(CSRC, src.replace(".hip", ".san.o" if sanitize else ".o"))
        cmd = ["hipcc", *FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    failed = False
    for src, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines()
                        if "packed-fp32-ops" not in l and "unknown target feature" not in l.lower())
        if p.returncode != 0:
            failed = True
            print(out)
        elif verbose and out.strip():
            print(out)
    if failed:
        raise RuntimeError("hipcc failed")
    lib = LIB_SAN if sanitize else LIB
    link = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-shared-libsan"] if sanitize else []
    subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", *link, "-o", lib, *objs], check=True)
    return lib


if __name__ == "__main__":
    import sys
    print(build(verbose="-v" in sys.argv, sanitize="--sanitize" in sys.argv))
