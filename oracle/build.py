"""Compiles the CPU checker (plain C, host compiler) into oracle/liboracle.so.

TEST INFRASTRUCTURE ONLY: see densify_oracle.c.

`sanitize=True` makes a second library, liboracle_san.so, with the address and
undefined-behaviour sanitizers (clang, shared runtime); a process that loads it must have
that runtime preloaded (SANITIZER_RUNTIME below), which tests/test_sanitizers.py does.
"""
import glob
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "densify_oracle.c")
LIB = os.path.join(HERE, "liboracle.so")
LIB_SAN = os.path.join(HERE, "liboracle_san.so")
CLANG = os.environ.get("CLANG", "/opt/rocm/llvm/bin/clang")


def sanitizer_runtime() -> str:
    """Path of clang's shared AddressSanitizer runtime (it also carries UBSan's)."""
    out = subprocess.run([CLANG, "-print-resource-dir"], capture_output=True, text=True, check=True).stdout.strip()
    hits = glob.glob(os.path.join(out, "lib", "*", "libclang_rt.asan-x86_64.so"))
    if not hits:
        raise FileNotFoundError("no shared AddressSanitizer runtime under " + out)
    return hits[0]


def build(force: bool = True, sanitize: bool = False) -> str:
    lib = LIB_SAN if sanitize else LIB
    if not force and os.path.exists(lib) and os.path.getmtime(lib) >= os.path.getmtime(SRC):
        return lib
    if sanitize:
        cmd = [CLANG, "-O1", "-g", "-std=c11", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-shared-libsan",
               "-o", lib, SRC, "-lm"]
    else:
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-Wall", "-Wextra", "-o", lib, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return lib


if __name__ == "__main__":
    print(build(force=True, sanitize="--sanitize" in sys.argv))
    sys.exit(0)
