"""Compiles csrc/*.hip for gfx950 into libts_densify.so next to this file."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRCS = [os.path.join(HERE, "csrc", f) for f in ("ts_densify.hip", "ts_accumulate.hip")]
LIB = os.path.join(HERE, "libts_densify.so")
LIB_SAN = os.path.join(HERE, "libts_densify_san.so")     # host code under ASan + UBSan (checks of the host logic)
INCLUDE = os.path.join(ROOT, "include")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # keep the compiler from forming packed-fp32 instructions out of float4 arithmetic
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wextra", "-I", INCLUDE,
]


SAN_FLAGS = ["-g", "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
             "-Xarch_host", "-fno-sanitize-recover=undefined", "-shared-libsan"]


def build(force: bool = True, verbose: bool = False, sanitize: bool = False) -> str:
    """sanitize=True: a second library whose HOST code runs under the address and
    undefined-behaviour sanitizers (device code unchanged); the loading process must have
    clang's shared sanitizer runtime preloaded."""
    lib = LIB_SAN if sanitize else LIB
    if not force and os.path.exists(lib):
        return lib
    cmd = [HIPCC] + FLAGS + (SAN_FLAGS if sanitize else []) + ["-o", lib] + SRCS
    if verbose:
        print(" ".join(cmd))
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if err.strip() and verbose:
        print(err)
    return lib


if __name__ == "__main__":
    print(build(force=True, verbose=True, sanitize="--sanitize" in sys.argv))
    sys.exit(0)
