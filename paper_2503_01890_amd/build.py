"""Builds libautohete.so (HIP, gfx950 only) in-tree with hipcc."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libautohete.so")
SOURCES = ["autohete_api.hip", "autohete_kernels.hip", "autohete_strategy.cpp", "autohete_host.cpp"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-pthread", "-Wall", "-Wextra",
         # hipcc -O3 must not form packed-fp32 instructions on the test machines
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def build(force=True, extra_flags=()):
    srcs = [os.path.join(CSRC, s) for s in SOURCES]
    deps = srcs + [os.path.join(CSRC, "autohete_internal.h"),
                   os.path.join(HERE, "..", "include", "autohete.h")]
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= max(os.path.getmtime(d) for d in deps):
        return LIB
    subprocess.check_call([HIPCC] + FLAGS + list(extra_flags) + ["-o", LIB] + srcs)
    return LIB


if __name__ == "__main__":
    print(build())
