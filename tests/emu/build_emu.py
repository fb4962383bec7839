"""Compile the library's sources against the CPU stand-in of tests/emu/hip_emu.h
(libckksmi_emu.so).  Test scaffolding: lets the kernel sources run through their
indexing on tiny shapes with guard pages, on the CPU, before any GPU launch."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
CSRC = os.path.join(ROOT, "paper_1911_11377_amd", "csrc")
LIB = os.path.join(HERE, "libckksmi_emu.so")


def build(force=False):
    srcs = [os.path.join(CSRC, s) for s in ("ckksmi_device.hip", "host_math.cpp", "host_crypto.cpp")] + [os.path.join(HERE, "hip_emu.cpp")]
    deps = srcs + [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")] + [os.path.join(HERE, "hip_emu.h")]
    if not force and os.path.exists(LIB) and all(os.path.getmtime(LIB) >= os.path.getmtime(d) for d in deps):
        return LIB
    tmp = LIB + ".tmp.%d" % os.getpid()
    cmd = ["g++", "-O1", "-g", "-std=c++17", "-fPIC", "-shared", "-mfma", "-ffp-contract=off", "-DCKKSMI_EMULATE",
           "-include", os.path.join(HERE, "hip_emu.h"), "-Wall", "-Wno-unused-function", "-Wno-unknown-pragmas", "-Wno-maybe-uninitialized", "-x", "c++"] + srcs + ["-o", tmp]
    subprocess.check_call(cmd)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
