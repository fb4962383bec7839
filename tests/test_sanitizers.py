"""The CPU-side code under AddressSanitizer and UndefinedBehaviorSanitizer: the C oracle, the library's host functions
(parameter search, encoding, key generation, encryption) and the library's kernel sources compiled for the CPU stand-in.
Each is built with -fsanitize=address,undefined -fno-sanitize-recover=all into a scratch directory and exercised by
sanitize_driver.py in a child process that preloads the sanitizer runtimes; a report makes the child fail."""
import os
import subprocess
import sys

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(ROOT, "paper_1911_11377_amd", "csrc")
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-O0"]  # -O0: the build is most of this test's time


def _runtime(name):
    path = subprocess.check_output(["gcc", "-print-file-name=" + name]).decode().strip()
    return path if os.path.isabs(path) and os.path.exists(path) else None


@pytest.mark.skipif(_runtime("libasan.so") is None or _runtime("libubsan.so") is None, reason="sanitizer runtimes not installed")
def test_oracle_and_host_code_under_address_and_ub_sanitizers(tmp_path):
    oracle_lib = str(tmp_path / "liboracle_san.so")
    subprocess.check_call(["gcc"] + SAN + ["-ffp-contract=off", "-Wall", "-shared", "-fPIC", "-o", oracle_lib,
                                           os.path.join(ROOT, "oracle", "ckks_oracle.c"), "-lm"])
    srcs = [os.path.join(CSRC, s) for s in ("ckksmi_device.hip", "host_math.cpp", "host_crypto.cpp")] + [os.path.join(HERE, "emu", "hip_emu.cpp")]
    emu_lib = str(tmp_path / "libckksmi_emu_san.so")
    subprocess.check_call(["g++"] + SAN + ["-std=c++17", "-fPIC", "-shared", "-mfma", "-ffp-contract=off", "-DCKKSMI_EMULATE", "-include",
                                           os.path.join(HERE, "emu", "hip_emu.h"), "-Wno-unknown-pragmas", "-x", "c++"] + srcs + ["-o", emu_lib])
    env = dict(os.environ)
    pre = [_runtime("libasan.so"), _runtime("libubsan.so")] + ([env["LD_PRELOAD"]] if env.get("LD_PRELOAD") else [])
    env["LD_PRELOAD"] = ":".join(pre)
    # Python itself leaks by design; the kernels' CPU stand-in switches stacks (fibres), which ASan must be told not to police
    env["ASAN_OPTIONS"] = "detect_leaks=0:halt_on_error=1:detect_stack_use_after_return=0"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    # the same sanitized build serves as the host library: a context with device = -1 never launches anything
    r = subprocess.run([sys.executable, os.path.join(HERE, "sanitize_driver.py"), oracle_lib, emu_lib, emu_lib], env=env,
                       stdout=subprocess.PIPE, stderr=subprocess.STDOUT, timeout=900)
    text = r.stdout.decode(errors="replace")
    assert r.returncode == 0 and "emulated kernel pass done" in text, text[-4000:]
    assert "runtime error" not in text and "AddressSanitizer" not in text, text[-4000:]
