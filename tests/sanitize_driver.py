"""Run in a child process with the sanitizer runtimes preloaded (see test_sanitizers.py): a small pass over the oracle,
the library's host functions and the library's kernel sources on the CPU stand-in, all three built with
-fsanitize=address,undefined.  Any report aborts the process (-fno-sanitize-recover, halt_on_error)."""
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(HERE))
sys.path.insert(0, HERE)
sys.path.insert(0, os.path.join(HERE, "emu"))

oracle_lib, host_lib, emu_lib = sys.argv[1:4]

from oracle import build as oracle_build  # noqa: E402

oracle_build.build = lambda force=False: oracle_lib  # the oracle module loads whatever its build step returns

import build_emu  # noqa: E402

build_emu.build = lambda force=False: emu_lib

import numpy as np  # noqa: E402

import parity_cases as pc  # noqa: E402
from paper_1911_11377_amd import ckksmi  # noqa: E402
from paper_1911_11377_amd import workloads as wl  # noqa: E402

# ---- oracle: definitions and the T1 pipeline at a tiny size
shape = (5, 5, 40, 2, 41, 2)
M = pc.make_material(shape, 11, rotations=(3,))
O = M.O
z = wl.slots_complex(O.N // 2, 11, "z")
ct = M.encrypt(z, 2.0 ** 30, 5, "z")
out = O.hmul_relin_rescale(ct, ct, M.rlk, 5)
O.rotate(ct, 3, M.gk[3], 5)
O.hmul_relin_rescale_merged(ct, ct, M.rlk, 5)
O.rotate_hoisted(ct, (3,), [M.gk[3]], 5)
dec = M.decrypt(out, 2.0 ** 60 / O.q[4], 4)
assert np.max(np.abs(dec - z * z)) < 1e-2
x = wl.uniform_limbs(O.q[:3], O.N, 11, "x", lead=(2, 4, 4, 2))
O.conv2d_mac(x, np.arange(-9, 9, dtype=np.int64).reshape(1, 2, 3, 3), 1, 1, 3)
O.sum_pool2d(x, 2, 3, 1)
print("oracle pass done", flush=True)

# ---- library, host side only (device = -1): parameter search, encode / decode, key generation, encrypt / decrypt
L = ckksmi.load(host_lib)
ctx = ckksmi.Context(*shape, device=-1, lib=host_lib)
assert ctx.moduli == O.moduli
pt = ctx.encode(z, 2.0 ** 30, 5)
back = ctx.decode(pt, 5, 2.0 ** 30)
assert np.max(np.abs(back - z)) < 1e-6
s = wl.ternary(O.N, 11, "s")
a = wl.uniform_limbs(O.q, O.N, 11, "pk.a")
e = wl.gaussian_error(O.N, 11, "pk.e")
pk = ctx.keygen_public(s, a, e)
assert np.array_equal(pk, O.keygen_public(s, a, e))
c2 = ctx.encrypt(pk, pt, wl.ternary(O.N, 11, "r"), wl.gaussian_error(O.N, 11, "e0"), wl.gaussian_error(O.N, 11, "e1"), 5)
ctx.decode(ctx.decrypt(s, c2, 5), 5, 2.0 ** 30)
ctx.close()
print("host library pass done", flush=True)

# ---- library kernels on the CPU stand-in (guard pages behind every buffer)
be = pc.EmuBackend()
pc.case_relin_and_composite(be, shape, seed=12, batch=2, levels=[5, 3])
pc.case_rotate(be, shape, seed=13, rotations=[1, 3], batch=2)
pc.case_rescale(be, (6, 3, 30, 1, 31, 1), seed=14)
pc.case_conv(be, (7, 2, 51, 0, 52, 1), seed=15, Cin=2, H=3, W=3, Oc=9, kh=3, stride=1, pad=1, rows_check=False)
with be.tuned(8):
    pc.case_relin_and_composite(be, (13, 2, 50, 1, 51, 1), seed=16, batch=2, levels=[2])
    pc.case_ntt(be, (13, 1, 50, 1, 51, 1), seed=17, batch=2)
    # rotations at a register-tiled size: the pair loads through the automorphism (plain and from a shared ModUp)
    pc.case_rotate(be, (12, 2, 50, 1, 51, 1), seed=18, rotations=[1, 700], batch=2)
    pc.case_rotate_hoisted(be, (12, 2, 50, 1, 51, 1), seed=19, rotations=(1, 700), batch=2)
pc.case_plain_mac(be, (6, 3, 30, 1, 31, 1), seed=20)
print("emulated kernel pass done", flush=True)
