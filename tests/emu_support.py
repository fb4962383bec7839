"""Loader for the CPU-emulated build of the library (tests/emu) plus guard-paged
"device" buffers.  Test scaffolding only."""
import ctypes as C
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.join(HERE, "emu"))
import build_emu  # noqa: E402

from paper_1911_11377_amd import ckksmi  # noqa: E402


def emu_lib_path():
    return build_emu.build(force=False)


class EmuBuf:
    """uint64/int64 buffer ending right against a PROT_NONE page"""

    def __init__(self, lib, shape, dtype=np.uint64):
        self._lib = lib
        self.shape = tuple(shape)
        n = int(np.prod(self.shape)) if len(self.shape) else 1
        self.nbytes = max(n, 1) * 8
        lib.emu_alloc.restype = C.c_void_p
        lib.emu_alloc.argtypes = [C.c_size_t]
        lib.emu_free.argtypes = [C.c_void_p]
        self.addr = lib.emu_alloc(self.nbytes)
        assert self.addr
        arr_t = C.c_uint64 * max(n, 1)
        self.np = np.frombuffer(arr_t.from_address(self.addr), dtype=dtype)[:n].reshape(self.shape)

    def data_ptr(self):
        return self.addr

    def is_contiguous(self):
        return True

    def reshape(self, *shape):
        """only the flat view (what the call-sequence modules use to carve buffers)"""
        assert shape in ((-1,), ((-1,),))
        return EmuView(self, 0, self.nbytes // 8)

    def __getitem__(self, sl):
        return self.reshape(-1)[sl]

    def __del__(self):
        try:
            self._lib.emu_free(self.addr)
        except Exception:
            pass


class EmuView:
    """a contiguous range of words of an EmuBuf (keeps its parent alive)"""

    def __init__(self, parent, start, count):
        self.parent, self.start, self.count = parent, start, count
        self.nbytes = count * 8

    def data_ptr(self):
        return self.parent.addr + 8 * self.start

    def is_contiguous(self):
        return True

    def reshape(self, *shape):
        assert shape in ((-1,), ((-1,),))
        return self

    def __getitem__(self, sl):
        assert isinstance(sl, slice) and sl.step in (None, 1)
        a, b, _ = sl.indices(self.count)
        return EmuView(self.parent, self.start + a, max(b - a, 0))


def emu_context(*args, **kw):
    path = emu_lib_path()
    ctx = ckksmi.Context(*args, device=0, lib=path, **kw)
    return ctx, ckksmi.load(path)


def to_emu(lib, arr, dtype=np.uint64):
    arr = np.ascontiguousarray(arr, dtype=dtype)
    b = EmuBuf(lib, arr.shape, dtype)
    b.np[...] = arr
    return b
