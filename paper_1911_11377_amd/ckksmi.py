"""Thin Python binding of the C ABI in include/ckksmi.h.

Argument marshalling only: every step of the hot path runs in the HIP library.
Host-side functions take and return numpy arrays.  Device-side functions take
device buffers -- torch tensors (int64/uint64, contiguous, on the context's GPU) or
raw integer addresses -- and enqueue on torch's current stream unless told otherwise.
PyTorch is used for device memory and streams and nothing else.

There is no CPU fallback: if the compiled library is missing, loading raises.
"""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
DEFAULT_LIB = os.path.join(_HERE, "libckksmi.so")

OK, EINVAL, ELEVEL, ENOKEY, EWORKSPACE, EDEVICE, EUNSUPPORTED = 0, -1, -2, -3, -4, -5, -6
OP_RELIN, OP_RESCALE, OP_HMUL_RELIN_RESCALE, OP_ROTATE, OP_CONV2D_MAC, OP_MUL_SCALAR_RESCALE = 1, 2, 3, 4, 5, 6

u64p = C.POINTER(C.c_uint64)
i64p = C.POINTER(C.c_int64)
f64p = C.POINTER(C.c_double)
intp = C.POINTER(C.c_int)
VP = C.c_void_p


class Params(C.Structure):
    _fields_ = [
        ("logN", C.c_int), ("n_q", C.c_int), ("q_bits", C.c_int), ("n_special", C.c_int),
        ("special_bits", C.c_int), ("alpha", C.c_int),
        ("moduli_override", u64p), ("psi_override", u64p), ("device", C.c_int),
    ]


class CkksmiError(RuntimeError):
    def __init__(self, code, what, detail=""):
        self.code = code
        super().__init__("%s failed: %s (%d)%s" % (what, detail, code, ""))


# name -> argtypes of every exported function (restype int unless listed below)
SIGNATURES = {
    "ckksmi_ctx_create": [C.POINTER(Params), C.POINTER(VP)],
    "ckksmi_ctx_destroy": [VP],
    "ckksmi_get_moduli": [VP, u64p, u64p],
    "ckksmi_strerror": [C.c_int],
    "ckksmi_last_device_error": [VP],
    "ckksmi_sample_ternary": [VP, C.c_uint64, i64p],
    "ckksmi_sample_error": [VP, C.c_uint64, i64p],
    "ckksmi_sample_uniform": [VP, C.c_uint64, intp, C.c_int, u64p],
    "ckksmi_encode": [VP, f64p, f64p, C.c_double, C.c_int, u64p],
    "ckksmi_decode": [VP, u64p, C.c_int, C.c_double, f64p, f64p],
    "ckksmi_keygen_public": [VP, i64p, u64p, i64p, u64p],
    "ckksmi_keygen_relin": [VP, i64p, u64p, i64p, u64p],
    "ckksmi_keygen_galois": [VP, i64p, C.c_int, u64p, i64p, u64p],
    "ckksmi_encrypt": [VP, u64p, u64p, i64p, i64p, i64p, C.c_int, u64p],
    "ckksmi_decrypt": [VP, i64p, u64p, C.c_int, C.c_int, u64p],
    "ckksmi_galois_key_register": [VP, C.c_int, VP],
    "ckksmi_ntt": [VP, VP, intp, C.c_int, C.c_int, VP],
    "ckksmi_intt": [VP, VP, intp, C.c_int, C.c_int, VP],
    "ckksmi_add": [VP, VP, VP, VP, C.c_int, C.c_int, VP],
    "ckksmi_sub": [VP, VP, VP, VP, C.c_int, C.c_int, VP],
    "ckksmi_mul_plain": [VP, VP, VP, C.c_size_t, VP, C.c_int, C.c_int, VP],
    "ckksmi_mul_scalar": [VP, VP, C.c_int64, VP, C.c_int, C.c_int, VP],
    "ckksmi_add_const": [VP, VP, C.c_int64, VP, C.c_int, C.c_int, VP],
    "ckksmi_mod_drop": [VP, VP, C.c_int, C.c_int, VP, C.c_int, VP],
    "ckksmi_hmul": [VP, VP, VP, VP, C.c_int, C.c_int, VP],
    "ckksmi_relin": [VP, VP, VP, VP, C.c_int, C.c_int, VP, C.c_size_t, VP],
    "ckksmi_rescale": [VP, VP, VP, C.c_int, C.c_int, VP, C.c_size_t, VP],
    "ckksmi_rescale_static": [VP, VP, VP, C.c_int, C.c_int, VP],
    "ckksmi_hmul_relin_rescale": [VP, VP, VP, VP, VP, C.c_int, C.c_int, VP, C.c_size_t, VP],
    "ckksmi_mul_scalar_rescale": [VP, VP, C.c_int64, VP, VP, C.c_int, C.c_int, C.c_int, VP, C.c_size_t, VP],
    "ckksmi_hmul_relin_rescale_merged": [VP, VP, VP, VP, VP, C.c_int, C.c_int, VP, C.c_size_t, VP],
    "ckksmi_hmul_sum_relin_rescale": [VP, VP, VP, C.c_int, VP, VP, C.c_int, C.c_int, VP, C.c_size_t, VP],
    "ckksmi_sample_device": [VP, C.c_int, C.c_double, C.c_uint64, C.c_uint64, C.c_int, VP, VP],
    "ckksmi_encode_device": [VP, VP, VP, C.c_double, C.c_int, C.c_int, VP, VP, C.c_size_t, VP],
    "ckksmi_encrypt_device": [VP, VP, VP, VP, VP, VP, C.c_int, C.c_int, VP, VP, C.c_size_t, VP],
    "ckksmi_rotate_hoisted": [VP, VP, intp, C.c_int, VP, C.c_int, C.c_int, VP, C.c_size_t, VP],
    "ckksmi_rotate_hoisted_workspace_bytes": [VP, C.c_int, C.c_int, C.c_int, C.POINTER(C.c_size_t)],
    "ckksmi_rotate": [VP, VP, intp, VP, C.c_int, C.c_int, VP, C.c_size_t, VP],
    "ckksmi_conv2d_mac": [VP, VP, VP] + [C.c_int] * 8 + [VP, C.c_int, VP, C.c_size_t, VP],
    "ckksmi_conv2d_workspace_bytes": [VP, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.POINTER(C.c_size_t)],
    "ckksmi_plain_mac": [VP, VP, C.c_int, VP, C.c_int, VP, C.c_int, VP, C.c_int, VP],
    "ckksmi_conv2d_mac_rows": [VP, VP, VP] + [C.c_int] * 12 + [VP, C.c_int, VP, C.c_size_t, VP],
    "ckksmi_fc_mac": [VP, VP, VP, C.c_int, C.c_int, VP, C.c_int, VP, C.c_size_t, VP],
    "ckksmi_sum_pool2d": [VP, VP, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, VP, C.c_int, VP],
    "ckksmi_workspace_bytes": [VP, C.c_int, C.c_int, C.c_int, C.POINTER(C.c_size_t)],
    "ckksmi_profile_enable": [VP, C.c_int],
    "ckksmi_profile_read": [VP, C.c_int, f64p, C.POINTER(C.c_longlong), f64p],
    "ckksmi_kernel_class_name": [VP, C.c_int],
    "ckksmi_tune": [VP, C.c_int, C.c_int],
}
_RESTYPES = {"ckksmi_ctx_destroy": None, "ckksmi_strerror": C.c_char_p, "ckksmi_kernel_class_name": C.c_char_p}
K_COUNT = 31

_LIBS = {}


def load(path=None):
    """Load the compiled library; raises if it has not been built."""
    path = os.path.abspath(path or DEFAULT_LIB)
    if path in _LIBS:
        return _LIBS[path]
    if not os.path.exists(path):
        raise RuntimeError("%s not found: build it first (python -c 'import __graft_entry__ as g; g.build()')" % path)
    L = C.CDLL(path)
    for name, args in SIGNATURES.items():
        f = getattr(L, name)
        f.argtypes = args
        f.restype = _RESTYPES.get(name, C.c_int)
    _LIBS[path] = L
    return L


def _ptr(x):
    """device address of a torch tensor / anything with data_ptr(), or a raw int"""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if hasattr(x, "data_ptr"):
        if hasattr(x, "is_contiguous") and not x.is_contiguous():
            raise ValueError("device buffer must be contiguous")
        return x.data_ptr()
    raise TypeError("expected a device buffer, got %r" % type(x))


def _nbytes(x):
    if hasattr(x, "numel"):
        return x.numel() * x.element_size()
    return x.nbytes


def _u64(a):
    return np.ascontiguousarray(a, dtype=np.uint64)


def _i64(a):
    return np.ascontiguousarray(a, dtype=np.int64)


class Context:
    def __init__(self, logN, n_q, q_bits, k, special_bits, alpha, device=0, moduli=None, psis=None, lib=None):
        self._L = load(lib)
        p = Params()
        p.logN, p.n_q, p.q_bits, p.n_special, p.special_bits, p.alpha, p.device = logN, n_q, q_bits, k, special_bits, alpha, device
        self._keep = []
        if moduli is not None:
            m = _u64(moduli)
            self._keep.append(m)
            p.moduli_override = m.ctypes.data_as(u64p)
            if psis is not None:
                s = _u64(psis)
                self._keep.append(s)
                p.psi_override = s.ctypes.data_as(u64p)
        h = VP()
        rc = self._L.ckksmi_ctx_create(C.byref(p), C.byref(h))
        self._h = None
        if rc != OK:
            raise CkksmiError(rc, "ckksmi_ctx_create", self._L.ckksmi_strerror(rc).decode())
        self._h = h
        self.logN, self.N, self.n_q, self.k, self.alpha, self.device = logN, 1 << logN, n_q, k, max(alpha, 1), device
        self.T = n_q + k
        self.beta_top = (n_q + self.alpha - 1) // self.alpha
        m = np.zeros(self.T, dtype=np.uint64)
        s = np.zeros(self.T, dtype=np.uint64)
        self._call("ckksmi_get_moduli", self._h, m.ctypes.data_as(u64p), s.ctypes.data_as(u64p))
        self.moduli = [int(x) for x in m]
        self.psis = [int(x) for x in s]
        self.q, self.p = self.moduli[:n_q], self.moduli[n_q:]

    def close(self):
        if getattr(self, "_h", None) is not None:
            self._L.ckksmi_ctx_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _call(self, name, *args):
        rc = getattr(self._L, name)(*args)
        if rc != OK:
            detail = self._L.ckksmi_strerror(rc).decode()
            if rc == EDEVICE and self._h is not None:
                detail += ", hip error %d" % self._L.ckksmi_last_device_error(self._h)
            raise CkksmiError(rc, name, detail)
        return rc

    @staticmethod
    def _stream(stream):
        if stream is not None:
            return stream
        import torch

        return torch.cuda.current_stream().cuda_stream

    # ------------------------------------------------------------ host side
    def sample_ternary(self, seed):
        out = np.empty(self.N, dtype=np.int64)
        self._call("ckksmi_sample_ternary", self._h, seed, out.ctypes.data_as(i64p))
        return out

    def sample_error(self, seed):
        out = np.empty(self.N, dtype=np.int64)
        self._call("ckksmi_sample_error", self._h, seed, out.ctypes.data_as(i64p))
        return out

    def sample_uniform(self, seed, index):
        idx = np.ascontiguousarray(index, dtype=np.int32)
        out = np.empty((len(idx), self.N), dtype=np.uint64)
        self._call("ckksmi_sample_uniform", self._h, seed, idx.ctypes.data_as(intp), len(idx), out.ctypes.data_as(u64p))
        return out

    def encode(self, z, scale, level):
        z = np.asarray(z, dtype=np.complex128)
        assert z.shape == (self.N // 2,)
        re = np.ascontiguousarray(z.real)
        im = np.ascontiguousarray(z.imag)
        pt = np.empty((level, self.N), dtype=np.uint64)
        self._call("ckksmi_encode", self._h, re.ctypes.data_as(f64p), im.ctypes.data_as(f64p), float(scale), level, pt.ctypes.data_as(u64p))
        return pt

    def decode(self, pt, level, scale):
        pt = _u64(pt)
        assert pt.shape == (level, self.N)
        re = np.empty(self.N // 2)
        im = np.empty(self.N // 2)
        self._call("ckksmi_decode", self._h, pt.ctypes.data_as(u64p), level, float(scale), re.ctypes.data_as(f64p), im.ctypes.data_as(f64p))
        return re + 1j * im

    def keygen_public(self, s, a, e):
        s, a, e = _i64(s), _u64(a), _i64(e)
        assert a.shape == (self.n_q, self.N)
        pk = np.empty((2, self.n_q, self.N), dtype=np.uint64)
        self._call("ckksmi_keygen_public", self._h, s.ctypes.data_as(i64p), a.ctypes.data_as(u64p), e.ctypes.data_as(i64p), pk.ctypes.data_as(u64p))
        return pk

    def keygen_relin(self, s, a, e):
        s, a, e = _i64(s), _u64(a), _i64(e)
        assert a.shape == (self.beta_top, self.T, self.N) and e.shape == (self.beta_top, self.N)
        evk = np.empty((self.beta_top, 2, self.T, self.N), dtype=np.uint64)
        self._call("ckksmi_keygen_relin", self._h, s.ctypes.data_as(i64p), a.ctypes.data_as(u64p), e.ctypes.data_as(i64p), evk.ctypes.data_as(u64p))
        return evk

    def keygen_galois(self, s, rot, a, e):
        s, a, e = _i64(s), _u64(a), _i64(e)
        assert a.shape == (self.beta_top, self.T, self.N) and e.shape == (self.beta_top, self.N)
        gk = np.empty((self.beta_top, 2, self.T, self.N), dtype=np.uint64)
        self._call("ckksmi_keygen_galois", self._h, s.ctypes.data_as(i64p), int(rot), a.ctypes.data_as(u64p), e.ctypes.data_as(i64p), gk.ctypes.data_as(u64p))
        return gk

    def encrypt(self, pk, pt, r, e0, e1, level):
        pk, pt, r, e0, e1 = _u64(pk), _u64(pt), _i64(r), _i64(e0), _i64(e1)
        assert pk.shape == (2, self.n_q, self.N) and pt.shape == (level, self.N)
        ct = np.empty((2, level, self.N), dtype=np.uint64)
        self._call("ckksmi_encrypt", self._h, pk.ctypes.data_as(u64p), pt.ctypes.data_as(u64p), r.ctypes.data_as(i64p), e0.ctypes.data_as(i64p),
                   e1.ctypes.data_as(i64p), level, ct.ctypes.data_as(u64p))
        return ct

    def decrypt(self, s, ct, level):
        s, ct = _i64(s), _u64(ct)
        n_comp = ct.shape[0]
        assert ct.shape == (n_comp, level, self.N)
        pt = np.empty((level, self.N), dtype=np.uint64)
        self._call("ckksmi_decrypt", self._h, s.ctypes.data_as(i64p), ct.ctypes.data_as(u64p), level, n_comp, pt.ctypes.data_as(u64p))
        return pt

    # ------------------------------------------------------------ device side
    def workspace_bytes(self, op, level, batch):
        n = C.c_size_t(0)
        self._call("ckksmi_workspace_bytes", self._h, op, level, batch, C.byref(n))
        return n.value

    def conv2d_workspace_bytes(self, Cin, O, kh, kw, level):
        n = C.c_size_t(0)
        self._call("ckksmi_conv2d_workspace_bytes", self._h, Cin, O, kh, kw, level, C.byref(n))
        return n.value

    def galois_key_register(self, rot, gk_dev):
        self._keep.append(gk_dev)
        self._call("ckksmi_galois_key_register", self._h, int(rot), _ptr(gk_dev))

    def ntt(self, limbs, index, batch, stream=None):
        idx = np.ascontiguousarray(index, dtype=np.int32)
        self._call("ckksmi_ntt", self._h, _ptr(limbs), idx.ctypes.data_as(intp), len(idx), batch, self._stream(stream))

    def intt(self, limbs, index, batch, stream=None):
        idx = np.ascontiguousarray(index, dtype=np.int32)
        self._call("ckksmi_intt", self._h, _ptr(limbs), idx.ctypes.data_as(intp), len(idx), batch, self._stream(stream))

    def add(self, a, b, out, level, batch, stream=None):
        self._call("ckksmi_add", self._h, _ptr(a), _ptr(b), _ptr(out), level, batch, self._stream(stream))

    def sub(self, a, b, out, level, batch, stream=None):
        self._call("ckksmi_sub", self._h, _ptr(a), _ptr(b), _ptr(out), level, batch, self._stream(stream))

    def mul_plain(self, a, pt, pt_stride, out, level, batch, stream=None):
        self._call("ckksmi_mul_plain", self._h, _ptr(a), _ptr(pt), pt_stride, _ptr(out), level, batch, self._stream(stream))

    def mul_scalar(self, a, c, out, level, batch, stream=None):
        self._call("ckksmi_mul_scalar", self._h, _ptr(a), int(c), _ptr(out), level, batch, self._stream(stream))

    def add_const(self, a, c, out, level, batch, stream=None):
        self._call("ckksmi_add_const", self._h, _ptr(a), int(c), _ptr(out), level, batch, self._stream(stream))

    def mod_drop(self, a, level_in, level_out, out, batch, stream=None):
        self._call("ckksmi_mod_drop", self._h, _ptr(a), level_in, level_out, _ptr(out), batch, self._stream(stream))

    def hmul(self, a, b, d, level, batch, stream=None):
        self._call("ckksmi_hmul", self._h, _ptr(a), _ptr(b), _ptr(d), level, batch, self._stream(stream))

    def relin(self, d, evk, out, level, batch, ws, stream=None):
        self._call("ckksmi_relin", self._h, _ptr(d), _ptr(evk), _ptr(out), level, batch, _ptr(ws), _nbytes(ws), self._stream(stream))

    def rescale(self, a, out, level, batch, ws, stream=None):
        self._call("ckksmi_rescale", self._h, _ptr(a), _ptr(out), level, batch, _ptr(ws), _nbytes(ws), self._stream(stream))

    def rescale_static(self, a, out, level, batch, stream=None):
        """ckksmi_rescale over the library's static scratch array: no workspace argument, allocates nothing"""
        self._call("ckksmi_rescale_static", self._h, _ptr(a), _ptr(out), level, batch, self._stream(stream))

    def mul_scalar_rescale(self, a, c, out, level, batch, ws, stream=None, level_in=None, addend=None):
        """out = Rescale(c * a) at `level` (+ addend, which may be out); level_in > level: a is stored with level_in limbs and
        dropped to `level` on the way"""
        self._call("ckksmi_mul_scalar_rescale", self._h, _ptr(a), int(c), _ptr(addend) if addend is not None else None, _ptr(out),
                   level_in or level, level, batch, _ptr(ws), _nbytes(ws), self._stream(stream))

    def hmul_relin_rescale(self, a, b, evk, out, level, batch, ws, stream=None):
        self._call("ckksmi_hmul_relin_rescale", self._h, _ptr(a), _ptr(b), _ptr(evk), _ptr(out), level, batch, _ptr(ws), _nbytes(ws),
                   self._stream(stream))

    def sample_device(self, kind, sigma, seed, first_index, rows, out, stream=None):
        """rows small polynomials (kind 0 ternary, 1 rounded Gaussian) into the device int64 buffer out [rows][N]"""
        self._call("ckksmi_sample_device", self._h, kind, float(sigma), seed, first_index, rows, _ptr(out), self._stream(stream))

    def encode_device(self, re, im, scale, level, batch, pt, ws, stream=None):
        """re, im: device float64 [batch][N/2] (im may be None); pt: device [batch][level][N]; ws: batch*N*16 bytes"""
        self._call("ckksmi_encode_device", self._h, _ptr(re), _ptr(im) if im is not None else None, float(scale), level, batch, _ptr(pt), _ptr(ws),
                   _nbytes(ws), self._stream(stream))

    def encrypt_device(self, pk, pt, r, e0, e1, level, batch, ct, ws, stream=None):
        """pk [2][n_q][N], pt [batch][level][N], r/e0/e1 int64 [batch][N] (all device); ct [batch][2][level][N]"""
        self._call("ckksmi_encrypt_device", self._h, _ptr(pk), _ptr(pt), _ptr(r), _ptr(e0), _ptr(e1), level, batch, _ptr(ct), _ptr(ws), _nbytes(ws),
                   self._stream(stream))

    def rotate_hoisted_workspace_bytes(self, level, batch, n_rot):
        n = C.c_size_t(0)
        self._call("ckksmi_rotate_hoisted_workspace_bytes", self._h, level, batch, n_rot, C.byref(n))
        return n.value

    def rotate_hoisted(self, a, rots, out, level, batch, ws, stream=None):
        """every item rotated by every offset in rots with one shared ModUp; out [batch][len(rots)][2][level][N]"""
        r = np.ascontiguousarray(rots, dtype=np.int32)
        self._call("ckksmi_rotate_hoisted", self._h, _ptr(a), r.ctypes.data_as(intp), len(r), _ptr(out), level, batch, _ptr(ws), _nbytes(ws),
                   self._stream(stream))

    def hmul_sum_relin_rescale(self, a, b, terms, evk, out, level, batch, ws, stream=None):
        """a, b: [batch][terms][2][level][N]; the sum of each item's products, relinearised and rescaled once"""
        self._call("ckksmi_hmul_sum_relin_rescale", self._h, _ptr(a), _ptr(b), terms, _ptr(evk), _ptr(out), level, batch, _ptr(ws), _nbytes(ws),
                   self._stream(stream))

    def hmul_relin_rescale_merged(self, a, b, evk, out, level, batch, ws, stream=None):
        self._call("ckksmi_hmul_relin_rescale_merged", self._h, _ptr(a), _ptr(b), _ptr(evk), _ptr(out), level, batch, _ptr(ws), _nbytes(ws),
                   self._stream(stream))

    def rotate(self, a, rot, out, level, batch, ws, stream=None):
        r = np.ascontiguousarray(rot, dtype=np.int32)
        assert r.shape == (batch,)
        self._call("ckksmi_rotate", self._h, _ptr(a), r.ctypes.data_as(intp), _ptr(out), level, batch, _ptr(ws), _nbytes(ws), self._stream(stream))

    def plain_mac(self, cts, n_ct, pts, n_pts, term, n_groups, out, level, stream=None):
        """out[g] = sum over s of pts[term[g][s]] * cts[s] where term[g][s] >= 0; term: device int32 [n_groups][n_ct]"""
        self._call("ckksmi_plain_mac", self._h, _ptr(cts), n_ct, _ptr(pts), n_pts, _ptr(term), n_groups, _ptr(out), level, self._stream(stream))

    def conv2d_mac(self, x, w, Cin, H, W, O, kh, kw, stride, pad, out, level, ws, stream=None):
        self._call("ckksmi_conv2d_mac", self._h, _ptr(x), _ptr(w), Cin, H, W, O, kh, kw, stride, pad, _ptr(out), level, _ptr(ws), _nbytes(ws),
                   self._stream(stream))

    def conv2d_mac_rows(self, x, w, Cin, H, W, O, kh, kw, stride, pad, in_row0, in_rows, out_row0, out_rows, out, level, ws, stream=None):
        self._call("ckksmi_conv2d_mac_rows", self._h, _ptr(x), _ptr(w), Cin, H, W, O, kh, kw, stride, pad, in_row0, in_rows, out_row0, out_rows,
                   _ptr(out), level, _ptr(ws), _nbytes(ws), self._stream(stream))

    def sum_pool2d(self, x, Cin, H, W, k, out, level, stream=None, pad=0):
        self._call("ckksmi_sum_pool2d", self._h, _ptr(x), Cin, H, W, k, pad, _ptr(out), level, self._stream(stream))

    def fc_mac(self, x, w, F, O, out, level, ws, stream=None):
        self._call("ckksmi_fc_mac", self._h, _ptr(x), _ptr(w), F, O, _ptr(out), level, _ptr(ws), _nbytes(ws), self._stream(stream))

    # ------------------------------------------------------------ measurement
    def tune_target_wgs(self, value):
        """workgroups a transform launch aims for before its workgroups loop over items (ckksmi_tune)"""
        self._call("ckksmi_tune", self._h, 0, int(value))

    def profile_enable(self, on=True):
        self._call("ckksmi_profile_enable", self._h, 1 if on else 0)

    def profile_read(self):
        """{kernel class name: (total ms, launches, units of work)} for classes that ran"""
        out = {}
        for kid in range(K_COUNT):
            ms, n, u = C.c_double(0), C.c_longlong(0), C.c_double(0)
            self._call("ckksmi_profile_read", self._h, kid, C.byref(ms), C.byref(n), C.byref(u))
            if n.value:
                name = self._L.ckksmi_kernel_class_name(self._h, kid).decode()
                if name in out:  # two classes that run the same kernel symbol (e.g. k = 1): one line, like a profiler shows it
                    ms0, n0, u0 = out[name]
                    out[name] = (ms0 + ms.value, n0 + n.value, u0 + u.value)
                else:
                    out[name] = (ms.value, n.value, u.value)
        return out
