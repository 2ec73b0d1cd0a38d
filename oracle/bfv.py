"""ctypes wrapper over the C oracle (test infrastructure; see src/bfv_oracle.c)."""
import ctypes as C
import os

import numpy as np

from . import build as _build

_U64P = C.POINTER(C.c_uint64)
_U32P = C.POINTER(C.c_uint32)
_lib = None


def load_library():
    global _lib
    if _lib is not None:
        return _lib
    path = _build.build()
    lib = C.CDLL(path)
    lib.orc_min_psi.restype = C.c_uint64
    lib.orc_min_psi.argtypes = [C.c_int, C.c_uint64]
    for name in ("orc_eval_odd", "orc_interp_odd"):
        f = getattr(lib, name)
        f.restype = None
        f.argtypes = [_U64P, _U64P, C.c_int, C.c_uint64, C.c_uint64]
    lib.orc_polymul.restype = None
    lib.orc_polymul.argtypes = [_U64P, _U64P, _U64P, C.c_int, C.c_uint64]
    for name in ("orc_ntt_forward", "orc_ntt_inverse"):
        f = getattr(lib, name)
        f.restype = None
        f.argtypes = [_U64P, _U64P, C.c_int, C.c_uint64]
    lib.orc_create.restype = C.c_void_p
    lib.orc_create.argtypes = [C.c_int, C.c_int, _U64P, C.c_int, _U64P,
                               C.c_uint64, C.c_int]
    lib.orc_destroy.restype = None
    lib.orc_destroy.argtypes = [C.c_void_p]
    lib.orc_num_threads.restype = C.c_int
    lib.orc_set_threads.argtypes = [C.c_int]
    lib.orc_add.argtypes = [C.c_void_p, _U64P, _U64P, _U64P, C.c_int]
    lib.orc_mul.argtypes = [C.c_void_p, _U64P, _U64P, _U64P]
    lib.orc_mul_sum.argtypes = [C.c_void_p, _U64P, _U64P, C.c_int, _U64P]
    lib.orc_mul_sum.restype = C.c_int
    lib.orc_keyswitch.argtypes = [C.c_void_p, _U64P, _U64P, _U64P]
    lib.orc_relin.argtypes = [C.c_void_p, _U64P, _U64P, _U64P]
    lib.orc_galois_poly.argtypes = [C.c_void_p, _U64P, C.c_uint64, _U64P]
    lib.orc_rotate.argtypes = [C.c_void_p, _U64P, C.c_uint64, _U64P, _U64P]
    lib.orc_rotate_hoisted.argtypes = [C.c_void_p, _U64P, C.c_uint64, _U64P, _U64P]
    lib.orc_rotate_sum_hoisted.argtypes = [C.c_void_p, _U64P, C.c_int, _U64P, C.POINTER(_U64P), _U64P]
    lib.orc_mul_plain.argtypes = [C.c_void_p, _U64P, _U64P, _U64P]
    lib.orc_add_plain.argtypes = [C.c_void_p, _U64P, _U64P, C.c_int, _U64P]
    lib.orc_test_crt.restype = C.c_int
    lib.orc_test_crt.argtypes = [_U64P, C.c_int, _U64P, _U32P, C.c_int]
    lib.orc_test_divmod.restype = C.c_int
    lib.orc_test_divmod.argtypes = [_U32P, C.c_int, _U32P, C.c_int, _U32P,
                                    C.POINTER(C.c_int), _U32P, C.POINTER(C.c_int)]
    lib.orc_test_is_prime.restype = C.c_int
    lib.orc_test_is_prime.argtypes = [C.c_uint64]
    lib.orc_private_basis.restype = C.c_int
    lib.orc_private_basis.argtypes = [C.c_void_p, _U64P, C.c_int]
    _lib = lib
    return lib


def _p(a: np.ndarray):
    assert a.dtype == np.uint64 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(_U64P)


def _u64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.uint64)


# ---- context-free helpers (single word-size prime) -------------------------
def min_psi(n: int, m: int) -> int:
    return int(load_library().orc_min_psi(n, m))


def polymul(a, b, m: int) -> np.ndarray:
    """Negacyclic product in Z_m[X]/(X^n+1)."""
    a, b = _u64(a), _u64(b)
    out = np.empty_like(a)
    load_library().orc_polymul(_p(a), _p(b), _p(out), a.shape[-1], m)
    return out


def eval_odd(a, m: int, psi: int) -> np.ndarray:
    """out[i] = a(psi^(2i+1))."""
    a = _u64(a)
    out = np.empty_like(a)
    load_library().orc_eval_odd(_p(a), _p(out), a.shape[-1], m, psi)
    return out


def interp_odd(ev, m: int, psi: int) -> np.ndarray:
    ev = _u64(ev)
    out = np.empty_like(ev)
    load_library().orc_interp_odd(_p(ev), _p(out), ev.shape[-1], m, psi)
    return out


def ntt_forward(a, m: int) -> np.ndarray:
    """out[i] = a(psi^(2*bitrev(i)+1)), psi the smallest primitive 2n-th root mod m."""
    a = _u64(a)
    out = np.empty_like(a)
    load_library().orc_ntt_forward(_p(a), _p(out), a.shape[-1], m)
    return out


def ntt_inverse(v, m: int) -> np.ndarray:
    v = _u64(v)
    out = np.empty_like(v)
    load_library().orc_ntt_inverse(_p(v), _p(out), v.shape[-1], m)
    return out


def is_prime(n: int) -> bool:
    return bool(load_library().orc_test_is_prime(n))


def crt_words(moduli, residues) -> int:
    m, r = _u64(moduli), _u64(residues)
    words = np.zeros(80, dtype=np.uint32)
    n = load_library().orc_test_crt(_p(m), len(m), _p(r),
                                    words.ctypes.data_as(_U32P), 80)
    assert n >= 0
    return sum(int(words[i]) << (32 * i) for i in range(n))


def _to_words(x: int) -> np.ndarray:
    w = []
    while x:
        w.append(x & 0xFFFFFFFF)
        x >>= 32
    return np.array(w or [0], dtype=np.uint32)


def big_divmod(a: int, b: int):
    """(a // b, a % b) computed by the oracle's long division."""
    aw, bw = _to_words(a), _to_words(b)
    q = np.zeros(80, dtype=np.uint32)
    r = np.zeros(80, dtype=np.uint32)
    qn, rn = C.c_int(0), C.c_int(0)
    rc = load_library().orc_test_divmod(
        aw.ctypes.data_as(_U32P), len(aw) if a else 0,
        bw.ctypes.data_as(_U32P), len(bw),
        q.ctypes.data_as(_U32P), C.byref(qn), r.ctypes.data_as(_U32P), C.byref(rn))
    assert rc == 0
    return (sum(int(q[i]) << (32 * i) for i in range(qn.value)),
            sum(int(r[i]) << (32 * i) for i in range(rn.value)))


class Oracle:
    """Evaluator operations on numpy uint64 arrays (layout as in the C file)."""

    def __init__(self, params):
        self.params = params
        self.lib = load_library()
        self.n, self.k, self.nsp = params.n, params.k, params.nsp
        self.q = [int(x) for x in params.q]
        self.p = [int(x) for x in params.p]
        self.qp = self.q + self.p
        self.t = int(params.t)
        q = _u64(self.q)
        p = _u64(self.p)
        self.ctx = self.lib.orc_create(params.log2n, self.k, _p(q), self.nsp,
                                       _p(p), self.t, params.alpha)
        if not self.ctx:
            raise ValueError("oracle rejected the parameter set")

    def __del__(self):
        if getattr(self, "ctx", None):
            self.lib.orc_destroy(self.ctx)
            self.ctx = None

    @property
    def threads(self) -> int:
        return int(self.lib.orc_num_threads())

    def set_threads(self, n: int):
        self.lib.orc_set_threads(int(n))

    def private_basis(self):
        m = np.zeros(32, dtype=np.uint64)
        n = self.lib.orc_private_basis(self.ctx, _p(m), 32)
        return [int(x) for x in m[:n]]

    def _ct(self, a, ncomp):
        a = _u64(a)
        assert a.shape == (ncomp, self.k, self.n), a.shape
        return a

    def add(self, a, b):
        a = _u64(a)
        ncomp = a.shape[0]
        a, b = self._ct(a, ncomp), self._ct(b, ncomp)
        out = np.empty_like(a)
        self.lib.orc_add(self.ctx, _p(a), _p(b), _p(out), ncomp)
        return out

    def mul(self, a2, b2):
        a2, b2 = self._ct(a2, 2), self._ct(b2, 2)
        out = np.empty((3, self.k, self.n), dtype=np.uint64)
        self.lib.orc_mul(self.ctx, _p(a2), _p(b2), _p(out))
        return out

    def mul_sum(self, a2s, b2s):
        """round(t/Q * sum_u a_u (x) b_u): the tensor products of the pairs summed over the integers
        before the one scaling (three components)."""
        a = np.ascontiguousarray(np.stack([self._ct(x, 2) for x in a2s]))
        b = np.ascontiguousarray(np.stack([self._ct(x, 2) for x in b2s]))
        assert len(a) == len(b) >= 1
        out = np.empty((3, self.k, self.n), dtype=np.uint64)
        if self.lib.orc_mul_sum(self.ctx, _p(a), _p(b), len(a), _p(out)):
            raise ValueError("too many products for the oracle's private basis")
        return out

    def _key(self, ksk):
        ksk = _u64(ksk)
        assert ksk.shape == (self.params.dnum, 2, self.k + self.nsp, self.n)
        return ksk

    def keyswitch(self, d, ksk):
        d = _u64(d)
        assert d.shape == (self.k, self.n)
        ksk = self._key(ksk)
        out = np.empty((2, self.k, self.n), dtype=np.uint64)
        self.lib.orc_keyswitch(self.ctx, _p(d), _p(ksk), _p(out))
        return out

    def relin(self, in3, rlk):
        in3, rlk = self._ct(in3, 3), self._key(rlk)
        out = np.empty((2, self.k, self.n), dtype=np.uint64)
        self.lib.orc_relin(self.ctx, _p(in3), _p(rlk), _p(out))
        return out

    def galois_poly(self, poly, g: int):
        poly = _u64(poly)
        assert poly.shape == (self.k, self.n)
        out = np.empty_like(poly)
        self.lib.orc_galois_poly(self.ctx, _p(poly), g, _p(out))
        return out

    def rotate(self, in2, g: int, gk):
        assert g % 2 == 1 and 0 < g < 2 * self.n
        in2, gk = self._ct(in2, 2), self._key(gk)
        out = np.empty_like(in2)
        self.lib.orc_rotate(self.ctx, _p(in2), g, _p(gk), _p(out))
        return out

    def rotate_hoisted(self, in2, g: int, gk):
        """Rotation with the digits taken from c1 before the Galois map (the form in which one
        decomposition serves a whole series of rotations of the same ciphertext)."""
        assert g % 2 == 1 and 0 < g < 2 * self.n
        in2, gk = self._ct(in2, 2), self._key(gk)
        out = np.empty_like(in2)
        self.lib.orc_rotate_hoisted(self.ctx, _p(in2), g, _p(gk), _p(out))
        return out

    def rotate_many(self, in2, gs, gks):
        """[rotate_hoisted(in2, g, gks[g]) for g in gs]: a series of rotations of one ciphertext."""
        return [self.rotate_hoisted(in2, g, gks[g]) for g in gs]

    def rotate_sum_hoisted(self, in2, gs, gks):
        """in2 + the sum of its hoisted rotations by every g of gs (keys gks[g]), the key-switch
        accumulators of the series summed before the one division by P."""
        in2 = self._ct(in2, 2)
        # gks: keys by Galois element, or a list with one key per position of gs
        keys = [self._key(k) for k in gks] if isinstance(gks, (list, tuple)) else [self._key(gks[g]) for g in gs]
        assert len(keys) == len(gs) and all(g % 2 == 1 and 0 < g < 2 * self.n for g in gs)
        garr = np.asarray(list(gs), dtype=np.uint64)
        kptr = (_U64P * max(1, len(keys)))(*[_p(k) for k in keys])
        out = np.empty_like(in2)
        self.lib.orc_rotate_sum_hoisted(self.ctx, _p(in2), len(keys), _p(garr), kptr, _p(out))
        return out

    def add_plain(self, in2, pt, negative=False):
        """(c0 +- floor(Q/t) pt, c1): Algorithm 1 step 1, the server's masking and unmasking."""
        in2 = self._ct(in2, 2)
        pt = _u64(pt)
        assert pt.shape == (self.n,)
        out = np.empty_like(in2)
        self.lib.orc_add_plain(self.ctx, _p(in2), _p(pt), 1 if negative else 0, _p(out))
        return out

    def mul_plain(self, in2, pt):
        in2 = self._ct(in2, 2)
        pt = _u64(pt)
        assert pt.shape == (self.n,)
        out = np.empty_like(in2)
        self.lib.orc_mul_plain(self.ctx, _p(in2), _p(pt), _p(out))
        return out
