"""ctypes binding of include/cryptogen.h -- argument marshalling only.

Ciphertexts, keys and plaintexts are torch.int64 CUDA tensors whose bit
patterns are the uint64 residues; every method passes data_ptr() values and
the current torch stream to the entry point of the same name.
"""
import ctypes as C
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.environ.get("CRYPTOGEN_HIP_LIB", os.path.join(_HERE, "libcryptogen_hip.so"))

_SYMBOLS = [
    "cg_create", "cg_destroy", "cg_get_sizes", "cg_workspace_bytes", "cg_strerror",
    "cg_ntt_forward", "cg_ntt_inverse", "cg_ksk_prepare", "cg_plain_prepare",
    "cg_mul", "cg_relin", "cg_mul_relin", "cg_rotate", "cg_add", "cg_mul_plain", "cg_add_plain",
    "cg_kv_append", "cg_decode_scores", "cg_decode_context", "cg_decode_scores_outer", "cg_decode_context_outer", "cg_prefill_qk",
    "cg_decode_step", "cg_decode_step_workspace_bytes", "cg_prefill_av", "cg_prefill_repack",
    "cg_cpvm", "cg_cache_extend", "cg_decode_scores_ext", "cg_decode_context_ext", "cg_decode_step_ext",
    "cg_bench_modmul", "cg_bench_exchange", "cg_profile_begin", "cg_profile_end", "cg_kernel_name",
    "cg_mul_relin_static", "cg_static_scratch_bytes",
    "cg_rotate_hoisted", "cg_prefill_qk_hoisted", "cg_prefill_av_hoisted", "cg_cpvm_hoisted",
    "cg_rotate_sum_hoisted", "cg_round_galois", "cg_decode_scores_hoisted", "cg_decode_context_hoisted",
    "cg_decode_step_hoisted", "cg_mul_sum",
]


class _Params(C.Structure):
    _fields_ = [("log2n", C.c_uint32), ("k", C.c_uint32), ("nsp", C.c_uint32),
                ("alpha", C.c_uint32), ("t", C.c_uint64),
                ("q", C.POINTER(C.c_uint64)), ("p", C.POINTER(C.c_uint64))]


class _Sizes(C.Structure):
    _fields_ = [("ct2_bytes", C.c_size_t), ("ct3_bytes", C.c_size_t),
                ("ksk_raw_bytes", C.c_size_t), ("ksk_bytes", C.c_size_t),
                ("plain_bytes", C.c_size_t), ("ws_bytes_per_unit", C.c_size_t), ("ct_ext_bytes", C.c_size_t)]


class _KernelStat(C.Structure):
    _fields_ = [("kernel_id", C.c_uint32), ("launches", C.c_uint32),
                ("total_ms", C.c_double), ("algo_bytes", C.c_double), ("work_items", C.c_double)]


class Library:
    """The loaded shared library with typed entry points."""

    def __init__(self, path: str = _LIB_PATH):
        if not os.path.exists(path):
            raise RuntimeError(
                f"{path} is missing: build it with `python -m paper_2602_08798_amd.build` "
                "(there is no CPU fallback)")
        self.path = path
        self.dll = C.CDLL(path)
        vp, u32, i32 = C.c_void_p, C.c_uint32, C.c_int
        d = self.dll
        d.cg_create.argtypes = [C.POINTER(vp), C.POINTER(_Params)]
        d.cg_destroy.argtypes = [vp]
        d.cg_get_sizes.argtypes = [vp, C.POINTER(_Sizes)]
        d.cg_workspace_bytes.argtypes = [vp, u32]
        d.cg_workspace_bytes.restype = C.c_size_t
        d.cg_strerror.argtypes = [i32]
        d.cg_strerror.restype = C.c_char_p
        d.cg_ntt_forward.argtypes = [vp, vp, vp, vp, C.POINTER(u32), u32]
        d.cg_ntt_inverse.argtypes = [vp, vp, vp, vp, C.POINTER(u32), u32]
        d.cg_ksk_prepare.argtypes = [vp, vp, vp, vp]
        d.cg_plain_prepare.argtypes = [vp, vp, vp, vp, u32]
        d.cg_mul.argtypes = [vp, vp, vp, vp, vp, u32, u32, vp]
        d.cg_relin.argtypes = [vp, vp, vp, vp, vp, u32, vp]
        d.cg_mul_relin.argtypes = [vp, vp, vp, vp, vp, vp, u32, u32, vp]
        d.cg_rotate_hoisted.argtypes = [vp, vp, vp, u32, C.POINTER(u32), C.POINTER(vp), vp, u32, vp]
        d.cg_rotate_sum_hoisted.argtypes = d.cg_rotate_hoisted.argtypes
        d.cg_round_galois.argtypes = [vp, i32, u32, u32, C.POINTER(u32), u32, C.POINTER(u32)]
        d.cg_decode_scores_hoisted.argtypes = [vp, vp, vp, vp, vp, u32, u32, u32, u32, u32, vp, C.POINTER(vp), vp, vp]
        d.cg_decode_context_hoisted.argtypes = [vp, vp, vp, vp, vp, u32, u32, u32, u32, u32, i32, vp, C.POINTER(vp),
                                                vp, vp]
        d.cg_decode_step_hoisted.argtypes = [vp, vp, vp, vp, vp, vp, u32, u32, u32, u32, u32, vp, vp, vp, u32,
                                             C.POINTER(vp), u32, i32, C.POINTER(vp), vp, vp, vp]
        d.cg_mul_sum.argtypes = [vp, vp, vp, vp, vp, u32, u32, vp]
        d.cg_prefill_qk_hoisted.argtypes = [vp, vp, vp, vp, u32, u32, u32, vp, C.POINTER(vp), C.POINTER(vp), vp, vp]
        d.cg_prefill_av_hoisted.argtypes = [vp, vp, vp, vp, u32, u32, i32, vp, C.POINTER(vp), vp, vp]
        d.cg_cpvm_hoisted.argtypes = [vp, vp, vp, vp, u32, u32, u32, u32, C.POINTER(vp), C.POINTER(vp), vp, vp]
        d.cg_mul_relin_static.argtypes = [vp, vp, vp, vp, vp, vp, u32, u32]
        d.cg_static_scratch_bytes.argtypes = []
        d.cg_static_scratch_bytes.restype = C.c_size_t
        d.cg_rotate.argtypes = [vp, vp, vp, u32, vp, vp, u32, i32, vp]
        d.cg_add.argtypes = [vp, vp, vp, vp, vp, u32, u32]
        d.cg_add_plain.argtypes = [vp, vp, vp, vp, u32, i32, vp, u32]
        d.cg_mul_plain.argtypes = [vp, vp, vp, vp, u32, vp, u32, vp]
        d.cg_kv_append.argtypes = [vp, vp, vp, u32, u32, u32, vp, vp, u32, vp]
        d.cg_decode_scores.argtypes = [vp, vp, vp, vp, u32, u32, u32, u32, vp, C.POINTER(vp), vp, vp]
        d.cg_decode_context.argtypes = [vp, vp, vp, vp, u32, u32, u32, u32, vp, C.POINTER(vp), vp, vp]
        d.cg_decode_scores_outer.argtypes = [vp, vp, vp, vp, u32, u32, vp, vp, C.POINTER(vp), vp, vp]
        d.cg_decode_context_outer.argtypes = [vp, vp, vp, vp, u32, u32, vp, C.POINTER(vp), vp, vp]
        d.cg_prefill_qk.argtypes = [vp, vp, vp, vp, u32, u32, vp, C.POINTER(vp), vp, vp, vp, vp]
        d.cg_cache_extend.argtypes = [vp, vp, vp, u32, u32, u32, vp]
        d.cg_decode_scores_ext.argtypes = d.cg_decode_scores.argtypes
        d.cg_decode_context_ext.argtypes = d.cg_decode_context.argtypes
        d.cg_decode_step_ext.argtypes = [vp, vp, vp, vp, vp, vp, u32, u32, u32, u32, u32, vp, vp, vp, C.POINTER(vp),
                                         C.POINTER(vp), vp, vp, vp]
        d.cg_prefill_av.argtypes = [vp, vp, vp, vp, u32, u32, vp, vp, vp, vp, vp]
        d.cg_prefill_repack.argtypes = [vp, vp, vp, u32, u32, vp, C.POINTER(vp), vp, vp]
        d.cg_cpvm.argtypes = [vp, vp, vp, vp, u32, u32, u32, C.POINTER(vp), C.POINTER(vp), vp, vp]
        d.cg_decode_step.argtypes = [vp, vp, vp, vp, vp, u32, u32, u32, u32, u32, vp, vp, vp, C.POINTER(vp),
                                     C.POINTER(vp), vp, vp, vp]
        d.cg_decode_step_workspace_bytes.argtypes = [vp, u32, u32]
        d.cg_decode_step_workspace_bytes.restype = C.c_size_t
        d.cg_bench_modmul.argtypes = [vp, vp, i32, u32, u32, vp]
        d.cg_bench_exchange.argtypes = [vp, vp, i32, u32, u32, vp]
        d.cg_profile_begin.argtypes = [vp, u32]
        d.cg_profile_end.argtypes = [vp, C.POINTER(_KernelStat), u32, C.POINTER(u32)]
        d.cg_kernel_name.argtypes = [u32]
        d.cg_kernel_name.restype = C.c_char_p
        for name in _SYMBOLS:
            if name not in ("cg_workspace_bytes", "cg_decode_step_workspace_bytes", "cg_strerror", "cg_kernel_name",
                            "cg_static_scratch_bytes"):
                getattr(d, name).restype = i32

    def strerror(self, status: int) -> str:
        return self.dll.cg_strerror(status).decode()


_lib = None


def load_library() -> Library:
    global _lib
    if _lib is None:
        _lib = Library()
    return _lib


def exported_symbols():
    return list(_SYMBOLS)


def to_device(arr: np.ndarray, device="cuda") -> torch.Tensor:
    """numpy uint64 array -> int64 device tensor with the same bits."""
    a = np.ascontiguousarray(arr, dtype=np.uint64)
    return torch.from_numpy(a.view(np.int64)).to(device)


def to_host(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().contiguous().numpy().view(np.uint64)


class CgError(RuntimeError):
    pass


class CgSizeError(CgError, ValueError):
    """A tensor handed to the binding is smaller than the call's arguments imply."""


def _need(t, numel: int, what: str):
    """Buffers cross the C ABI as bare pointers: catch undersized tensors here, on the host."""
    if t.numel() < numel:
        raise CgSizeError(f"{what}: {t.numel()} elements, at least {numel} needed")


def _ptr(t) -> int:
    if t is None:
        return 0
    assert t.is_cuda and t.is_contiguous() and t.dtype in (torch.int64, torch.float64, torch.uint8)
    return t.data_ptr()


class Context:
    """One cg_ctx plus a reusable workspace tensor."""

    def __init__(self, params, device="cuda"):
        self.lib = load_library()
        self.params = params
        self.device = torch.device(device)
        self.n, self.k, self.nsp = params.n, params.k, params.nsp
        self.dnum = params.k // params.alpha
        self.L = self.k + self.nsp
        q = (C.c_uint64 * self.k)(*[int(x) for x in params.q])
        p = (C.c_uint64 * self.nsp)(*[int(x) for x in params.p])
        prm = _Params(params.log2n, self.k, self.nsp, params.alpha, int(params.t), q, p)
        h = C.c_void_p()
        with torch.cuda.device(self.device):
            self._check(self.lib.dll.cg_create(C.byref(h), C.byref(prm)))
        self.h = h
        self._rounds = {}
        s = _Sizes()
        self._check(self.lib.dll.cg_get_sizes(self.h, C.byref(s)))
        self.sizes = s
        self._ws = None
        self._ws_step = None

    def close(self):
        if getattr(self, "h", None):
            self.lib.dll.cg_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, status: int):
        if status != 0:
            raise CgError(f"cryptogen: {self.lib.strerror(status)} ({status})")

    @property
    def stream(self) -> int:
        return torch.cuda.current_stream(self.device).cuda_stream

    def workspace_bytes(self, batch: int) -> int:
        return int(self.lib.dll.cg_workspace_bytes(self.h, batch))

    def workspace(self, batch: int) -> torch.Tensor:
        need = self.workspace_bytes(batch)
        if self._ws is None or self._ws.numel() < need:
            self._ws = None
            self._ws = torch.empty(need, dtype=torch.uint8, device=self.device)
        return self._ws

    def empty_ct(self, *lead, ncomp=2) -> torch.Tensor:
        return torch.empty(*lead, ncomp, self.k, self.n, dtype=torch.int64, device=self.device)

    # element counts implied by the arguments, checked before a pointer crosses the C ABI
    def _cts(self, count, ncomp=2) -> int:
        return max(0, int(count)) * ncomp * self.k * self.n

    def _need_key(self, key, what="key"):
        _need(key, int(self.sizes.ksk_bytes) // 8, what + " (prepared)")

    # ---- entry points (same names as the C ABI, without the cg_ prefix) ----
    def ntt_forward(self, x, prime_idx, out=None, inverse=False):
        out = torch.empty_like(x) if out is None else out
        _need(x, len(prime_idx) * self.n, "x")
        _need(out, len(prime_idx) * self.n, "out")
        idx = (C.c_uint32 * len(prime_idx))(*prime_idx)
        f = self.lib.dll.cg_ntt_inverse if inverse else self.lib.dll.cg_ntt_forward
        self._check(f(self.h, self.stream, _ptr(x), _ptr(out), idx, len(prime_idx)))
        return out

    def ntt_inverse(self, x, prime_idx, out=None):
        return self.ntt_forward(x, prime_idx, out, inverse=True)

    def ksk_prepare(self, raw):
        assert raw.shape == (self.dnum, 2, self.L, self.n)
        out = torch.empty(self.sizes.ksk_bytes // 8, dtype=torch.float64, device=self.device)
        self._check(self.lib.dll.cg_ksk_prepare(self.h, self.stream, _ptr(raw), _ptr(out)))
        return out

    def plain_prepare(self, pt):
        batch = pt.numel() // self.n
        out = torch.empty(batch * self.sizes.plain_bytes // 8, dtype=torch.float64, device=self.device)
        self._check(self.lib.dll.cg_plain_prepare(self.h, self.stream, _ptr(pt), _ptr(out), batch))
        return out

    def mul(self, a2, b2, batch, a_group=1, out=None):
        out = self.empty_ct(batch, ncomp=3) if out is None else out
        self._need_mul(a2, b2, batch, a_group)
        _need(out, self._cts(batch, 3), "out")
        ws = self.workspace(batch)
        self._check(self.lib.dll.cg_mul(self.h, self.stream, _ptr(a2), _ptr(b2), _ptr(out), batch,
                                        a_group, _ptr(ws)))
        return out

    def mul_sum(self, a2, b2, n_groups, group_len, out=None):
        """out[g] = one scaling of the sum of the group's tensor products (three components)."""
        batch = max(0, int(n_groups)) * max(0, int(group_len))
        out = self.empty_ct(n_groups, ncomp=3) if out is None else out
        _need(a2, self._cts(batch), "a")
        _need(b2, self._cts(batch), "b")
        _need(out, self._cts(n_groups, 3), "out")
        ws = self.workspace(batch)
        self._check(self.lib.dll.cg_mul_sum(self.h, self.stream, _ptr(a2), _ptr(b2), _ptr(out), n_groups, group_len,
                                            _ptr(ws)))
        return out

    def _need_mul(self, a2, b2, batch, a_group):
        _need(a2, self._cts(-(-int(batch) // max(1, int(a_group)))), "a")
        _need(b2, self._cts(batch), "b")

    def relin(self, in3, rlk, batch, out=None):
        out = self.empty_ct(batch) if out is None else out
        _need(in3, self._cts(batch, 3), "in")
        _need(out, self._cts(batch), "out")
        self._need_key(rlk, "rlk")
        ws = self.workspace(batch)
        self._check(self.lib.dll.cg_relin(self.h, self.stream, _ptr(in3), _ptr(rlk), _ptr(out), batch,
                                          _ptr(ws)))
        return out

    def mul_relin(self, a2, b2, rlk, batch, a_group=1, out=None):
        out = self.empty_ct(batch) if out is None else out
        self._need_mul(a2, b2, batch, a_group)
        _need(out, self._cts(batch), "out")
        self._need_key(rlk, "rlk")
        ws = self.workspace(batch)
        self._check(self.lib.dll.cg_mul_relin(self.h, self.stream, _ptr(a2), _ptr(b2), _ptr(rlk),
                                              _ptr(out), batch, a_group, _ptr(ws)))
        return out

    def mul_relin_static(self, a2, b2, rlk, batch, a_group=1, out=None):
        """cg_mul_relin_static: the scratch is the library's own static array; `out` should be given
        by callers that must not allocate."""
        out = self.empty_ct(batch) if out is None else out
        self._need_mul(a2, b2, batch, a_group)
        _need(out, self._cts(batch), "out")
        self._need_key(rlk, "rlk")
        self._check(self.lib.dll.cg_mul_relin_static(self.h, self.stream, _ptr(a2), _ptr(b2), _ptr(rlk),
                                                     _ptr(out), batch, a_group))
        return out

    def rotate(self, in2, galois_elt, gk, batch, accumulate=False, out=None):
        out = self.empty_ct(batch) if out is None else out
        _need(in2, self._cts(batch), "in")
        _need(out, self._cts(batch), "out")
        self._need_key(gk, "gk")
        ws = self.workspace(batch)
        self._check(self.lib.dll.cg_rotate(self.h, self.stream, _ptr(in2), galois_elt, _ptr(gk),
                                           _ptr(out), batch, int(accumulate), _ptr(ws)))
        return out

    def rotate_hoisted(self, in2, galois_elts, gks, batch, out=None):
        """A series of rotations of each of `batch` ciphertexts: out[b][i] = rotation i of in2[b]."""
        n_rot = len(galois_elts)
        out = self.empty_ct(batch, n_rot) if out is None else out
        _need(in2, self._cts(batch), "in")
        _need(out, self._cts(batch * n_rot), "out")
        for i, key in enumerate(gks):
            self._need_key(key, f"Galois key {i}")
        if len(gks) != n_rot:
            raise CgSizeError(f"{n_rot} Galois elements but {len(gks)} keys")
        ws = self.workspace(batch * min(n_rot, 128) + batch)
        gs = (C.c_uint32 * max(1, n_rot))(*[int(g) for g in galois_elts])
        self._check(self.lib.dll.cg_rotate_hoisted(self.h, self.stream, _ptr(in2), n_rot, gs, self._keys(gks),
                                                   _ptr(out), batch, _ptr(ws)))
        return out

    def rotate_sum_hoisted(self, in2, galois_elts, gks, batch, out=None):
        """out[b] = in2[b] + the sum of its rotations by the given Galois elements (hoisted, one mod-down)."""
        n_rot = len(galois_elts)
        out = self.empty_ct(batch) if out is None else out
        _need(in2, self._cts(batch), "in")
        _need(out, self._cts(batch), "out")
        for i, key in enumerate(gks):
            self._need_key(key, f"Galois key {i}")
        if len(gks) != n_rot:
            raise CgSizeError(f"{n_rot} Galois elements but {len(gks)} keys")
        ws = self.workspace(batch)
        gs = (C.c_uint32 * max(1, n_rot))(*[int(g) for g in galois_elts])
        self._check(self.lib.dll.cg_rotate_sum_hoisted(self.h, self.stream, _ptr(in2), n_rot, gs, self._keys(gks),
                                                       _ptr(out), batch, _ptr(ws)))
        return out

    def add(self, a, b, ncomp, batch, out=None):
        out = torch.empty_like(a) if out is None else out
        for t, what in ((a, "a"), (b, "b"), (out, "out")):
            _need(t, self._cts(batch, max(0, int(ncomp))), what)
        self._check(self.lib.dll.cg_add(self.h, self.stream, _ptr(a), _ptr(b), _ptr(out), ncomp, batch))
        return out

    def add_plain(self, in2, pt, batch, negative=False, out=None):
        """pt: uint64 tensor [n_plain][N] of plaintext polynomials (coefficients in [0, t))."""
        out = torch.empty_like(in2) if out is None else out
        _need(in2, self._cts(batch), "in")
        _need(out, self._cts(batch), "out")
        _need(pt, pt.shape[0] * self.n, "pt")
        self._check(self.lib.dll.cg_add_plain(self.h, self.stream, _ptr(in2), _ptr(pt), pt.shape[0],
                                              1 if negative else 0, _ptr(out), batch))
        return out

    def mul_plain(self, in2, plain, batch, plain_stride=0, out=None):
        out = self.empty_ct(batch) if out is None else out
        _need(in2, self._cts(batch), "in")
        _need(out, self._cts(batch), "out")
        _need(plain, ((int(batch) - 1) * int(plain_stride) + 1) * self.k * self.n if batch > 0 else 0, "plain (prepared)")
        ws = self.workspace(batch)
        self._check(self.lib.dll.cg_mul_plain(self.h, self.stream, _ptr(in2), _ptr(plain), plain_stride,
                                              _ptr(out), batch, _ptr(ws)))
        return out

    def _check_append(self, cache, cache_stride_cts, n_caches, tau, rows, masks, d2):
        ct = 2 * self.k * self.n
        blocks = max(1, self.n // max(1, d2))
        _need(cache, n_caches * cache_stride_cts * ct, "cache")
        _need(rows, n_caches * ct, "rows")
        _need(masks, (tau % blocks + 1) * self.k * self.n, "masks (prepared, indexed by block)")

    def kv_append(self, cache, cache_stride_cts, n_caches, tau, rows, masks, d2):
        self._check_append(cache, cache_stride_cts, n_caches, tau, rows, masks, d2)
        ws = self.workspace(n_caches)
        self._check(self.lib.dll.cg_kv_append(self.h, self.stream, _ptr(cache), cache_stride_cts, n_caches,
                                              tau, _ptr(rows), _ptr(masks), d2, _ptr(ws)))
        return cache

    def _keys(self, keys):
        return (C.c_void_p * len(keys))(*[_ptr(k) for k in keys])

    def _need_products(self, left, n_left, cache, per_ct, heads, n_cts, stride, out, n_out, rlk, keys):
        """Operands of the decode products: `left` ciphertexts against `heads` cache groups of n_cts
        ciphertexts (per_ct elements each) spaced `stride` apart."""
        heads, n_cts, stride = max(0, int(heads)), max(0, int(n_cts)), max(0, int(stride))
        _need(left, self._cts(n_left), "left operand")
        _need(cache, ((heads - 1) * stride + n_cts) * per_ct if heads and n_cts else 0, "cache")
        _need(out, self._cts(n_out), "out")
        self._need_key(rlk, "rlk")
        for i, key in enumerate(keys):
            self._need_key(key, f"Galois key {i}")

    def decode_scores(self, q, kcache, heads, n_cts, d2, rlk, gk_fold, out=None, cache_stride_cts=None):
        out = self.empty_ct(heads, n_cts) if out is None else out
        ws = self.workspace(heads * n_cts)
        stride = n_cts if cache_stride_cts is None else cache_stride_cts
        self._need_products(q, heads, kcache, self._cts(1), heads, n_cts, stride, out, heads * n_cts, rlk, gk_fold)
        self._check(self.lib.dll.cg_decode_scores(self.h, self.stream, _ptr(q), _ptr(kcache), heads, n_cts,
                                                  stride, d2, _ptr(rlk), self._keys(gk_fold), _ptr(out), _ptr(ws)))
        return out

    def decode_context(self, a, vcache, heads, n_cts, d2, rlk, gk_block, out=None, cache_stride_cts=None):
        out = self.empty_ct(heads) if out is None else out
        ws = self.workspace(heads * n_cts)
        stride = n_cts if cache_stride_cts is None else cache_stride_cts
        self._need_products(a, heads * n_cts, vcache, self._cts(1), heads, n_cts, stride, out, heads, rlk, gk_block)
        self._check(self.lib.dll.cg_decode_context(self.h, self.stream, _ptr(a), _ptr(vcache), heads, n_cts,
                                                   stride, d2, _ptr(rlk), self._keys(gk_block), _ptr(out), _ptr(ws)))
        return out

    def empty_ext(self, n_cts) -> torch.Tensor:
        """Room for n_cts ciphertexts in transformed form (cache_extend output)."""
        return torch.empty(n_cts, int(self.sizes.ct_ext_bytes) // 8, dtype=torch.float64, device=self.device)

    def cache_extend(self, cts, n_groups, group_len, group_stride_cts, ext):
        span = (max(0, int(n_groups)) - 1) * int(group_stride_cts) + int(group_len) if n_groups > 0 else 0
        _need(cts, self._cts(span), "cts")
        _need(ext, span * (int(self.sizes.ct_ext_bytes) // 8), "ext")
        self._check(self.lib.dll.cg_cache_extend(self.h, self.stream, _ptr(cts), n_groups, group_len,
                                                 group_stride_cts, _ptr(ext)))
        return ext

    def decode_scores_ext(self, q, kext, heads, n_cts, d2, rlk, gk_fold, out=None, cache_stride_cts=None):
        out = self.empty_ct(heads, n_cts) if out is None else out
        ws = self.workspace(heads * n_cts)
        stride = n_cts if cache_stride_cts is None else cache_stride_cts
        self._need_products(q, heads, kext, int(self.sizes.ct_ext_bytes) // 8, heads, n_cts, stride, out,
                            heads * n_cts, rlk, gk_fold)
        self._check(self.lib.dll.cg_decode_scores_ext(self.h, self.stream, _ptr(q), _ptr(kext), heads, n_cts, stride,
                                                      d2, _ptr(rlk), self._keys(gk_fold), _ptr(out), _ptr(ws)))
        return out

    def decode_context_ext(self, a, vext, heads, n_cts, d2, rlk, gk_block, out=None, cache_stride_cts=None):
        out = self.empty_ct(heads) if out is None else out
        ws = self.workspace(heads * n_cts)
        stride = n_cts if cache_stride_cts is None else cache_stride_cts
        self._need_products(a, heads * n_cts, vext, int(self.sizes.ct_ext_bytes) // 8, heads, n_cts, stride, out,
                            heads, rlk, gk_block)
        self._check(self.lib.dll.cg_decode_context_ext(self.h, self.stream, _ptr(a), _ptr(vext), heads, n_cts, stride,
                                                       d2, _ptr(rlk), self._keys(gk_block), _ptr(out), _ptr(ws)))
        return out

    def decode_step(self, q, a, cache, heads, n_cts, cache_stride_cts, d2, tau, rows, masks, rlk, gk_fold,
                    gk_block, scores=None, context=None, cache_ext=None):
        scores = self.empty_ct(heads, n_cts) if scores is None else scores
        context = self.empty_ct(heads) if context is None else context
        ct = 2 * self.k * self.n
        self._check_append(cache, cache_stride_cts, 2 * heads, tau, rows, masks, d2)
        _need(q, heads * ct, "q")
        _need(a, heads * n_cts * ct, "a")
        _need(scores, heads * n_cts * ct, "scores")
        _need(context, heads * ct, "context")
        if cache_ext is not None:
            _need(cache_ext, 2 * heads * cache_stride_cts * (int(self.sizes.ct_ext_bytes) // 8), "cache_ext")
        need = int(self.lib.dll.cg_decode_step_workspace_bytes(self.h, heads, n_cts))
        if need == 0:
            raise CgError("cryptogen: invalid decode-step shape")
        if self._ws_step is None or self._ws_step.numel() < need:
            self._ws_step = None
            self._ws_step = torch.empty(need, dtype=torch.uint8, device=self.device)
        if cache_ext is None:
            self._check(self.lib.dll.cg_decode_step(
                self.h, self.stream, _ptr(q), _ptr(a), _ptr(cache), heads, n_cts, cache_stride_cts, d2, tau,
                _ptr(rows), _ptr(masks), _ptr(rlk), self._keys(gk_fold), self._keys(gk_block), _ptr(scores),
                _ptr(context), _ptr(self._ws_step)))
        else:
            self._check(self.lib.dll.cg_decode_step_ext(
                self.h, self.stream, _ptr(q), _ptr(a), _ptr(cache), _ptr(cache_ext), heads, n_cts, cache_stride_cts,
                d2, tau, _ptr(rows), _ptr(masks), _ptr(rlk), self._keys(gk_fold), self._keys(gk_block),
                _ptr(scores), _ptr(context), _ptr(self._ws_step)))
        return scores, context

    def round_galois(self, which, d2, round_bits):
        """Galois elements of all rounds of a folding sum, in key order: which = 0 scores, 1 context."""
        key = (int(which), int(d2), int(round_bits))
        if key not in self._rounds:                       # the answer depends on the arguments only
            n = C.c_uint32(0)
            self._check(self.lib.dll.cg_round_galois(self.h, which, d2, round_bits, None, 0, C.byref(n)))
            buf = (C.c_uint32 * max(1, n.value))()
            self._check(self.lib.dll.cg_round_galois(self.h, which, d2, round_bits, buf, n.value, C.byref(n)))
            self._rounds[key] = [int(buf[i]) for i in range(n.value)]
        return list(self._rounds[key])

    def _need_round_keys(self, which, d2, round_bits, keys):
        want = len(self.round_galois(which, d2, round_bits))
        if len(keys) != want:
            raise CgSizeError(f"{want} round keys needed, {len(keys)} given")

    def decode_scores_hoisted(self, q, kcache, heads, n_cts, d2, round_bits, rlk, gk_rounds, out=None,
                              cache_stride_cts=None, kext=None):
        out = self.empty_ct(heads, n_cts) if out is None else out
        ws = self.workspace(heads * n_cts)
        stride = n_cts if cache_stride_cts is None else cache_stride_cts
        self._need_round_keys(0, d2, round_bits, gk_rounds)
        if kext is None:
            self._need_products(q, heads, kcache, self._cts(1), heads, n_cts, stride, out, heads * n_cts, rlk, gk_rounds)
        else:
            self._need_products(q, heads, kext, int(self.sizes.ct_ext_bytes) // 8, heads, n_cts, stride, out,
                                heads * n_cts, rlk, gk_rounds)
        self._check(self.lib.dll.cg_decode_scores_hoisted(
            self.h, self.stream, _ptr(q), _ptr(kcache), _ptr(kext), heads, n_cts, stride, d2, round_bits, _ptr(rlk),
            self._keys(gk_rounds), _ptr(out), _ptr(ws)))
        return out

    def decode_context_hoisted(self, a, vcache, heads, n_cts, d2, round_bits, rlk, gk_rounds, out=None,
                               cache_stride_cts=None, vext=None, sum_before_scaling=False):
        out = self.empty_ct(heads) if out is None else out
        ws = self.workspace(heads * n_cts)
        stride = n_cts if cache_stride_cts is None else cache_stride_cts
        self._need_round_keys(1, d2, round_bits, gk_rounds)
        if vext is None:
            self._need_products(a, heads * n_cts, vcache, self._cts(1), heads, n_cts, stride, out, heads, rlk, gk_rounds)
        else:
            self._need_products(a, heads * n_cts, vext, int(self.sizes.ct_ext_bytes) // 8, heads, n_cts, stride, out,
                                heads, rlk, gk_rounds)
        self._check(self.lib.dll.cg_decode_context_hoisted(
            self.h, self.stream, _ptr(a), _ptr(vcache), _ptr(vext), heads, n_cts, stride, d2, round_bits,
            1 if sum_before_scaling else 0, _ptr(rlk), self._keys(gk_rounds), _ptr(out), _ptr(ws)))
        return out

    def decode_step_hoisted(self, q, a, cache, heads, n_cts, cache_stride_cts, d2, tau, rows, masks, rlk,
                            fold_round_bits, gk_fold_rounds, block_round_bits, gk_block_rounds, scores=None,
                            context=None, cache_ext=None, sum_before_scaling=False):
        scores = self.empty_ct(heads, n_cts) if scores is None else scores
        context = self.empty_ct(heads) if context is None else context
        ct = 2 * self.k * self.n
        self._check_append(cache, cache_stride_cts, 2 * heads, tau, rows, masks, d2)
        _need(q, heads * ct, "q")
        _need(a, heads * n_cts * ct, "a")
        _need(scores, heads * n_cts * ct, "scores")
        _need(context, heads * ct, "context")
        self._need_key(rlk, "rlk")
        self._need_round_keys(0, d2, fold_round_bits, gk_fold_rounds)
        self._need_round_keys(1, d2, block_round_bits, gk_block_rounds)
        for i, key in enumerate(list(gk_fold_rounds) + list(gk_block_rounds)):
            self._need_key(key, f"Galois key {i}")
        if cache_ext is not None:
            _need(cache_ext, 2 * heads * cache_stride_cts * (int(self.sizes.ct_ext_bytes) // 8), "cache_ext")
        need = int(self.lib.dll.cg_decode_step_workspace_bytes(self.h, heads, n_cts))
        if need == 0:
            raise CgError("cryptogen: invalid decode-step shape")
        if self._ws_step is None or self._ws_step.numel() < need:
            self._ws_step = None
            self._ws_step = torch.empty(need, dtype=torch.uint8, device=self.device)
        self._check(self.lib.dll.cg_decode_step_hoisted(
            self.h, self.stream, _ptr(q), _ptr(a), _ptr(cache), _ptr(cache_ext), heads, n_cts, cache_stride_cts, d2,
            tau, _ptr(rows), _ptr(masks), _ptr(rlk), fold_round_bits, self._keys(gk_fold_rounds), block_round_bits,
            1 if sum_before_scaling else 0, self._keys(gk_block_rounds), _ptr(scores), _ptr(context),
            _ptr(self._ws_step)))
        return scores, context

    def decode_scores_outer(self, q, kcols, heads, d2, masks, rlk, gk_fold, out=None):
        out = self.empty_ct(heads) if out is None else out
        ws = self.workspace(heads * d2)
        self._check(self.lib.dll.cg_decode_scores_outer(self.h, self.stream, _ptr(q), _ptr(kcols), heads, d2,
                                                        _ptr(masks), _ptr(rlk), self._keys(gk_fold), _ptr(out),
                                                        _ptr(ws)))
        return out

    def decode_context_outer(self, a, vcols, heads, d2, rlk, gk_all, out=None):
        out = self.empty_ct(heads, d2) if out is None else out
        ws = self.workspace(heads * d2)
        self._check(self.lib.dll.cg_decode_context_outer(self.h, self.stream, _ptr(a), _ptr(vcols), heads, d2,
                                                         _ptr(rlk), self._keys(gk_all), _ptr(out), _ptr(ws)))
        return out

    def prefill_qk(self, q, k, heads, d2, rlk, gk_fold, gk_blk, gk_swap, out=None):
        m = self.n // d2
        out = self.empty_ct(heads, m) if out is None else out
        ws = self.workspace(heads * m)
        self._check(self.lib.dll.cg_prefill_qk(self.h, self.stream, _ptr(q), _ptr(k), heads, d2, _ptr(rlk),
                                               self._keys(gk_fold), _ptr(gk_blk), _ptr(gk_swap), _ptr(out),
                                               _ptr(ws)))
        return out

    def prefill_av(self, a, v, heads, d2, rlk, gk_blk, gk_swap, out=None):
        out = self.empty_ct(heads) if out is None else out
        ws = self.workspace(heads * (self.n // d2))
        self._check(self.lib.dll.cg_prefill_av(self.h, self.stream, _ptr(a), _ptr(v), heads, d2, _ptr(rlk),
                                               _ptr(gk_blk), _ptr(gk_swap), _ptr(out), _ptr(ws)))
        return out

    def _need_fold_keys(self, which, d2, round_bits, keys):
        """Key count of a folding sum: the rounds' keys, or (round_bits = 0) one per generator."""
        if round_bits:
            self._need_round_keys(which, d2, round_bits, keys)
        else:
            want = len(self.round_galois(which, d2, 1))
            if len(keys) != want:
                raise CgSizeError(f"{want} rotation keys needed, {len(keys)} given")

    def prefill_qk_hoisted(self, q, k, heads, d2, rlk, gk_fold, gk_copies, out=None, fold_round_bits=0):
        m = self.n // d2
        out = self.empty_ct(heads, m) if out is None else out
        if len(gk_copies) != m - 1:
            raise CgSizeError(f"{m - 1} copy keys needed, {len(gk_copies)} given")
        self._need_fold_keys(0, d2, fold_round_bits, gk_fold)
        ws = self.workspace(heads * m)
        self._check(self.lib.dll.cg_prefill_qk_hoisted(self.h, self.stream, _ptr(q), _ptr(k), heads, d2,
                                                       fold_round_bits, _ptr(rlk), self._keys(gk_fold),
                                                       self._keys(gk_copies), _ptr(out), _ptr(ws)))
        return out

    def prefill_av_hoisted(self, a, v, heads, d2, rlk, gk_copies, out=None, sum_before_scaling=False):
        m = self.n // d2
        out = self.empty_ct(heads) if out is None else out
        if len(gk_copies) != m - 1:
            raise CgSizeError(f"{m - 1} copy keys needed, {len(gk_copies)} given")
        ws = self.workspace(heads * m)
        self._check(self.lib.dll.cg_prefill_av_hoisted(self.h, self.stream, _ptr(a), _ptr(v), heads, d2,
                                                       1 if sum_before_scaling else 0, _ptr(rlk),
                                                       self._keys(gk_copies), _ptr(out), _ptr(ws)))
        return out

    def prefill_repack(self, x, heads, d2, mask0, gk_right, out=None):
        m = self.n // d2
        w = min(d2, m // 2)
        out = self.empty_ct(heads * m // w) if out is None else out
        ws = self.workspace(heads * m)
        self._check(self.lib.dll.cg_prefill_repack(self.h, self.stream, _ptr(x), heads, d2, _ptr(mask0),
                                                   self._keys(gk_right), _ptr(out), _ptr(ws)))
        return out

    def cpvm(self, x, diags, units, n_diag, d2, gk_shift, gk_block, out=None):
        """x: one ciphertext (the token); diags: prepared plaintexts [units][n_diag] (flat)."""
        out = self.empty_ct(units) if out is None else out
        _need(x, self._cts(1), "x")
        _need(diags, max(0, int(units)) * max(0, int(n_diag)) * self.k * self.n, "diags (prepared)")
        _need(out, self._cts(units), "out")
        for i, key in enumerate(list(gk_shift) + list(gk_block)):
            self._need_key(key, f"Galois key {i}")
        ws = self.workspace(units + n_diag)
        shift = self._keys(gk_shift) if len(gk_shift) else None
        self._check(self.lib.dll.cg_cpvm(self.h, self.stream, _ptr(x), _ptr(diags), units, n_diag, d2, shift,
                                         self._keys(gk_block), _ptr(out), _ptr(ws)))
        return out

    def cpvm_hoisted(self, x, diags, units, n_diag, d2, gk_copies, gk_block, out=None, block_round_bits=0):
        """cpvm with the token's copies made by one series of hoisted rotations (keys for 3^1 .. 3^(n_diag-1));
        block_round_bits >= 1: the sum over residue classes in rounds (gk_block: the rounds' keys)."""
        out = self.empty_ct(units) if out is None else out
        _need(x, self._cts(1), "x")
        _need(diags, max(0, int(units)) * max(0, int(n_diag)) * self.k * self.n, "diags (prepared)")
        _need(out, self._cts(units), "out")
        for i, key in enumerate(list(gk_copies) + list(gk_block)):
            self._need_key(key, f"Galois key {i}")
        if len(gk_copies) != max(0, int(n_diag) - 1):
            raise CgSizeError(f"{int(n_diag) - 1} copy keys needed, {len(gk_copies)} given")
        self._need_fold_keys(1, d2, block_round_bits, gk_block)
        ws = self.workspace(units + n_diag)
        copies = self._keys(gk_copies) if len(gk_copies) else None
        self._check(self.lib.dll.cg_cpvm_hoisted(self.h, self.stream, _ptr(x), _ptr(diags), units, n_diag, d2,
                                                 block_round_bits, copies, self._keys(gk_block), _ptr(out), _ptr(ws)))
        return out

    def profile_begin(self, max_launches=65536):
        self._check(self.lib.dll.cg_profile_begin(self.h, max_launches))

    def profile_end(self):
        """-> list of dicts {name, launches, total_ms, algo_bytes, work_items} per kernel class."""
        stats = (_KernelStat * 32)()
        n = C.c_uint32(0)
        self._check(self.lib.dll.cg_profile_end(self.h, stats, 32, C.byref(n)))
        return [dict(name=self.lib.dll.cg_kernel_name(stats[i].kernel_id).decode(),
                     launches=int(stats[i].launches), total_ms=float(stats[i].total_ms),
                     algo_bytes=float(stats[i].algo_bytes), work_items=float(stats[i].work_items))
                for i in range(n.value)]

    def bench_exchange(self, kind, n_blocks, iters, out=None):
        out = torch.empty(n_blocks * 1024, dtype=torch.float64, device=self.device) if out is None else out
        self._check(self.lib.dll.cg_bench_exchange(self.h, self.stream, kind, n_blocks, iters, _ptr(out)))
        return out

    def bench_modmul(self, kind, n_lanes, iters, out=None):
        out = torch.empty(n_lanes, dtype=torch.int64, device=self.device) if out is None else out
        self._check(self.lib.dll.cg_bench_modmul(self.h, self.stream, kind, n_lanes, iters, _ptr(out)))
        return out
