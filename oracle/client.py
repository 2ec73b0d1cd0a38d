"""Host-side party that owns the secret key (test infrastructure only).

Slot encoding, key generation, symmetric encryption and decryption for BFV,
written with Python integers and the oracle's word-size polynomial product.
None of this runs on the GPU path: the server-side library is keygen-free.

Conventions (the paper names BFV with SIMD batching and leaves these open):
  * plaintext slots form 2 rows of N/2; flat slot j = row * N/2 + pos;
    slot j is the plaintext polynomial evaluated at zeta^e_j with
    e_j = 3^pos (row 0) or -3^pos (row 1) mod 2N, zeta the smallest primitive
    2N-th root of unity modulo t;
  * the Galois map X -> X^(3^r) rotates both rows left by r, X -> X^(2N-1)
    swaps the rows;
  * secret: uniform ternary; errors: rounded normal, sigma 3.2, clipped at 19;
  * ciphertext (c0, c1) = (-a s + e + floor(Q/t) m, a), decrypting as
    round(t (c0 + c1 s + c2 s^2) / Q) mod t.
  * switching key for s' -> s, digit j (alpha consecutive ciphertext primes,
    product Q_j):  (-a_j s + e_j + P T_j s', a_j) modulo P Q, with
    T_j = (Q/Q_j) * ((Q/Q_j)^-1 mod Q_j).
"""
from math import log2, prod

import numpy as np

from workloads import Stream, gaussian_error, ternary_secret, uniform_residues

from . import bfv


class SlotCodec:
    """Batch encoding: N values modulo t <-> plaintext polynomial (public, no key)."""

    def __init__(self, params):
        self.n, self.t = params.n, int(params.t)
        n = self.n
        self.zeta = bfv.min_psi(n, self.t)
        e = np.empty(n, dtype=np.int64)
        pw = 1
        for pos in range(n // 2):
            e[pos] = pw
            e[n // 2 + pos] = (2 * n - pw) % (2 * n)
            pw = pw * 3 % (2 * n)
        self.exponent = e
        self.index = (e - 1) // 2       # position of slot j among zeta^(2i+1)

    def encode(self, values) -> np.ndarray:
        v = np.mod(np.asarray(values, dtype=np.int64), self.t).astype(np.uint64)
        assert v.shape == (self.n,)
        ev = np.zeros(self.n, dtype=np.uint64)
        ev[self.index] = v
        return bfv.interp_odd(ev, self.t, self.zeta)

    def decode(self, pt) -> np.ndarray:
        ev = bfv.eval_odd(np.asarray(pt, dtype=np.uint64), self.t, self.zeta)
        return ev[self.index].astype(np.int64)


def galois_rot(n: int, r: int) -> int:
    """Galois element rotating both slot rows left by r."""
    return pow(3, r, 2 * n)


def galois_swap(n: int) -> int:
    return 2 * n - 1


class Client:
    def __init__(self, params, seed: int, oracle: "bfv.Oracle" = None):
        self.params = params
        self.n, self.t = params.n, int(params.t)
        self.q = [int(x) for x in params.q]
        self.p = [int(x) for x in params.p]
        self.qp = self.q + self.p
        self.Q, self.P = prod(self.q), prod(self.p)
        self.delta = self.Q // self.t
        self.codec = SlotCodec(params)
        self.oracle = oracle
        self.seed = seed
        self.s = ternary_secret(Stream(seed, 1), self.n)
        self._ctr = 0
        self._s2 = None

    # -- small helpers -------------------------------------------------------
    def _fresh(self) -> np.random.Generator:
        self._ctr += 1
        return Stream(self.seed, 2, self._ctr)

    @staticmethod
    def _res(poly, m: int) -> np.ndarray:
        """Residues of a small signed integer polynomial modulo m."""
        return np.mod(np.asarray(poly, dtype=np.int64), np.int64(m)).astype(np.uint64)

    def _centre_small(self, res, m: int) -> np.ndarray:
        r = np.asarray(res, dtype=np.uint64).astype(np.int64)
        return np.where(r > m // 2, r - m, r)

    def secret_square(self) -> np.ndarray:
        """s^2 over the integers (|coefficients| <= N)."""
        if self._s2 is None:
            m = self.q[0]
            sr = self._res(self.s, m)
            self._s2 = self._centre_small(bfv.polymul(sr, sr, m), m)
        return self._s2

    def secret_galois(self, g: int) -> np.ndarray:
        """s(X^g) over the integers."""
        n = self.n
        out = np.zeros(n, dtype=np.int64)
        for i in range(n):
            e = i * g % (2 * n)
            if e >= n:
                out[e - n] = -self.s[i]
            else:
                out[e] = self.s[i]
        return out

    # -- encryption ----------------------------------------------------------
    def encrypt_poly(self, pt) -> np.ndarray:
        """Fresh symmetric encryption of plaintext polynomial pt (values mod t)."""
        g = self._fresh()
        n, k = self.n, len(self.q)
        a = uniform_residues(g, self.q, n)
        e = gaussian_error(g, n, self.params.sigma, self.params.err_clip)
        ct = np.empty((2, k, n), dtype=np.uint64)
        pt_int = [int(x) for x in np.asarray(pt, dtype=np.uint64)]
        for i, m in enumerate(self.q):
            as_ = bfv.polymul(a[i], self._res(self.s, m), m)
            dm = self.delta % m
            scaled = np.array([dm * x % m for x in pt_int], dtype=np.uint64)
            c0 = (self._res(e, m).astype(object) + scaled.astype(object)
                  + (m - as_.astype(object))) % m
            ct[0, i] = c0.astype(np.uint64)
            ct[1, i] = a[i]
        return ct

    def encrypt_slots(self, values) -> np.ndarray:
        return self.encrypt_poly(self.codec.encode(values))

    def trivial(self, pt) -> np.ndarray:
        """Noise-free, key-free ciphertext (floor(Q/t) m, 0)."""
        n, k = self.n, len(self.q)
        ct = np.zeros((2, k, n), dtype=np.uint64)
        pt_int = [int(x) for x in np.asarray(pt, dtype=np.uint64)]
        for i, m in enumerate(self.q):
            dm = self.delta % m
            ct[0, i] = np.array([dm * x % m for x in pt_int], dtype=np.uint64)
        return ct

    # -- decryption ----------------------------------------------------------
    def _phase(self, ct):
        """Centred integer coefficients of c0 + c1 s + c2 s^2 mod Q."""
        ct = np.asarray(ct, dtype=np.uint64)
        ncomp = ct.shape[0]
        k = len(self.q)
        res = []
        for i, m in enumerate(self.q):
            acc = ct[0, i].astype(object)
            acc = acc + bfv.polymul(ct[1, i], self._res(self.s, m), m).astype(object)
            if ncomp == 3:
                acc = acc + bfv.polymul(ct[2, i], self._res(self.secret_square(), m),
                                        m).astype(object)
            res.append(acc % m)
        hats = [self.Q // m for m in self.q]
        invs = [pow(h % m, -1, m) for h, m in zip(hats, self.q)]
        out = []
        for j in range(self.n):
            x = sum(int(res[i][j]) * invs[i] % self.q[i] * hats[i] for i in range(k)) % self.Q
            out.append(x - self.Q if x > self.Q // 2 else x)
        return out

    def decrypt_poly(self, ct) -> np.ndarray:
        t, Q = self.t, self.Q
        return np.array([((2 * t * x + Q) // (2 * Q)) % t for x in self._phase(ct)],
                        dtype=np.uint64)

    def decrypt_slots(self, ct) -> np.ndarray:
        return self.codec.decode(self.decrypt_poly(ct))

    def noise_budget_bits(self, ct, pt) -> float:
        """log2(Q/2) - log2(max |t x - Q m| centred mod tQ): decryption is correct iff > 0."""
        t, Q = self.t, self.Q
        worst = 1
        for x, m in zip(self._phase(ct), [int(v) for v in np.asarray(pt, dtype=np.uint64)]):
            r = (t * x - Q * m) % (t * Q)
            if r > t * Q // 2:
                r -= t * Q
            worst = max(worst, abs(r))
        return log2(Q / 2) - log2(worst)

    def refresh(self, share_ct) -> np.ndarray:
        """The client's part of the lazy noise refresh (Algorithm 1 step 1): decrypt the masked
        share and encrypt it afresh."""
        return self.encrypt_poly(self.decrypt_poly(share_ct))

    # -- switching keys ------------------------------------------------------
    def switch_key(self, s_prime) -> np.ndarray:
        """Key that moves a component under s_prime to the key s."""
        prm = self.params
        n, k, alpha, dnum = self.n, prm.k, prm.alpha, prm.dnum
        L = k + prm.nsp
        ksk = np.empty((dnum, 2, L, n), dtype=np.uint64)
        sp = [int(x) for x in np.asarray(s_prime, dtype=np.int64)]
        for j in range(dnum):
            g = self._fresh()
            qj = prod(self.q[j * alpha:(j + 1) * alpha])
            qhat = self.Q // qj
            tj = qhat * pow(qhat % qj, -1, qj) % self.Q
            a = uniform_residues(g, self.qp, n)
            e = gaussian_error(g, n, prm.sigma, prm.err_clip)
            for r, m in enumerate(self.qp):
                as_ = bfv.polymul(a[r], self._res(self.s, m), m)
                c = self.P * tj % m
                gadget = np.array([c * x % m for x in sp], dtype=object)
                b = (self._res(e, m).astype(object) + gadget + (m - as_.astype(object))) % m
                ksk[j, 0, r] = b.astype(np.uint64)
                ksk[j, 1, r] = a[r]
        return ksk

    def relin_key(self) -> np.ndarray:
        return self.switch_key(self.secret_square())

    def galois_key(self, g: int) -> np.ndarray:
        return self.switch_key(self.secret_galois(g))
