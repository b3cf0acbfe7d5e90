"""CPU oracle for the CKKS ct x pt matmul path -- TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this package.  The product path never does.

`Oracle` is a ctypes view of ckks_oracle.c (integer arithmetic, the bit-exact
definition); `encoding` holds the fp64 slot encode/decode and the plaintext
diagonal layout of the projection kernel in numpy.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build
from . import encoding  # noqa: F401

_u64p = C.POINTER(C.c_uint64)
_i64p = C.POINTER(C.c_int64)
_i8p = C.POINTER(C.c_int8)

CONJ = "conj"


def _lib():
    # CKKS_ORACLE_LIB: a library built elsewhere from (a copy of) ckks_oracle.c; the mutation tests point it at
    # deliberately broken builds to show that the pins catch them
    lib = C.CDLL(os.environ.get("CKKS_ORACLE_LIB") or _build.build())
    lib.orc_mulmod.restype = C.c_uint64
    lib.orc_mulmod.argtypes = [C.c_uint64] * 3
    lib.orc_powmod.restype = C.c_uint64
    lib.orc_powmod.argtypes = [C.c_uint64] * 3
    lib.orc_is_prime.restype = C.c_int
    lib.orc_is_prime.argtypes = [C.c_uint64]
    lib.orc_find_primes.restype = C.c_int
    lib.orc_find_primes.argtypes = [C.c_int, C.c_int, C.c_int, _u64p]
    lib.orc_min_root.restype = C.c_uint64
    lib.orc_min_root.argtypes = [C.c_uint64, C.c_int]
    lib.orc_ctx_create.restype = C.c_void_p
    lib.orc_ctx_create.argtypes = [C.c_int, _u64p, C.c_int, _u64p, C.c_int, C.c_int]
    lib.orc_ctx_destroy.argtypes = [C.c_void_p]
    lib.orc_modulus.restype = C.c_uint64
    lib.orc_modulus.argtypes = [C.c_void_p, C.c_int]
    lib.orc_psi.restype = C.c_uint64
    lib.orc_psi.argtypes = [C.c_void_p, C.c_int]
    lib.orc_ntt_naive.argtypes = [C.c_void_p, C.c_int, _u64p, _u64p]
    lib.orc_ntt.argtypes = [C.c_void_p, C.c_int, _u64p]
    lib.orc_intt.argtypes = [C.c_void_p, C.c_int, _u64p]
    lib.orc_galois_elt.restype = C.c_uint64
    lib.orc_galois_elt.argtypes = [C.c_void_p, C.c_int64, C.c_int]
    lib.orc_automorph_coeff.argtypes = [C.c_void_p, C.c_int, C.c_uint64, _u64p, _u64p]
    lib.orc_automorph_ntt.argtypes = [C.c_void_p, C.c_uint64, _u64p, _u64p]
    lib.orc_modup.argtypes = [C.c_void_p, C.c_int, C.c_int, _u64p, _u64p]
    lib.orc_moddown.argtypes = [C.c_void_p, C.c_int, _u64p, _u64p]
    lib.orc_rotate_hoisted.argtypes = [C.c_void_p, _u64p, C.c_int, _u64p, C.c_int, C.POINTER(_u64p), _u64p]
    lib.orc_expand_plain.argtypes = [C.c_void_p, C.c_int, _i64p, _u64p]
    lib.orc_ctpt_matmul.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                                    _i64p, _i64p, C.c_uint64, _u64p, C.POINTER(_u64p), C.POINTER(_u64p), _u64p,
                                    _u64p, C.c_int, C.c_int, C.c_int, C.c_int]
    lib.orc_rescale.argtypes = [C.c_void_p, _u64p, C.c_int, C.c_int, _u64p]
    lib.orc_galois_keygen.argtypes = [C.c_void_p, _i8p, C.c_uint64, _u64p, _i64p, _u64p]
    lib.orc_add.argtypes = [C.c_void_p, _u64p, _u64p, C.c_int, C.c_int, _u64p]
    lib.orc_ptmul.argtypes = [C.c_void_p, _u64p, C.c_int, _u64p, _u64p]
    lib.orc_mod_switch.argtypes = [C.c_void_p, _u64p, C.c_int, C.c_int, _u64p]
    lib.orc_rot_first.argtypes = [C.c_void_p, _u64p, C.c_int, _u64p, C.POINTER(_u64p), _u64p, _u64p, _u64p]
    lib.orc_shift_bank.argtypes = [C.c_void_p, _u64p, C.c_int, C.c_int, _u64p, C.POINTER(_u64p), _u64p, _u64p]
    lib.orc_relin_keygen.argtypes = [C.c_void_p, _i8p, _u64p, _i64p, _u64p]
    lib.orc_ctmul.argtypes = [C.c_void_p, _u64p, _u64p, C.c_int, _u64p, _u64p]
    lib.orc_encrypt.argtypes = [C.c_void_p, C.c_int, _i64p, _i8p, _u64p, _i64p, _u64p]
    lib.orc_decrypt.argtypes = [C.c_void_p, _u64p, C.c_int, _i8p, C.c_int, _u64p]
    return lib


LIB = _lib()


def _u64(a):
    a = np.ascontiguousarray(a, dtype=np.uint64)
    return a, a.ctypes.data_as(_u64p)


def _i64(a):
    a = np.ascontiguousarray(a, dtype=np.int64)
    return a, a.ctypes.data_as(_i64p)


def _i8(a):
    a = np.ascontiguousarray(a, dtype=np.int8)
    return a, a.ctypes.data_as(_i8p)


def find_primes(bits, logN, count):
    out = np.zeros(count, dtype=np.uint64)
    n = LIB.orc_find_primes(bits, logN, count, out.ctypes.data_as(_u64p))
    assert n == count
    return [int(x) for x in out]


def is_prime(n):
    return bool(LIB.orc_is_prime(n))


def min_root(q, logN):
    return int(LIB.orc_min_root(q, logN))


def mulmod(a, b, q):
    return int(LIB.orc_mulmod(a, b, q))


class Oracle:
    """One parameter set: ring degree 2^logN, ciphertext primes q, special primes p, dnum digits."""

    def __init__(self, logN, q, p, dnum):
        self.logN, self.N, self.n = logN, 1 << logN, 1 << (logN - 1)
        self.q, self.p = [int(x) for x in q], [int(x) for x in p]
        self.L, self.K, self.dnum = len(q), len(p), dnum
        self.alpha = self.L // dnum
        qa, qp = _u64(self.q)
        pa, pp = _u64(self.p)
        self._h = LIB.orc_ctx_create(logN, qp, self.L, pp, self.K, dnum)
        if not self._h:
            raise ValueError("bad oracle parameters")
        self.moduli = self.q + self.p

    def __del__(self):
        if getattr(self, "_h", None):
            LIB.orc_ctx_destroy(self._h)
            self._h = None

    def psi(self, limb):
        return int(LIB.orc_psi(self._h, limb))

    # -- transforms ---------------------------------------------------
    def ntt(self, limb, a):
        a, p = _u64(np.array(a, dtype=np.uint64))
        LIB.orc_ntt(self._h, limb, p)
        return a

    def intt(self, limb, a):
        a, p = _u64(np.array(a, dtype=np.uint64))
        LIB.orc_intt(self._h, limb, p)
        return a

    def ntt_naive(self, limb, a):
        a, p = _u64(a)
        out = np.zeros_like(a)
        LIB.orc_ntt_naive(self._h, limb, p, out.ctypes.data_as(_u64p))
        return out

    def ntt_batch(self, data, limb_ids, inverse=False):
        """data [batch][n_limbs][N]; returns a transformed copy."""
        data = np.array(data, dtype=np.uint64)
        flat = data.reshape(-1, len(limb_ids), self.N)
        f = LIB.orc_intt if inverse else LIB.orc_ntt
        for b in range(flat.shape[0]):
            for i, limb in enumerate(limb_ids):
                f(self._h, int(limb), flat[b, i].ctypes.data_as(_u64p))
        return data

    # -- automorphisms ------------------------------------------------
    def galois_elt(self, step):
        if step == CONJ:
            return int(LIB.orc_galois_elt(self._h, 0, 1))
        return int(LIB.orc_galois_elt(self._h, int(step), 0))

    def automorph_coeff(self, limb, g, a):
        a, p = _u64(a)
        out = np.zeros_like(a)
        LIB.orc_automorph_coeff(self._h, limb, g, p, out.ctypes.data_as(_u64p))
        return out

    def automorph_ntt(self, g, a):
        a, p = _u64(a)
        out = np.zeros_like(a)
        LIB.orc_automorph_ntt(self._h, g, p, out.ctypes.data_as(_u64p))
        return out

    # -- base conversion ----------------------------------------------
    def modup(self, level, j, c_coeff):
        a, p = _u64(c_coeff)
        assert a.shape == (level, self.N)
        out = np.zeros((level + self.K, self.N), dtype=np.uint64)
        LIB.orc_modup(self._h, level, j, p, out.ctypes.data_as(_u64p))
        return out

    def moddown(self, level, u):
        a, p = _u64(u)
        assert a.shape == (level + self.K, self.N)
        out = np.zeros((level, self.N), dtype=np.uint64)
        LIB.orc_moddown(self._h, level, p, out.ctypes.data_as(_u64p))
        return out

    # -- rotations ----------------------------------------------------
    def rotate_hoisted(self, ct, level, gelts, keys):
        """ct [2][level][N]; gelts list of Galois elements (1 = identity); keys list (None for identity)."""
        a, p = _u64(ct)
        assert a.shape == (2, level, self.N)
        n = len(gelts)
        g, gp = _u64(np.array(gelts, dtype=np.uint64))
        keep = []
        kp = (_u64p * n)()
        for i, k in enumerate(keys):
            if k is None:
                kp[i] = None
            else:
                ka, kptr = _u64(k)
                assert ka.shape == (self.dnum, 2, self.L + self.K, self.N)
                keep.append(ka)
                kp[i] = kptr
        out = np.zeros((n, 2, level, self.N), dtype=np.uint64)
        LIB.orc_rotate_hoisted(self._h, p, level, gp, n, kp, out.ctypes.data_as(_u64p))
        return out

    # -- matmul -------------------------------------------------------
    def expand_plain(self, level, coef):
        a, p = _i64(coef)
        out = np.zeros((level, self.N), dtype=np.uint64)
        LIB.orc_expand_plain(self._h, level, p, out.ctypes.data_as(_u64p))
        return out

    def ctpt_matmul(self, level, m, G, B_out, N1, N2, diag, bias, bias_mul, ct_x, baby_keys, giant_keys,
                    b_first=0, b_count=None, conj_key=None, merged=False, conj_per_acc=False):
        if b_count is None:
            b_count = B_out
        d, dp = _i64(diag)
        assert d.shape == (B_out, N2, G, N1, self.N)
        if bias is not None:
            bb, bp = _i64(bias)
            assert bb.shape == (B_out, self.N)
        else:
            bp = None
        x, xp = _u64(ct_x)
        assert x.shape == (G, 2, level, self.N)
        keep = []

        def ptrs(keys, cnt):
            arr = (_u64p * max(cnt, 1))()
            assert len(keys) == cnt
            for i, k in enumerate(keys):
                ka, kptr = _u64(k)
                keep.append(ka)
                arr[i] = kptr
            return arr

        bk, gk = ptrs(baby_keys, N1 - 1), ptrs(giant_keys, N2 - 1)
        ck = None
        if conj_key is not None:
            cka, ck = _u64(conj_key)
            keep.append(cka)
        out = np.zeros((B_out, 2, level, self.N), dtype=np.uint64)
        LIB.orc_ctpt_matmul(self._h, level, m, G, B_out, N1, N2, dp, bp, bias_mul, xp, bk, gk, ck,
                            out.ctypes.data_as(_u64p), b_first, b_count, int(merged), int(conj_per_acc))
        return out

    def rescale(self, ct, level):
        a, p = _u64(ct)
        n_ct = a.shape[0]
        assert a.shape == (n_ct, 2, level, self.N)
        out = np.zeros((n_ct, 2, level - 1, self.N), dtype=np.uint64)
        LIB.orc_rescale(self._h, p, level, n_ct, out.ctypes.data_as(_u64p))
        return out

    # -- client -------------------------------------------------------
    def galois_keygen(self, s, g, a, e):
        s_, sp = _i8(s)
        a_, ap = _u64(a)
        e_, ep = _i64(e)
        W = self.L + self.K
        assert a_.shape == (self.dnum, W, self.N) and e_.shape == (self.dnum, self.N)
        key = np.zeros((self.dnum, 2, W, self.N), dtype=np.uint64)
        LIB.orc_galois_keygen(self._h, sp, g, ap, ep, key.ctypes.data_as(_u64p))
        return key

    def add(self, a, b, level):
        a_, ap = _u64(a)
        b_, bp = _u64(b)
        n_ct = a_.size // (2 * level * self.N)
        out = np.zeros_like(a_)
        LIB.orc_add(self._h, ap, bp, level, n_ct, out.ctypes.data_as(_u64p))
        return out

    def ptmul(self, ct, level, pt):
        c_, cp = _u64(ct)
        p_, pp = _u64(pt)
        assert c_.shape == (2, level, self.N) and p_.shape == (level, self.N)
        out = np.zeros_like(c_)
        LIB.orc_ptmul(self._h, cp, level, pp, out.ctypes.data_as(_u64p))
        return out

    def mod_switch(self, ct, level):
        c_, cp = _u64(ct)
        n_ct = c_.shape[0]
        assert c_.shape == (n_ct, 2, level, self.N)
        out = np.zeros((n_ct, 2, level - 1, self.N), dtype=np.uint64)
        LIB.orc_mod_switch(self._h, cp, level, n_ct, out.ctypes.data_as(_u64p))
        return out

    def rot_first(self, ct, level, gelts, keys, mask_a, mask_b):
        c_, cp = _u64(ct)
        g_, gp = _u64(np.array(gelts, dtype=np.uint64))
        keep, kp = [], (_u64p * 2)()
        for i, k in enumerate(keys):
            if k is None:
                kp[i] = None
            else:
                ka, kptr = _u64(k)
                keep.append(ka)
                kp[i] = kptr
        a_, ap = _u64(mask_a)
        b_, bp = _u64(mask_b)
        out = np.zeros_like(c_)
        LIB.orc_rot_first(self._h, cp, level, gp, kp, ap, bp, out.ctypes.data_as(_u64p))
        return out

    def shift_bank(self, ct, level, gelts, keys, masks):
        """gelts, keys: n_out pairs; masks [n_out][2][level][N] -> [n_out][2][level][N]."""
        c_, cp = _u64(ct)
        n_out = len(gelts)
        g_, gp = _u64(np.array(gelts, dtype=np.uint64).reshape(-1))
        keep, kp = [], (_u64p * (2 * n_out))()
        for i, pair in enumerate(keys):
            for e, k in enumerate(pair):
                if k is None:
                    kp[2 * i + e] = None
                else:
                    ka, kptr = _u64(k)
                    keep.append(ka)
                    kp[2 * i + e] = kptr
        m_, mp = _u64(masks)
        assert m_.shape == (n_out, 2, level, self.N)
        out = np.zeros((n_out, 2, level, self.N), dtype=np.uint64)
        LIB.orc_shift_bank(self._h, cp, level, n_out, gp, kp, mp, out.ctypes.data_as(_u64p))
        return out

    def relin_keygen(self, s, a, e):
        s_, sp = _i8(s)
        a_, ap = _u64(a)
        e_, ep = _i64(e)
        W = self.L + self.K
        assert a_.shape == (self.dnum, W, self.N) and e_.shape == (self.dnum, self.N)
        key = np.zeros((self.dnum, 2, W, self.N), dtype=np.uint64)
        LIB.orc_relin_keygen(self._h, sp, ap, ep, key.ctypes.data_as(_u64p))
        return key

    def ctmul(self, ct_a, ct_b, level, relin_key):
        a_, ap = _u64(ct_a)
        b_, bp = _u64(ct_b)
        k_, kp = _u64(relin_key)
        assert a_.shape == b_.shape == (2, level, self.N)
        out = np.zeros((2, level, self.N), dtype=np.uint64)
        LIB.orc_ctmul(self._h, ap, bp, level, kp, out.ctypes.data_as(_u64p))
        return out

    def encrypt(self, level, m, s, a, e):
        m_, mp = _i64(m)
        s_, sp = _i8(s)
        a_, ap = _u64(a)
        e_, ep = _i64(e)
        assert a_.shape == (level, self.N)
        ct = np.zeros((2, level, self.N), dtype=np.uint64)
        LIB.orc_encrypt(self._h, level, mp, sp, ap, ep, ct.ctypes.data_as(_u64p))
        return ct

    def decrypt(self, ct, level, s, nlimbs):
        """Coefficient-domain residues of c0 + c1*s on the first nlimbs limbs, [nlimbs][N]."""
        c_, cp = _u64(ct)
        s_, sp = _i8(s)
        out = np.zeros((nlimbs, self.N), dtype=np.uint64)
        LIB.orc_decrypt(self._h, cp, level, sp, nlimbs, out.ctypes.data_as(_u64p))
        return out

    def decrypt_centred(self, ct, level, s, nlimbs):
        """Decrypt and CRT-lift to centred Python integers (list of N ints)."""
        res = self.decrypt(ct, level, s, nlimbs)
        return encoding.crt_centre(res, self.q[:nlimbs])
