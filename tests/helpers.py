"""Test-side harness: builds oracle parameter sets and client material (keys,
ciphertexts) from the seeded raw inputs.  Everything here runs on the oracle;
nothing comes from the HIP path."""
import numpy as np

import oracle
from oracle import encoding as E
from paper_2604_09975_amd import workload as W


def ring_primes(spec):
    """Descending search per bit size; special primes take the earliest hits of their size."""
    need = {}
    for b in spec.p_bits + spec.q_bits:
        need[b] = need.get(b, 0) + 1
    hits = {b: oracle.find_primes(b, spec.logN, c) for b, c in need.items()}
    pos = {b: 0 for b in need}
    p, q = [], []
    for b in spec.p_bits:
        p.append(hits[b][pos[b]]); pos[b] += 1
    for b in spec.q_bits:
        q.append(hits[b][pos[b]]); pos[b] += 1
    return q, p


def make_oracle(spec):
    q, p = ring_primes(spec)
    return oracle.Oracle(spec.logN, q, p, spec.dnum)


def small_oracle(logN, L=3, K=1, dnum=3, qbits=30, pbits=32):
    """Tiny rings for brute-force pins."""
    q = oracle.find_primes(qbits, logN, L)
    p = oracle.find_primes(pbits, logN, K)
    return oracle.Oracle(logN, q, p, dnum)


class Client:
    """Holds a secret key and draws key-switching / encryption randomness from one rng."""

    def __init__(self, O, seed, hamming_weight=64):
        self.O = O
        self.r = W.rng(seed)
        self.s = W.ternary_secret(self.r, O.N, hamming_weight)

    def galois_key(self, g):
        O = self.O
        a = W.uniform_residues(self.r, O.moduli, O.N, lead=(O.dnum,))
        e = W.gaussian_error(self.r, (O.dnum, O.N))
        return O.galois_keygen(self.s, g, a, e)

    def relin_key(self):
        O = self.O
        a = W.uniform_residues(self.r, O.moduli, O.N, lead=(O.dnum,))
        e = W.gaussian_error(self.r, (O.dnum, O.N))
        return O.relin_keygen(self.s, a, e)

    def encrypt_coeffs(self, m, level):
        O = self.O
        a = W.uniform_residues(self.r, O.q[:level], O.N)
        e = W.gaussian_error(self.r, (O.N,))
        return O.encrypt(level, m, self.s, a, e)

    def encrypt_slots(self, z, scale, level):
        return self.encrypt_coeffs(E.encode(z, scale, self.O.N), level)

    def decrypt_slots(self, ct, level, scale, nlimbs=None):
        O = self.O
        if nlimbs is None:
            nlimbs = min(level, 3)
        m = O.decrypt_centred(ct, level, self.s, nlimbs)
        return E.decode(m, scale, O.N)


def brev(k, bits):
    r = 0
    for i in range(bits):
        r |= ((k >> i) & 1) << (bits - 1 - i)
    return r


def crt_nonneg(res_cols, moduli):
    """Python-int CRT to [0, M) of one coefficient given its residues."""
    M = 1
    for q in moduli:
        M *= q
    v = 0
    for r, q in zip(res_cols, moduli):
        Mi = M // q
        v += int(r) * Mi * pow(Mi % q, -1, q)
    return v % M, M
