"""The few values the paper prints for this path (tests/golden/paper_values.txt), reproduced by the oracle's packing and
ciphertext layout and by the product's host-side packing: block counts, segment counts, complexified input counts,
ciphertext bytes."""
import os

import numpy as np

import oracle
from oracle import encoding as OE
from paper_2604_09975_amd import client as CL

HERE = os.path.dirname(os.path.abspath(__file__))


def rows():
    out = []
    for line in open(os.path.join(HERE, "golden", "paper_values.txt")):
        if line.startswith("#") or not line.strip():
            continue
        key, args, value, cite = [p.strip() for p in line.split("|")]
        out.append((key, dict((k, int(v)) for k, v in (a.split("=") for a in args.split())), int(value), cite))
    return out


def ct_bytes(N, L):
    """Bytes of a fresh ciphertext as the oracle lays it out (Sec. 5: two polynomials of N residues per limb)."""
    logN = N.bit_length() - 1
    dnum = 3
    O = oracle.Oracle(logN, oracle.find_primes(50, logN, L), oracle.find_primes(60, logN, L // dnum), dnum)
    z = np.zeros(N, dtype=np.int64)
    ct = O.encrypt(L, z, np.zeros(N, dtype=np.int8), np.zeros((L, N), dtype=np.uint64), z)
    return ct.nbytes


def blocks(d, C, n=16384, m=128):
    """Ciphertexts that hold a d-column matrix with C active columns each: what the two packers emit."""
    X = np.arange(m * d, dtype=np.float64).reshape(m, d)
    a, b = OE.pack_columns(X, n, C), CL.pack_columns(X, n, C)
    assert np.array_equal(a, b)
    return a.shape[0]


def segments(n, m):
    """Segments of m slots in a ciphertext of n slots, read off the packed layout: with C = n/m every segment c
    holds column c, so the number of distinct columns found at stride m is N_seg."""
    C = n // m
    X = np.tile(np.arange(1, C + 1, dtype=np.float64), (m, 1))          # column c is constant c + 1
    packed = OE.pack_columns(X, n, C)
    assert packed.shape == (1, n)
    firsts = packed[0, ::m]
    assert np.array_equal(packed[0], np.repeat(firsts, m))
    return len(set(firsts.tolist()))


def pairs(G, n=16384, m=128, C=128):
    """Complexified inputs for G real input groups: what the two packers emit."""
    X = np.arange(m * G * C, dtype=np.float64).reshape(m, G * C)
    a, b = OE.pack_columns_complex(X, n, C), CL.pack_columns_complex(X, n, C)
    assert np.array_equal(a, b)
    return a.shape[0]


def test_paper_values():
    seen = set()
    for key, a, value, cite in rows():
        assert cite, "every golden value carries its citation"
        got = {"ct_bytes": ct_bytes, "blocks": blocks, "segments": segments, "pairs": pairs}[key](**a)
        assert got == value, (key, a, got, value, cite)
        seen.add(key)
    assert seen == {"ct_bytes", "blocks", "segments", "pairs"}
