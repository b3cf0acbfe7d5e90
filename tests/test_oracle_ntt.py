"""Pins for the oracle's negacyclic NTT."""
import numpy as np
import pytest

import oracle
from tests import helpers
from paper_2604_09975_amd import workload as W


def schoolbook_negacyclic(a, b, q):
    N = len(a)
    out = [0] * N
    for i in range(N):
        for j in range(N):
            k = i + j
            v = int(a[i]) * int(b[j])
            if k < N:
                out[k] += v
            else:
                out[k - N] -= v
    return [x % q for x in out]


@pytest.mark.parametrize("logN", [2, 3, 5, 8])
def test_convolution_theorem_vs_schoolbook(logN):
    O = helpers.small_oracle(logN)
    r = np.random.default_rng(logN)
    for limb in range(O.L + O.K):
        q = O.moduli[limb]
        a = r.integers(0, q, O.N, dtype=np.uint64)
        b = r.integers(0, q, O.N, dtype=np.uint64)
        A, B = O.ntt(limb, a), O.ntt(limb, b)
        prod = np.array([int(x) * int(y) % q for x, y in zip(A, B)], dtype=np.uint64)
        c = O.intt(limb, prod)
        assert [int(x) for x in c] == schoolbook_negacyclic(a, b, q)


@pytest.mark.parametrize("logN", [1, 2, 4, 7, 10])
def test_fast_equals_definition(logN):
    O = helpers.small_oracle(logN)
    r = np.random.default_rng(100 + logN)
    q = O.moduli[0]
    a = r.integers(0, q, O.N, dtype=np.uint64)
    assert (O.ntt(0, a) == O.ntt_naive(0, a)).all()


@pytest.mark.parametrize("logN", [3, 6, 12])
def test_output_order_is_bit_reversed_odd_powers(logN):
    """NTT(X)[k] = psi^(2*brev(k)+1): fixes root, direction and output order."""
    O = helpers.small_oracle(logN)
    for limb in (0, O.L):
        q, psi = O.moduli[limb], O.psi(limb)
        x = np.zeros(O.N, dtype=np.uint64)
        x[1] = 1
        X = O.ntt(limb, x)
        for k in range(O.N):
            assert int(X[k]) == pow(psi, 2 * helpers.brev(k, logN) + 1, q)
        # and a constant polynomial evaluates to itself everywhere
        cst = np.zeros(O.N, dtype=np.uint64)
        cst[0] = 12345
        assert (O.ntt(limb, cst) == 12345).all()


def test_roundtrip_big_ring():
    O = helpers.make_oracle(W.BIG_RING)
    r = np.random.default_rng(5)
    for limb in (0, 23, 24, 31):
        q = O.moduli[limb]
        a = r.integers(0, q, O.N, dtype=np.uint64)
        a[:3] = (0, 1, q - 1)
        A = O.ntt(limb, a)
        assert (A < q).all()
        assert (O.intt(limb, A) == a).all()
        assert (O.ntt(limb, O.intt(limb, a)) == a).all()


def test_linearity_and_shift_big_ring():
    """NTT(X*a)[k] = psi^(2brev(k)+1) * NTT(a)[k] at N = 2^16 (spot indices)."""
    O = helpers.make_oracle(W.BIG_RING)
    r = np.random.default_rng(6)
    limb = 30
    q, psi = O.moduli[limb], O.psi(limb)
    a = r.integers(0, q, O.N, dtype=np.uint64)
    xa = np.roll(a, 1)
    xa[0] = (q - int(a[-1])) % q
    A, XA = O.ntt(limb, a), O.ntt(limb, xa)
    for k in list(range(0, O.N, 4099)) + [O.N - 1]:
        assert int(XA[k]) == int(A[k]) * pow(psi, 2 * helpers.brev(k, 16) + 1, q) % q
