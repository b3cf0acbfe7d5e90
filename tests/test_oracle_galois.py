"""Pins for automorphisms and the slot encoding (rot = cyclic LEFT shift, Sec. 3.1)."""
import numpy as np
import pytest

from oracle import encoding as E
from tests import helpers


def _centre(res, q):
    return [int(v) if int(v) <= q // 2 else int(v) - q for v in res]


@pytest.mark.parametrize("logN", [3, 4, 6])
def test_encode_fft_equals_direct_sum(logN):
    N = 1 << logN
    r = np.random.default_rng(logN)
    z = r.standard_normal(N // 2) + 1j * r.standard_normal(N // 2)
    a, b = E.encode(z, 2.0**30, N), E.encode_direct(z, 2.0**30, N)
    assert np.abs(a - b).max() <= 1        # two fp64 evaluations may round a tie differently
    assert np.abs(E.decode(a, 2.0**30, N) - E.decode_direct(a, 2.0**30, N)).max() < 1e-9


@pytest.mark.parametrize("logN", [4, 10, 12])
def test_decode_inverts_encode(logN):
    N = 1 << logN
    r = np.random.default_rng(logN)
    z = r.standard_normal(N // 2) + 1j * r.standard_normal(N // 2)
    m = E.encode(z, 2.0**40, N)
    assert np.abs(E.decode(m, 2.0**40, N) - z).max() <= N / 2.0**40


def test_product_of_polynomials_is_slotwise_product():
    O = helpers.small_oracle(6, qbits=50, pbits=52)
    N, q = O.N, O.q[0]
    r = np.random.default_rng(3)
    z1 = r.uniform(-1, 1, N // 2) + 1j * r.uniform(-1, 1, N // 2)
    z2 = r.uniform(-1, 1, N // 2) + 1j * r.uniform(-1, 1, N // 2)
    m1, m2 = E.encode(z1, 2.0**20, N), E.encode(z2, 2.0**20, N)
    A = O.ntt(0, np.array([int(v) % q for v in m1], dtype=np.uint64))
    B = O.ntt(0, np.array([int(v) % q for v in m2], dtype=np.uint64))
    prod = O.intt(0, np.array([int(a) * int(b) % q for a, b in zip(A, B)], dtype=np.uint64))
    zz = E.decode(_centre(prod, q), 2.0**40, N)
    assert np.abs(zz - z1 * z2).max() < 1e-4


@pytest.mark.parametrize("logN", [3, 5, 8])
def test_rotation_is_left_shift_and_conj_is_conjugate(logN):
    O = helpers.small_oracle(logN, qbits=50, pbits=52)
    N, n, q = O.N, O.N // 2, O.q[0]
    r = np.random.default_rng(logN)
    z = r.standard_normal(n) + 1j * r.standard_normal(n)
    m = E.encode(z, 2.0**30, N)
    res = np.array([int(v) % q for v in m], dtype=np.uint64)
    for step in (1, 2, n - 1, -1, n + 3):
        g = O.galois_elt(step)
        zz = E.decode(_centre(O.automorph_coeff(0, g, res), q), 2.0**30, N)
        assert np.abs(zz - np.roll(z, -step)).max() < 1e-6       # (v_r, v_{r+1}, ..., v_0, ...)
    g = O.galois_elt("conj")
    assert g == 2 * N - 1
    zz = E.decode(_centre(O.automorph_coeff(0, g, res), q), 2.0**30, N)
    assert np.abs(zz - np.conj(z)).max() < 1e-6
    assert O.galois_elt(0) == 1 and O.galois_elt(n) == 1          # full turn = identity


@pytest.mark.parametrize("logN", [3, 7, 12])
def test_coefficient_and_ntt_forms_agree(logN):
    O = helpers.small_oracle(logN)
    r = np.random.default_rng(10 + logN)
    for limb in (0, O.L):
        q = O.moduli[limb]
        a = r.integers(0, q, O.N, dtype=np.uint64)
        a[0] = 0
        for step in (1, 3, "conj"):
            g = O.galois_elt(step)
            lhs = O.ntt(limb, O.automorph_coeff(limb, g, a))
            rhs = O.automorph_ntt(g, O.ntt(limb, a))
            assert (lhs == rhs).all()


def test_group_law():
    O = helpers.small_oracle(6)
    r = np.random.default_rng(1)
    q = O.q[0]
    a = r.integers(0, q, O.N, dtype=np.uint64)
    g, h = O.galois_elt(5), O.galois_elt(9)
    gh = g * h % (2 * O.N)
    assert gh == O.galois_elt(14)
    assert (O.automorph_coeff(0, g, O.automorph_coeff(0, h, a)) == O.automorph_coeff(0, gh, a)).all()
    assert (O.automorph_ntt(g, O.automorph_ntt(h, a)) == O.automorph_ntt(gh, a)).all()
    c = O.galois_elt("conj")
    assert (O.automorph_coeff(0, c, O.automorph_coeff(0, c, a)) == a).all()
    assert (O.automorph_ntt(1, a) == a).all()
    # hand-computed: N = 8 would give X -> X^5; here check one monomial: X^3 -> X^(3g mod 2N), sign by wrap
    x3 = np.zeros(O.N, dtype=np.uint64)
    x3[3] = 1
    out = O.automorph_coeff(0, g, x3)
    e = 3 * g % (2 * O.N)
    exp = np.zeros(O.N, dtype=np.uint64)
    exp[e % O.N] = 1 if e < O.N else q - 1
    assert (out == exp).all()
