"""Pins for ctmul + relinearisation (Table 1)."""
import numpy as np
import pytest

from oracle import encoding as E
from tests import helpers
from tests.test_oracle_keyswitch import ks_bound
from tests.test_oracle_matmul import int_negacyclic
from paper_2604_09975_amd import workload as W


def test_tiny_ring_product_against_integer_polynomials():
    """N = 32: decrypt(ctmul) equals the product of the two decrypted polynomials over Z[X]/(X^N+1) up to
    the relinearisation noise (the fresh errors are part of the decrypted inputs, so they cancel)."""
    O = helpers.small_oracle(5, L=3, K=1, dnum=3, qbits=30, pbits=33)
    N, hw = O.N, 8
    cl = helpers.Client(O, 3, hamming_weight=hw)
    r = np.random.default_rng(3)
    za, zb = W.unit_disk_slots(r, O.n), W.unit_disk_slots(r, O.n)
    ca, cb = cl.encrypt_slots(za, 2.0**22, 3), cl.encrypt_slots(zb, 2.0**22, 3)
    rk = cl.relin_key()
    out = O.ctmul(ca, cb, 3, rk)
    Q = O.q[0] * O.q[1] * O.q[2]
    ma, mb = O.decrypt_centred(ca, 3, cl.s, 3), O.decrypt_centred(cb, 3, cl.s, 3)
    want = int_negacyclic(ma, mb, N)
    got = O.decrypt_centred(out, 3, cl.s, 3)
    err = max(abs(((a - b + Q // 2) % Q) - Q // 2) for a, b in zip(got, want))
    assert err <= ks_bound(O, 3, hw)
    assert max(abs(v) for v in want) > 1000 * ks_bound(O, 3, hw)
    # commutes
    assert (O.ctmul(cb, ca, 3, rk) == out).all()


@pytest.mark.parametrize("level", [3, 2])
def test_toy_ring_slotwise_product(toy_oracle, level):
    O = toy_oracle
    cl = helpers.Client(O, 51)
    r = np.random.default_rng(51)
    za, zb = W.unit_disk_slots(r, O.n), W.unit_disk_slots(r, O.n)
    ca, cb = cl.encrypt_slots(za, 2.0**30, level), cl.encrypt_slots(zb, 2.0**30, level)
    out = O.rescale(O.ctmul(ca, cb, level, cl.relin_key())[None], level)[0]
    zz = cl.decrypt_slots(out, level - 1, 2.0**60 / O.q[level - 1], nlimbs=min(level - 1, 2))
    assert np.abs(zz - za * zb).max() < 2e-3


def test_relin_key_decrypts_to_P_times_s_squared():
    """b_j + a_j*s = e_j + P*T_j*s^2 on every limb: the key material itself, checked with Python ints."""
    O = helpers.small_oracle(4, L=4, K=2, dnum=2, qbits=30, pbits=31)
    cl = helpers.Client(O, 9, hamming_weight=4)
    key = cl.relin_key()
    s = [int(v) for v in cl.s]
    s2 = int_negacyclic(s, s, O.N)
    P = O.p[0] * O.p[1]
    W_ = O.L + O.K
    for j in range(O.dnum):
        for t in range(W_):
            q = O.moduli[t]
            b = O.intt(t, key[j, 0, t])
            a = O.intt(t, key[j, 1, t])
            a_s = int_negacyclic([int(v) for v in a], s, O.N)
            f = P % q if (t < O.L and t // O.alpha == j) else 0
            for x in range(O.N):
                e = (int(b[x]) + a_s[x] - f * s2[x]) % q
                e = e - q if e > q // 2 else e
                assert abs(e) <= 19
