"""Pins for the hoisted key switch: big-integer decryption bound, slot semantics, edge cases."""
import numpy as np
import pytest

from oracle import encoding as E
from tests import helpers
from paper_2604_09975_amd import workload as W


def int_automorph(m, g, N):
    """sigma_g on an integer polynomial (Python ints), independent of the oracle."""
    out = [0] * N
    for j, v in enumerate(m):
        r = g * j % (2 * N)
        if r < N:
            out[r] += v
        else:
            out[r - N] -= v
    return out


def ks_bound(O, level, hw):
    """beta*N*alpha*max(Q_D)*6sigma/P + (K+1)(1+h): worst-case coefficient error of one key switch."""
    beta = -(-level // O.alpha)
    P = 1
    for p in O.p:
        P *= p
    QD = 1
    for j in range(beta):
        d = 1
        for q in O.q[j * O.alpha:min((j + 1) * O.alpha, level)]:
            d *= q
        QD = max(QD, d)
    return beta * O.N * O.alpha * QD * 19 // P + (O.K + 1) * (1 + hw) + 1


def _check_rotations(O, level, steps, seed, scale, hw):
    cl = helpers.Client(O, seed, hamming_weight=hw)
    r = np.random.default_rng(seed)
    z = W.unit_disk_slots(r, O.n)
    ct = cl.encrypt_slots(z, scale, level)
    gel = [O.galois_elt(s) for s in steps]
    keys = [None if g == 1 else cl.galois_key(g) for g in gel]
    out = O.rotate_hoisted(ct, level, gel, keys)
    m_in = O.decrypt_centred(ct, level, cl.s, level)
    bound = ks_bound(O, level, hw)
    Q = 1
    for q in O.q[:level]:
        Q *= q
    for i, (s, g) in enumerate(zip(steps, gel)):
        if g == 1:
            assert (out[i] == ct).all()
            continue
        m_out = O.decrypt_centred(out[i], level, cl.s, level)
        ref = int_automorph(m_in, g, O.N)
        err = max(abs(((a - b + Q // 2) % Q) - Q // 2) for a, b in zip(m_out, ref))
        assert err <= bound, (s, err, bound)
        zz = E.decode(m_out, scale, O.N)
        want = np.conj(z) if s == "conj" else np.roll(z, -s)
        assert np.abs(zz - want).max() < 64 * bound / scale + 1e-6
    return cl, ct, out


def test_toy_ring_rotations_and_identity(toy_oracle):
    O = toy_oracle
    _check_rotations(O, 3, [0, 1, 5, O.n - 1, "conj", O.n, 16, -3], seed=11, scale=2.0**30, hw=64)


def test_toy_ring_lower_level(toy_oracle):
    _check_rotations(toy_oracle, 2, [1, "conj"], seed=12, scale=2.0**30, hw=64)
    _check_rotations(toy_oracle, 1, [7], seed=13, scale=2.0**30, hw=64)


@pytest.mark.parametrize("L,K,dnum,level", [(4, 2, 2, 4), (4, 2, 2, 3), (6, 3, 2, 5), (6, 2, 3, 2)])
def test_multi_limb_digits(L, K, dnum, level):
    O = helpers.small_oracle(6, L=L, K=K, dnum=dnum, qbits=30, pbits=31)
    _check_rotations(O, level, [1, 2, "conj", 0], seed=L * 7 + level, scale=2.0**24, hw=8)


def test_rotate_then_rotate_back(toy_oracle):
    O = toy_oracle
    cl = helpers.Client(O, 21)
    z = W.unit_disk_slots(np.random.default_rng(21), O.n)
    ct = cl.encrypt_slots(z, 2.0**30, 3)
    g1, g2 = O.galois_elt(9), O.galois_elt(O.n - 9)
    a = O.rotate_hoisted(ct, 3, [g1], [cl.galois_key(g1)])[0]
    b = O.rotate_hoisted(a, 3, [g2], [cl.galois_key(g2)])[0]
    # P is only as large as the biggest digit here, so each switch adds ~1e-4 of slot noise
    assert np.abs(cl.decrypt_slots(b, 3, 2.0**30) - z).max() < 2e-3
    assert not (b == ct).all()


def test_hoisted_batch_equals_single_calls(toy_oracle):
    """The shared ModUp is computed once: a batch gives the same bits as one call per element."""
    O = toy_oracle
    cl = helpers.Client(O, 31)
    ct = cl.encrypt_slots(W.unit_disk_slots(np.random.default_rng(31), O.n), 2.0**30, 3)
    gel = [O.galois_elt(s) for s in (1, 2, 3, 4, "conj")]
    keys = [cl.galois_key(g) for g in gel]
    batch = O.rotate_hoisted(ct, 3, gel, keys)
    for i in range(len(gel)):
        assert (O.rotate_hoisted(ct, 3, gel[i:i + 1], keys[i:i + 1])[0] == batch[i]).all()


def test_encrypt_decrypt_roundtrip(toy_oracle):
    O = toy_oracle
    cl = helpers.Client(O, 41)
    z = W.unit_disk_slots(np.random.default_rng(41), O.n)
    ct = cl.encrypt_slots(z, 2.0**30, 3)
    m = E.encode(z, 2.0**30, O.N)
    dec = O.decrypt_centred(ct, 3, cl.s, 3)
    assert max(abs(int(a) - int(b)) for a, b in zip(dec, m)) <= 19      # only the fresh error separates them
    assert (ct[1] < np.array(O.q, dtype=np.uint64)[:, None]).all()
