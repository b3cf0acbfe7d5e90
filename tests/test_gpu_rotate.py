"""GPU parity: hoisted rotations / conjugation against the oracle, bit for bit."""
import numpy as np
import pytest
import torch

from tests import helpers
from tests.gpu_util import load_keys, make_pair, to_dev, to_host
from paper_2604_09975_amd import workload as W

pytestmark = pytest.mark.gpu


def _B():
    from paper_2604_09975_amd import binding as B
    return B


def _run(O, P, level, steps, seed, scale, hw=64):
    B = _B()
    cl = helpers.Client(O, seed, hamming_weight=hw)
    z = W.unit_disk_slots(W.rng(seed), O.n)
    ct = cl.encrypt_slots(z, scale, level)
    np_keys, handles = load_keys(P, O, cl, steps)
    gel = [O.galois_elt(s) for s in steps]
    want = O.rotate_hoisted(ct, level, gel, np_keys)
    got = to_host(B.ckks_rotate_hoisted(P, to_dev(ct), level, steps, handles))
    torch.cuda.synchronize()
    for i, s in enumerate(steps):
        assert (got[i] == want[i]).all(), f"step {s}"
    return cl, z, ct, got


def test_toy_ring_all_kinds_of_steps():
    O, P = make_pair(W.TOY_RING)
    cl, z, ct, got = _run(O, P, 3, [0, 1, 5, O.n - 1, "conj", O.n, 16, -3], 11, 2.0**30)
    assert (got[0] == ct).all() and (got[5] == ct).all()
    zz = cl.decrypt_slots(got[1], 3, 2.0**30)
    assert np.abs(zz - np.roll(z, -1)).max() < 2e-3


@pytest.mark.parametrize("level", [1, 2])
def test_toy_ring_lower_levels(level):
    O, P = make_pair(W.TOY_RING)
    _run(O, P, level, [1, "conj", 7], 12 + level, 2.0**30)


@pytest.mark.parametrize("L,K,dnum,level", [(4, 2, 2, 4), (4, 2, 2, 3), (6, 3, 2, 5), (6, 2, 3, 2), (6, 3, 1, 6), (12, 4, 1, 12), (12, 12, 1, 11), (16, 16, 1, 16)])
def test_multi_limb_digits_and_partial_last_digit(L, K, dnum, level):
    O = helpers.small_oracle(10, L=L, K=K, dnum=dnum, qbits=40, pbits=45)
    _, P = make_pair(O)
    _run(O, P, level, [1, 2, "conj", 0, 33], L * 7 + level, 2.0**30, hw=16)


@pytest.mark.parametrize("logN", [11, 13, 15, 17])
def test_other_ring_degrees(logN):
    """Key switching on the generic transform path: degrees between and beyond the two tuned ones, up to the
    largest admitted (2^17)."""
    O = helpers.small_oracle(logN, L=4, K=2, dnum=2, qbits=45, pbits=50)
    _, P = make_pair(O)
    _run(O, P, 3, [1, "conj", (1 << (logN - 1)) - 1], 90 + logN, 2.0**36, hw=32)


def test_largest_primes_and_widest_digits():
    """16-limb digit and 16 special primes at the largest prime size the library admits for them (16 lazy
    products must stay below 2^64 times the modulus: primes below 2^60), and the refusal one bit above."""
    B = _B()
    O = helpers.small_oracle(10, L=16, K=16, dnum=1, qbits=58, pbits=59)
    _, P = make_pair(O)
    _run(O, P, 16, [1, "conj"], 5, 2.0**40, hw=16)
    O = helpers.small_oracle(10, L=4, K=16, dnum=2, qbits=58, pbits=59)
    _, P = make_pair(O)
    _run(O, P, 3, [3], 6, 2.0**40, hw=16)
    import oracle
    with pytest.raises(B.CkksError) as err:
        B.ckks_params_create(10, oracle.find_primes(60, 10, 16), oracle.find_primes(61, 10, 16), 1)
    assert err.value.code == -1
    # 61-bit primes are fine with narrow digits
    O = helpers.small_oracle(10, L=4, K=2, dnum=2, qbits=60, pbits=61)
    _, P = make_pair(O)
    _run(O, P, 4, [2], 7, 2.0**40, hw=16)


def test_more_steps_than_one_batch():
    """40 key switches: more than the library keeps in flight at once (32)."""
    O, P = make_pair(W.TOY_RING)
    _run(O, P, 3, list(range(1, 40)) + ["conj"], 17, 2.0**30)


def test_full_size_hoisted_batch():
    """N = 2^16, 24 + 8 limbs, dnum = 3: the 26 listed rotations, conjugation and the full turn 2^15
    (identity) from one fresh ciphertext, every output residue compared."""
    O, P = make_pair(W.BIG_RING)
    steps = list(W.HOISTED_STEPS)
    cl, z, ct, got = _run(O, P, 24, steps, W.HOISTED_SEED, 2.0**40)
    assert (got[steps.index(1 << 15)] == ct).all()
    for s in (1, 1 << 14, "conj"):
        zz = cl.decrypt_slots(got[steps.index(s)], 24, 2.0**40)
        want = np.conj(z) if s == "conj" else np.roll(z, -s)
        # worst-case coefficient error of one switch here is (K+1)(1+h) = 585 (the P-part is negligible);
        # a slot sums N coefficients
        assert np.abs(zz - want).max() < 585 * O.N / 2.0**40


@pytest.mark.parametrize("level", [1, 7, 8, 9, 16, 17, 23])
def test_full_ring_lower_levels(level):
    """N = 2^16 below the full level: one limb, a partial first digit, exactly one digit, one digit and one limb,
    two digits, two and one limb, all but the last limb: the kernels that run the base conversions between the
    column passes see every digit shape."""
    O, P = make_pair(W.BIG_RING)
    _run(O, P, level, [1, 300, "conj"], 900 + level, 2.0**40)


def test_rotate_errors():
    B = _B()
    O, P = make_pair(W.TOY_RING)
    cl = helpers.Client(O, 5)
    ct = to_dev(cl.encrypt_slots(W.unit_disk_slots(W.rng(5), O.n), 2.0**30, 3))
    _, (k1,) = load_keys(P, O, cl, [1])
    with pytest.raises(B.CkksError) as e:
        B.ckks_rotate_hoisted(P, ct, 3, [1], [None])
    assert e.value.code == -3                                   # missing key
    with pytest.raises(B.CkksError) as e:
        B.ckks_rotate_hoisted(P, ct, 3, [2], [k1])
    assert e.value.code == -1                                   # key of another element
    for bad_level in (0, 4):                                    # level 0 and level > L
        rc = B.lib.ckks_rotate_hoisted(P.h, ct.data_ptr(), bad_level, None, 0, None, None, None)
        assert rc == -2
    out = B.ckks_rotate_hoisted(P, ct, 3, [], [])               # no steps: nothing to do
    assert out.numel() == 0
