"""Pins for add / ptmul / ModSwitchToNext and the restricted rotation RotFirst (Table 1, Sec. 5.4, App. A.1)."""
import numpy as np
import pytest

from oracle import encoding as E
from tests import helpers
from paper_2604_09975_amd import workload as W


def test_add_ptmul_modswitch(toy_oracle):
    O = toy_oracle
    cl = helpers.Client(O, 61)
    r = np.random.default_rng(61)
    za, zb = W.unit_disk_slots(r, O.n), W.unit_disk_slots(r, O.n)
    ca, cb = cl.encrypt_slots(za, 2.0**30, 3), cl.encrypt_slots(zb, 2.0**30, 3)
    s = cl.decrypt_slots(O.add(ca, cb, 3), 3, 2.0**30)
    assert np.abs(s - (za + zb)).max() < 1e-6
    pt = O.expand_plain(3, E.encode(zb, 2.0**30, O.N))
    prod = O.rescale(O.ptmul(ca, 3, pt)[None], 3)[0]
    assert np.abs(cl.decrypt_slots(prod, 2, 2.0**60 / O.q[2], nlimbs=2) - za * zb).max() < 1e-5
    # dropping a prime leaves value and scale alone, and commutes with decryption on the remaining limbs
    low = O.mod_switch(ca[None], 3)[0]
    assert (low == ca[:, :2]).all()
    assert np.abs(cl.decrypt_slots(low, 2, 2.0**30, nlimbs=2) - za).max() < 1e-6


@pytest.mark.parametrize("L,tau", [(96, 16), (96, 0), (64, 63), (128, 5), (128, 133)])
def test_rot_first_is_a_cyclic_shift_of_the_first_L_slots(L, tau):
    """n = 128 slots; slots L..n-1 hold zeros and stay zero."""
    O = helpers.small_oracle(8, L=3, K=1, dnum=3, qbits=40, pbits=42)
    n = O.n
    cl = helpers.Client(O, 71, hamming_weight=16)
    r = np.random.default_rng(L + tau)
    z = np.zeros(n)
    z[:L] = r.uniform(-1, 1, L)
    ct = cl.encrypt_slots(z + 0j, 2.0**30, 3)
    a, b, steps = E.rot_first_masks(n, L, tau)
    gel = [O.galois_elt(s) for s in steps]
    keys = [None if g == 1 else cl.galois_key(g) for g in gel]
    ma = O.expand_plain(3, E.encode(a + 0j, 2.0**30, O.N))
    mb = O.expand_plain(3, E.encode(b + 0j, 2.0**30, O.N))
    out = O.rescale(O.rot_first(ct, 3, gel, keys, ma, mb)[None], 3)[0]
    got = cl.decrypt_slots(out, 2, 2.0**60 / O.q[2], nlimbs=2)
    want = np.zeros(n)
    want[:L] = np.roll(z[:L], -(tau % L))
    assert np.abs(got - want).max() < 1e-3


def test_restricted_segment_shift_equals_plain_rot_when_all_segments_are_active():
    """Phi_C^Delta = RotFirst_{Cm}(Delta*m); with C = N_seg it is the plain rotation by Delta*m (Alg. 1 of App. A.1)."""
    n, m = 128, 4
    a, b, steps = E.rot_first_masks(n, n, 3 * m)
    assert steps == (3 * m, (3 * m - n) % n) and steps[0] == steps[1]
    assert (a + b == 1).all()


@pytest.mark.parametrize("m,ts", [(16, [1, 5, 15]), (4, [0, 3]), (128, [64])])
def test_psi_bank_is_the_intra_segment_shift(m, ts):
    """Bank of Psi^t from one input (Sec. 3.1, App. A.1): slot s*m + r of Psi^t(x) holds x[s*m + (r+t) mod m];
    the bank equals the shifts made one by one (hoisting shares only the decomposition)."""
    O = helpers.small_oracle(8, L=3, K=1, dnum=3, qbits=40, pbits=42)
    n = O.n
    cl = helpers.Client(O, 81, hamming_weight=16)
    r = np.random.default_rng(m)
    z = r.uniform(-1, 1, n) + 1j * r.uniform(-1, 1, n)
    ct = cl.encrypt_slots(z, 2.0**30, 3)
    gel, keys, masks = [], [], []
    cache = {}
    for t in ts:
        h, u, steps = E.psi_masks(n, m, t)
        assert ((h + u) == 1).all()
        g = [O.galois_elt(s) for s in steps]
        for x in g:
            if x != 1 and x not in cache:
                cache[x] = cl.galois_key(x)
        gel.append(g)
        keys.append([cache.get(x) for x in g])
        masks.append([O.expand_plain(3, E.encode(h + 0j, 2.0**30, O.N)), O.expand_plain(3, E.encode(u + 0j, 2.0**30, O.N))])
    masks = np.array(masks)
    bank = O.shift_bank(ct, 3, gel, keys, masks)
    for i, t in enumerate(ts):
        one = O.rot_first(ct, 3, gel[i], keys[i], masks[i, 0], masks[i, 1])
        assert (bank[i] == one).all()
        out = O.rescale(bank[i][None], 3)[0]
        got = cl.decrypt_slots(out, 2, 2.0**60 / O.q[2], nlimbs=2)
        assert np.abs(got - E.psi_shift(z, m, t)).max() < 1e-3
    # composing the definition: Psi^t then Psi^(m-t) is the identity
    assert np.allclose(E.psi_shift(E.psi_shift(z, m, ts[0]), m, m - ts[0]), z)
