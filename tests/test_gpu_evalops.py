"""GPU parity: add, ptmul, ModSwitchToNext and RotFirst (Table 1, Sec. 5.4, App. A.1) against the oracle, bit for bit."""
import numpy as np
import pytest
import torch

from oracle import encoding as E
from tests import helpers
from tests.gpu_util import make_pair, to_dev, to_host
from paper_2604_09975_amd import workload as W

pytestmark = pytest.mark.gpu


def _plain(O, P, B, z, scale, level):
    coef = E.encode(z + 0j, scale, O.N)
    got = to_host(B.ckks_plain_expand(P, level, to_dev(coef[None])))[0]
    want = O.expand_plain(level, coef)
    assert (got == want).all()
    return want


def _elementwise(O, P, level, seed, scale):
    from paper_2604_09975_amd import binding as B
    cl = helpers.Client(O, seed, hamming_weight=16)
    r = W.rng(seed)
    cts = np.stack([cl.encrypt_slots(W.unit_disk_slots(r, O.n), scale, level) for _ in range(3)])
    got = to_host(B.ckks_add(P, to_dev(cts[:2]), to_dev(cts[1:]), level, 2))
    assert (got == O.add(cts[:2], cts[1:], level)).all()
    pt = _plain(O, P, B, r.uniform(-1, 1, O.n), scale, level)
    got = to_host(B.ckks_ptmul(P, to_dev(cts[0]), level, to_dev(pt)))
    assert (got == O.ptmul(cts[0], level, pt)).all()
    if level > 1:
        got = to_host(B.ckks_mod_switch_to_next(P, to_dev(cts), level, 3))
        assert (got == O.mod_switch(cts, level)).all()


@pytest.mark.parametrize("level", [3, 1])
def test_elementwise_toy(level):
    O, P = make_pair(W.TOY_RING)
    _elementwise(O, P, level, 30 + level, 2.0**30)


def test_elementwise_wide_primes():
    O = helpers.small_oracle(10, L=6, K=3, dnum=2, qbits=52, pbits=55)
    _, P = make_pair(O)
    _elementwise(O, P, 5, 35, 2.0**40)


def test_elementwise_full_ring():
    O, P = make_pair(W.BIG_RING)
    _elementwise(O, P, 24, 36, 2.0**40)


def _rot_first(O, P, level, L, tau, seed, scale, hw=16, check=True):
    from paper_2604_09975_amd import binding as B
    from paper_2604_09975_amd import client as CL
    cl = helpers.Client(O, seed, hamming_weight=hw)
    r = W.rng(seed)
    z = np.zeros(O.n)
    z[:L] = r.uniform(-1, 1, L)
    ct = cl.encrypt_slots(z + 0j, scale, level)
    a, b, steps = E.rot_first_masks(O.n, L, tau)
    a2, b2, steps2 = CL.rot_first_masks(O.n, L, tau)
    assert (a == a2).all() and (b == b2).all() and steps == steps2
    gel = [O.galois_elt(s) for s in steps]
    keys = [None if g == 1 else cl.galois_key(g) for g in gel]
    ma, mb = _plain(O, P, B, a, scale, level), _plain(O, P, B, b, scale, level)
    want = O.rot_first(ct, level, gel, keys, ma, mb)
    hk = [None if k is None else B.ckks_galois_key_load(P, g, to_dev(k)) for g, k in zip(gel, keys)]
    got = to_host(B.ckks_rot_first(P, to_dev(ct), level, L, tau, hk[0], hk[1], to_dev(ma), to_dev(mb)))
    assert (got == want).all()
    if check and level > 1:
        out = to_host(B.ckks_rescale(P, to_dev(got[None]), level, 1))[0]
        zz = cl.decrypt_slots(out, level - 1, scale * scale / O.q[level - 1], nlimbs=min(level - 1, 2))
        ref = np.zeros(O.n)
        ref[:L] = np.roll(z[:L], -(tau % L))
        assert np.abs(zz - ref).max() < 2e-3


@pytest.mark.parametrize("L,tau", [(1024, 16), (1024, 0), (2048, 7), (96, 95), (1024, 1024 + 48)])
def test_rot_first_toy(L, tau):
    O, P = make_pair(W.TOY_RING)
    _rot_first(O, P, 3, L, tau, 40 + tau % 7, 2.0**30, hw=64)


def test_rot_first_generic_path():
    O = helpers.small_oracle(10, L=4, K=2, dnum=2, qbits=40, pbits=45)
    _, P = make_pair(O)
    _rot_first(O, P, 3, 320, 64, 47, 2.0**30)


def test_rot_first_full_ring_restricted_segment_shift():
    """Phi_C^Delta on the BERT layout: m = 128, C = 192 of N_seg = 256 segments active, shift by 5 segments."""
    O, P = make_pair(W.BIG_RING)
    _rot_first(O, P, 24, 192 * 128, 5 * 128, 48, 2.0**40, hw=64)


def test_error_paths():
    from paper_2604_09975_amd import binding as B
    O, P = make_pair(W.TOY_RING)
    ct = torch.zeros((2, 3, O.N), dtype=torch.int64, device="cuda")
    pt = torch.zeros((3, O.N), dtype=torch.int64, device="cuda")
    out = torch.zeros_like(ct)
    p = lambda t: t.data_ptr()
    assert B.lib.ckks_add(P.h, p(ct), p(ct), 4, 1, p(out), None) == -2
    assert B.lib.ckks_add(P.h, None, p(ct), 3, 1, p(out), None) == -1
    assert B.lib.ckks_add(P.h, None, None, 3, 0, None, None) == 0
    assert B.lib.ckks_ptmul(P.h, p(ct), 0, p(pt), p(out), None) == -2
    assert B.lib.ckks_mod_switch_to_next(P.h, p(ct), 1, 1, p(out), None) == -2
    assert B.lib.ckks_rot_first(P.h, p(ct), 3, 0, 1, None, None, p(pt), p(pt), p(out), None) == -1
    assert B.lib.ckks_rot_first(P.h, p(ct), 3, O.n + 1, 1, None, None, p(pt), p(pt), p(out), None) == -1
    assert B.lib.ckks_rot_first(P.h, p(ct), 3, 64, 1, None, None, p(pt), p(pt), p(out), None) == -3
    assert B.lib.ckks_plain_expand(P.h, 4, p(ct), 1, p(out), None) == -2


def _psi_bank(O, P, level, m, ts, seed, scale, hw=16):
    """Bank of Psi^t, t in ts, against the oracle's bank bit for bit and against the definition of the shift."""
    from paper_2604_09975_amd import binding as B
    from paper_2604_09975_amd import client as CL
    cl = helpers.Client(O, seed, hamming_weight=hw)
    r = W.rng(seed)
    z = W.unit_disk_slots(r, O.n)
    ct = cl.encrypt_slots(z, scale, level)
    gel, keys, masks, steps_flat, cache = [], [], [], [], {}
    for t in ts:
        h, u, steps = E.psi_masks(O.n, m, t)
        h2, u2, steps2 = CL.psi_masks(O.n, m, t)
        assert (h == h2).all() and (u == u2).all() and steps == steps2
        g = [O.galois_elt(s) for s in steps]
        for x in g:
            if x != 1 and x not in cache:
                k = cl.galois_key(x)
                cache[x] = (k, B.ckks_galois_key_load(P, x, to_dev(k)))
        gel.append(g)
        keys.append([cache[x] if x != 1 else (None, None) for x in g])
        masks.append([_plain(O, P, B, h, scale, level), _plain(O, P, B, u, scale, level)])
        steps_flat += list(steps)
    masks = np.array(masks)
    want = O.shift_bank(ct, level, gel, [[k[0] for k in pair] for pair in keys], masks)
    got = to_host(B.ckks_shift_bank(P, to_dev(ct), level, steps_flat, [k[1] for pair in keys for k in pair],
                                    to_dev(masks)))
    assert (got == want).all()
    if level > 1:
        out = to_host(B.ckks_rescale(P, to_dev(got), level, len(ts)))
        for i, t in enumerate(ts):
            zz = cl.decrypt_slots(out[i], level - 1, scale * scale / O.q[level - 1], nlimbs=min(level - 1, 2))
            assert np.abs(zz - E.psi_shift(z, m, t)).max() < 2e-3


def test_psi_bank_toy():
    O, P = make_pair(W.TOY_RING)
    _psi_bank(O, P, 3, 16, [1, 2, 3, 5, 8, 15], 51, 2.0**30, hw=64)


def test_psi_bank_more_outputs_than_one_batch_and_identity_terms():
    """19 outputs = 38 rotations (two batches of key switches); t = 0 has an identity first term."""
    O = helpers.small_oracle(10, L=4, K=2, dnum=2, qbits=40, pbits=45)
    _, P = make_pair(O)
    _psi_bank(O, P, 4, 32, list(range(0, 19)), 52, 2.0**30)


def test_psi_bank_full_ring():
    """m = 128 (the BERT / GPT-2 sequence length): Psi^1, Psi^64 (the half-segment shift of the value kernel) and
    Psi^127 from one ciphertext at N = 2^16, level 24."""
    O, P = make_pair(W.BIG_RING)
    _psi_bank(O, P, 24, 128, [1, 64, 127], 53, 2.0**40, hw=64)


def test_shift_bank_errors():
    from paper_2604_09975_amd import binding as B
    O, P = make_pair(W.TOY_RING)
    ct = torch.zeros((2, 3, O.N), dtype=torch.int64, device="cuda")
    masks = torch.zeros((1, 2, 3, O.N), dtype=torch.int64, device="cuda")
    with pytest.raises(B.CkksError) as err:
        B.ckks_shift_bank(P, ct, 3, [1, 0], [None, None], masks)
    assert err.value.code == -3
    cl = helpers.Client(O, 8)
    k2 = B.ckks_galois_key_load(P, O.galois_elt(2), to_dev(cl.galois_key(O.galois_elt(2))))
    with pytest.raises(B.CkksError) as err:
        B.ckks_shift_bank(P, ct, 3, [1, 0], [k2, None], masks)
    assert err.value.code == -1
    out = B.ckks_shift_bank(P, ct, 3, [0, 0], [None, None], masks)           # identity terms need no keys
    assert int(out.abs().sum()) == 0
    assert B.lib.ckks_shift_bank(P.h, ct.data_ptr(), 4, 0, None, None, None, None, None) == -2
    assert B.lib.ckks_shift_bank(P.h, ct.data_ptr(), 3, 0, None, None, None, None, None) == 0


def test_probe_kernels_compute_what_they_time():
    """The ceiling probes: the product chains end in x0 * psi^iters mod q (all three arithmetics, checked against
    Python integers), the copy kernel copies, the write kernel writes every word; bad arguments are refused."""
    from paper_2604_09975_amd import binding as B
    O, P = make_pair(W.BIG_RING)
    lanes, iters = 512, 37
    for kind, limb in ((B.PROBE_FP64, 0), (B.PROBE_FP64, 23), (B.PROBE_INT64, 5), (B.PROBE_INT64, 24 + 7),
                       (B.PROBE_INT64_LAZY, 3), (B.PROBE_INT64_LAZY, 24), (B.PROBE_INT64_LAZY, 24 + 7)):
        q = int(O.moduli[limb])
        psi = B.ckks_params_root(P, limb)
        assert pow(psi, 2 * O.N, q) == 1 and pow(psi, O.N, q) == q - 1
        f = pow(psi, iters, q)
        got = to_host(B.ckks_probe_mulmod(P, limb, kind, lanes, iters))
        for t in (0, 1, 255, 256, 511):
            want = 0
            for c in range(4):
                want ^= ((4 * t + c + 1) % (1 << 20)) * f % q
            assert int(got[t]) == want, (kind, limb, t)
    src = torch.arange(1 << 16, dtype=torch.int64, device="cuda") * 3 + 1
    dst = torch.zeros_like(src)
    B.ckks_probe_stream(dst, src, B.PROBE_COPY)
    assert bool((dst == src).all())
    B.ckks_probe_stream(dst, None, B.PROBE_WRITE)
    d = dst.cpu().numpy().view(np.uint64).reshape(-1, 2)
    assert (d[:, 0] == np.arange(1 << 15, dtype=np.uint64)).all() and (d[:, 1] == ~np.arange(1 << 15, dtype=np.uint64)).all()
    before = dst.clone()
    B.ckks_probe_stream(dst, src, B.PROBE_READ)
    assert bool((dst == before).all())
    with pytest.raises(B.CkksError):
        B.ckks_probe_mulmod(P, 24, B.PROBE_FP64, lanes, iters)       # 60-bit prime: no fp64 product
    with pytest.raises(B.CkksError):
        B.ckks_probe_mulmod(P, 0, B.PROBE_INT64, 100, iters)
    with pytest.raises(B.CkksError):
        B.ckks_probe_stream(dst, src, 3)
