"""Big-integer closed forms for ModUp, ModDown and rescale."""
import numpy as np
import pytest

from tests import helpers
from paper_2604_09975_amd import workload as W


def _rand_limbs(r, moduli, N):
    return np.stack([r.integers(0, q, N, dtype=np.uint64) for q in moduli])


@pytest.mark.parametrize("L,K,dnum,level", [(3, 1, 3, 3), (4, 2, 2, 4), (4, 2, 2, 3), (6, 3, 2, 5), (6, 2, 3, 6)])
def test_modup_is_c_plus_small_multiple_of_QD(L, K, dnum, level):
    O = helpers.small_oracle(4, L=L, K=K, dnum=dnum, qbits=30, pbits=33)
    r = np.random.default_rng(L * 10 + K)
    c = _rand_limbs(r, O.q[:level], O.N)
    c[:, 0] = 0
    c[:, 1] = [q - 1 for q in O.q[:level]]
    alpha = O.alpha
    beta = -(-level // alpha)
    ext = O.q[:level] + O.p
    for j in range(beta):
        lo, hi = j * alpha, min((j + 1) * alpha, level)
        out = O.modup(level, j, c)
        assert (out[lo:hi] == c[lo:hi]).all()
        for x in range(O.N):
            v, QD = helpers.crt_nonneg(c[lo:hi, x], O.q[lo:hi])
            full, M = helpers.crt_nonneg(out[:, x], ext)
            # the extended value is one integer congruent to out on every limb; find u from one outside limb
            us = set()
            for t, mt in enumerate(ext):
                if lo <= t < hi:
                    continue
                found = [u for u in range(hi - lo) if (v + u * QD) % mt == int(out[t, x])]
                assert found, "no admissible overflow count"
                us.add(found[0])
            assert len(us) == 1 and 0 <= us.pop() < hi - lo


@pytest.mark.parametrize("L,K,dnum,level", [(3, 1, 3, 3), (4, 2, 2, 3), (6, 3, 2, 6)])
def test_moddown_is_floor_division_up_to_K(L, K, dnum, level):
    O = helpers.small_oracle(4, L=L, K=K, dnum=dnum, qbits=30, pbits=33)
    r = np.random.default_rng(L + K)
    ext = O.q[:level] + O.p
    ext_ids = list(range(level)) + [O.L + k for k in range(K)]
    u_coeff = _rand_limbs(r, ext, O.N)
    u_ntt = np.stack([O.ntt(ext_ids[t], u_coeff[t]) for t in range(len(ext))])
    v = O.moddown(level, u_ntt)
    v_coeff = np.stack([O.intt(i, v[i]) for i in range(level)])
    P = 1
    for p in O.p:
        P *= p
    for x in range(O.N):
        big, M = helpers.crt_nonneg(u_coeff[:, x], ext)
        got, Q = helpers.crt_nonneg(v_coeff[:, x], O.q[:level])
        diff = (got - big // P) % Q
        if diff > Q // 2:
            diff -= Q
        assert -K <= diff <= 0


@pytest.mark.parametrize("level", [2, 3, 5])
def test_rescale_is_exact_rounded_division(level):
    O = helpers.small_oracle(4, L=5, K=1, dnum=5, qbits=30, pbits=33)
    r = np.random.default_rng(level)
    coeff = _rand_limbs(r, O.q[:level], O.N)
    coeff = np.stack([coeff, _rand_limbs(r, O.q[:level], O.N)])[None]     # [1][2][level][N]
    ct = np.zeros_like(coeff)
    for comp in range(2):
        for i in range(level):
            ct[0, comp, i] = O.ntt(i, coeff[0, comp, i])
    out = O.rescale(ct, level)
    ql = O.q[level - 1]
    for comp in range(2):
        oc = np.stack([O.intt(i, out[0, comp, i]) for i in range(level - 1)])
        for x in range(O.N):
            big, Q = helpers.crt_nonneg(coeff[0, comp, :, x], O.q[:level])
            if big > Q // 2:
                big -= Q
            # exact nearest integer to big/ql (ql odd: no ties)
            expect = (2 * big + ql) // (2 * ql)
            got, Q1 = helpers.crt_nonneg(oc[:, x], O.q[:level - 1])
            assert (got - expect) % Q1 == 0


def test_rescale_halves_scale_on_real_parameters():
    """At the toy ring: a plaintext at scale q_last*2^20 comes back at scale 2^20."""
    from oracle import encoding as E
    O = helpers.make_oracle(W.TOY_RING)
    r = np.random.default_rng(2)
    z = r.uniform(-1, 1, O.n) + 0j
    ql = O.q[2]
    m = E.encode(z, float(ql) * 2.0**20, O.N)
    ct = np.zeros((1, 2, 3, O.N), dtype=np.uint64)
    ct[0, 0] = O.expand_plain(3, m)          # trivial encryption (c1 = 0)
    out = O.rescale(ct, 3)
    s = np.zeros(O.N, dtype=np.int8)
    zz = E.decode(O.decrypt_centred(out[0], 2, s, 2), 2.0**20, O.N)
    assert np.abs(zz - z).max() < 1e-4
