"""GPU parity over a seeded sweep of small projection shapes: rings 2^10 .. 2^12, random chain lengths, digit counts, prime
sizes (fp64 and Montgomery arithmetic), levels, segment lengths, active-column counts, baby/giant splits, ragged
d_in / d_out, bias on or off, both giant-step orders, real / general / mixed diagonals, and complex-pair
compression (Sec. 3.2) with and without a real last group.  Every output residue is compared with the oracle, before
and after rescale, and the decrypted product with fp64."""
import numpy as np
import pytest
import torch

from oracle import encoding as E
from tests import helpers
from tests.gpu_util import load_keys, make_pair, to_dev, to_host
from tests.test_gpu_matmul import make_real, run_case
from paper_2604_09975_amd import workload as W

pytestmark = pytest.mark.gpu


def _draw(seed):
    r = W.rng(7000 + seed)
    logN = int(r.choice([10, 11, 12]))
    n = 1 << (logN - 1)
    L = int(r.choice([2, 3, 4, 6]))
    dnum = int(r.choice([d for d in (1, 2, 3, 6) if L % d == 0]))
    alpha = L // dnum
    K = alpha + int(r.integers(0, 2))
    qbits = int(r.choice([40, 45, 49, 52]))
    level = int(r.integers(2, L + 1))
    m = int(r.choice([4, 8, 16]))
    C = int(r.choice([c for c in (2, 4, 8, 16, 32) if c <= n // m]))
    N1 = int(r.choice([d for d in (1, 2, 4, 8, 16, 32) if d <= C]))
    d_in, d_out = int(r.integers(1, 3 * C + 1)), int(r.integers(1, 3 * C + 1))
    return dict(logN=logN, L=L, dnum=dnum, K=K, qbits=qbits, pbits=qbits + 6, level=level, m=m, C=C, N1=N1, d_in=d_in,
                d_out=d_out, bias=bool(r.integers(2)), merged=bool(r.integers(2)),
                real=[False, True, "first_upload"][int(r.integers(3))], seed=seed)


@pytest.mark.parametrize("seed", range(48))
def test_projection_sweep(seed):
    c = _draw(seed)
    O = helpers.small_oracle(c["logN"], L=c["L"], K=c["K"], dnum=c["dnum"], qbits=c["qbits"], pbits=c["pbits"])
    _, P = make_pair(O)
    r = W.rng(9000 + seed)
    X = r.uniform(-1, 1, (c["m"], c["d_in"]))
    Wm = r.uniform(-0.5, 0.5, (c["d_in"], c["d_out"]))
    bias = r.uniform(-0.5, 0.5, c["d_out"]) if c["bias"] else None
    Y, ref, _, slots = run_case(O, P, X, Wm, bias, c["m"], c["C"], c["N1"], c["qbits"] - 10, c["level"],
                                100 + seed, hw=16, real=c["real"], merged=c["merged"])
    assert np.abs(Y - ref).max() <= 1e-3, c
    assert np.abs(slots.imag).max() <= 1e-3, c


@pytest.mark.parametrize("seed", range(100, 124))
def test_pair_compression_sweep(seed):
    """Complexified inputs x^(2u) + i x^(2u+1), weights (W_even - i W_odd)/2, one conjugation per output block (odd
    seeds: one per giant-step accumulator, the order Sec. 3.2 displays); when the number of real input groups is odd
    the last complexified group is real and may keep half records."""
    from paper_2604_09975_amd import binding as B
    c = _draw(seed)
    O = helpers.small_oracle(c["logN"], L=c["L"], K=c["K"], dnum=c["dnum"], qbits=c["qbits"], pbits=c["pbits"])
    _, P = make_pair(O)
    N, n, m, C, N1, level = O.N, O.n, c["m"], c["C"], c["N1"], c["level"]
    r = W.rng(9000 + seed)
    X = r.uniform(-1, 1, (m, c["d_in"]))
    Wm = r.uniform(-0.5, 0.5, (c["d_in"], c["d_out"]))
    bias = r.uniform(-0.5, 0.5, c["d_out"])
    G, B_out, N2 = -(-c["d_in"] // C), -(-c["d_out"] // C), C // N1
    U = -(-G // 2)
    cl = helpers.Client(O, 300 + seed, hamming_weight=16)
    sc = 2.0 ** (c["qbits"] - 10)
    mx = E.encode(E.pack_columns_complex(X, n, C), sc, N)
    ct_x = np.stack([cl.encrypt_coeffs(mx[u], level) for u in range(U)])
    diag = E.encode_diagonals_complex(Wm, m, N, C, N1, sc, half=True)
    if G % 2 == 1 and c["real"]:
        diag[:, :, U - 1] = make_real(diag[:, :, U - 1])
    bias_c = np.stack([E.encode(E.bias_slots(bias, m, n, C, b) + 0j, sc, N) for b in range(B_out)])
    baby_np, baby_h = load_keys(P, O, cl, [q * m for q in range(1, N1)])
    giant_np, giant_h = load_keys(P, O, cl, [p * N1 * m for p in range(1, N2)])
    (conj_np,), (conj_h,) = load_keys(P, O, cl, ["conj"])
    w = B.ckks_weights_create(P, level, m, C, U, B_out, N1)
    B.ckks_weights_set_diagonals(w, 0, to_dev(diag.reshape(-1, N)))
    B.ckks_weights_set_bias(w, to_dev(bias_c), int(sc))
    per_acc = seed % 2 == 1
    y_dev, cnt = B.ckks_ctpt_matmul(P, w, to_dev(ct_x), baby_h, giant_h, conj_key=conj_h,
                                    flags=(B.MATMUL_MERGED_GIANT if c["merged"] else 0) |
                                          (B.MATMUL_CONJ_PER_ACC if per_acc else 0))
    y_res = B.ckks_rescale(P, y_dev, level, B_out)
    torch.cuda.synchronize()
    want = O.ctpt_matmul(level, m, U, B_out, N1, N2, diag, bias_c, int(sc), ct_x, baby_np, giant_np,
                         merged=c["merged"], conj_key=conj_np, conj_per_acc=per_acc)
    assert (to_host(y_dev) == want).all(), c
    assert cnt.key_switches >= B_out * (N2 if per_acc else 1)
    got = to_host(y_res)
    assert (got == O.rescale(want, level)).all(), c
    slots = np.stack([cl.decrypt_slots(got[b], level - 1, sc * sc / O.q[level - 1], nlimbs=min(level - 1, 2))
                      for b in range(B_out)])
    assert np.abs(E.unpack_columns(slots.real, m, C, c["d_out"]) - (X @ Wm + bias)).max() <= 1e-3, c
    assert np.abs(slots.imag).max() <= 1e-3, c


@pytest.mark.parametrize("seed", range(200, 232))
def test_key_switch_sweep(seed):
    """Hoisted rotations (random steps with repeats, the identity and conjugation), ctmul + relinearisation and a
    small bank of intra-segment shifts on random chains, levels (1 included) and ring degrees 2^10 .. 2^13."""
    from tests.test_gpu_ctmul import _case as ctmul_case
    from tests.test_gpu_evalops import _psi_bank
    from tests.test_gpu_rotate import _run as rotate_case
    r = W.rng(seed)
    logN = int(r.choice([10, 11, 12, 13]))
    L = int(r.choice([1, 2, 3, 4, 6, 8]))
    dnum = int(r.choice([d for d in (1, 2, 3, 4, 6, 8) if L % d == 0]))
    K = L // dnum + 1          # P exceeds every digit product by a whole prime: the helpers' decode bounds hold
    qbits = int(r.choice([40, 45, 49, 52, 55]))
    level = int(r.integers(1, L + 1))
    O = helpers.small_oracle(logN, L=L, K=K, dnum=dnum, qbits=qbits, pbits=min(qbits + 6, 60))
    _, P = make_pair(O)
    n = O.n
    steps = [int(s) for s in r.integers(0, n, int(r.integers(1, 6)))] + ["conj", 0]
    steps.append(steps[0])                                   # a repeated step
    scale = 2.0 ** (qbits - 4)      # after a mask product and one rescale the scale is still about 2^(qbits - 8)
    rotate_case(O, P, level, steps, seed, scale, hw=16)
    ctmul_case(O, P, level, seed + 1, scale, 16)
    m = int(r.choice([8, 16, 32]))
    _psi_bank(O, P, level, m, [int(t) for t in r.integers(0, m, 3)], seed + 2, scale)
