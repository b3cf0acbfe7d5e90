"""Pins for the projection kernel Y = XW (Sec. 3.2, App. A.2.1)."""
import numpy as np
import pytest

from oracle import encoding as E
from tests import helpers
from tests.test_oracle_keyswitch import int_automorph, ks_bound
from paper_2604_09975_amd import workload as W


def int_negacyclic(a, b, N):
    out = [0] * N
    for i, x in enumerate(a):
        if x == 0:
            continue
        for j, y in enumerate(b):
            k = i + j
            if k < N:
                out[k] += x * y
            else:
                out[k - N] -= x * y
    return out


def run_matmul(O, cl, X, Wm, bias, m, C, N1, sx, sw, level, blocks=None, merged=False):
    N, n = O.N, O.n
    d_in, d_out = Wm.shape
    G, B_out, N2 = -(-d_in // C), -(-d_out // C), C // N1
    xs = E.pack_columns(X, n, C)
    mx = E.encode(xs + 0j, sx, N)
    ct_x = np.stack([cl.encrypt_coeffs(mx[g], level) for g in range(G)])
    diag = E.encode_diagonals(Wm, m, N, C, N1, sw)
    bias_c = None
    if bias is not None:
        bias_c = np.stack([E.encode(E.bias_slots(bias, m, n, C, b) + 0j, sx, N) for b in range(B_out)])
    baby = [cl.galois_key(O.galois_elt(q * m)) for q in range(1, N1)]
    giant = [cl.galois_key(O.galois_elt(p * N1 * m)) for p in range(1, N2)]
    y = O.ctpt_matmul(level, m, G, B_out, N1, N2, diag, bias_c, int(sw), ct_x, baby, giant, merged=merged)
    return dict(ct_x=ct_x, mx=mx, diag=diag, bias_c=bias_c, y=y, G=G, B_out=B_out, N2=N2)


@pytest.mark.parametrize("merged", [False, True])
def test_tiny_ring_against_integer_polynomials(merged):
    """N = 32, m = 2, C = N_seg = 8: every step redone over Z[X]/(X^N+1) with Python ints, no RNS.
    merged: the giant-step variant with one ModDown per output block (same integers up to the switch noise)."""
    O = helpers.small_oracle(5, L=3, K=1, dnum=3, qbits=30, pbits=33)
    N, n, m, C, N1 = O.N, O.n, 2, 8, 4
    r = np.random.default_rng(77)
    X = r.uniform(-1, 1, (m, 16))
    Wm = r.uniform(-1, 1, (16, 13))           # ragged d_out: last block partly empty
    bias = r.uniform(-1, 1, 13)
    sx, sw = 2.0**25, 2.0**20
    hw = 8
    cl = helpers.Client(O, 5, hamming_weight=hw)
    R = run_matmul(O, cl, X, Wm, bias, m, C, N1, sx, sw, 3, merged=merged)
    G, B_out, N2 = R["G"], R["B_out"], R["N2"]
    assert (G, B_out, N2) == (2, 2, 2)
    Q = O.q[0] * O.q[1] * O.q[2]
    ksb = ks_bound(O, 3, hw)
    wmax = int(np.abs(R["diag"]).max())
    bound = G * N1 * N * wmax * (19 + ksb) + N2 * ksb
    mx = [[int(v) for v in R["mx"][g]] for g in range(G)]
    for b in range(B_out):
        total = [0] * N
        for p in range(N2):
            acc = [0] * N
            for g in range(G):
                for q in range(N1):
                    xr = int_automorph(mx[g], O.galois_elt(q * m), N)
                    w = [int(v) for v in R["diag"][b, p, g, q]]
                    acc = [a + c for a, c in zip(acc, int_negacyclic(xr, w, N))]
            rot = int_automorph(acc, O.galois_elt(p * N1 * m), N)
            total = [a + c for a, c in zip(total, rot)]
        total = [a + int(c) * int(sw) for a, c in zip(total, R["bias_c"][b])]
        got = O.decrypt_centred(R["y"][b], 3, cl.s, 3)
        err = max(abs(((a - c + Q // 2) % Q) - Q // 2) for a, c in zip(got, total))
        assert err <= bound
        assert max(abs(v) for v in total) > 64 * bound          # the signal dwarfs the bound: wrong indices fail
    # and the integers decode to X @ W + bias
    Y = X @ Wm + bias
    slots = np.stack([E.decode(O.decrypt_centred(R["y"][b], 3, cl.s, 3), sx * sw, N) for b in range(B_out)])
    assert np.abs(E.unpack_columns(slots.real, m, C, 13) - Y).max() < 1e-3
    assert np.abs(slots.imag).max() < 1e-3


def test_toy_config_matches_fp64_matmul(toy_oracle):
    """Toy CKKS ct-pt matmul: N = 2^12, scale 2^30, 16x64 times 64x64, all 64 rotations, one rescale."""
    O = toy_oracle
    spec = W.TOY_MATMUL
    X, Wm, _ = W.matmul_inputs(spec)
    cl = helpers.Client(O, spec.seed)
    R = run_matmul(O, cl, X, Wm, None, spec.m, spec.C, spec.N1, 2.0**30, 2.0**30, 3)
    assert (R["G"], R["B_out"], R["N2"]) == (1, 1, 1)
    y = O.rescale(R["y"], 3)
    scale = 2.0**60 / O.q[2]
    slots = cl.decrypt_slots(y[0], 2, scale, nlimbs=2)[None]
    Y = E.unpack_columns(slots.real, spec.m, spec.C, 64)
    assert np.abs(Y - X @ Wm).max() <= 1e-3
    # the replicated copy in segments 64..127 holds the same columns
    Y2 = np.stack([slots[0, (64 + c) * 16:(65 + c) * 16].real for c in range(64)], axis=1)
    assert np.abs(Y2 - X @ Wm).max() <= 1e-3


def test_merged_giant_step_differs_in_bits_but_not_in_value():
    O = helpers.small_oracle(8, L=3, K=1, dnum=3, qbits=40, pbits=42)
    m, C, N1 = 4, 16, 2
    r = np.random.default_rng(10)
    X, Wm = r.uniform(-1, 1, (m, 40)), r.uniform(-0.5, 0.5, (40, 20))
    outs = []
    for merged in (False, True):
        cl = helpers.Client(O, 20, hamming_weight=16)
        R = run_matmul(O, cl, X, Wm, None, m, C, N1, 2.0**30, 2.0**30, 3, merged=merged)
        y = O.rescale(R["y"], 3)
        slots = np.stack([cl.decrypt_slots(y[b], 2, 2.0**60 / O.q[2], nlimbs=2) for b in range(R["B_out"])])
        assert np.abs(E.unpack_columns(slots.real, m, C, 20) - X @ Wm).max() < 1e-3
        outs.append(R["y"])
    assert not (outs[0] == outs[1]).all()           # ModDown is not linear: a different, equally valid ciphertext
    O1 = helpers.small_oracle(8, L=3, K=1, dnum=3, qbits=40, pbits=42)
    cl = helpers.Client(O1, 20, hamming_weight=16)
    R1 = run_matmul(O1, cl, X, Wm, None, m, C, 16, 2.0**30, 2.0**30, 3, merged=True)      # N2 = 1: nothing to merge
    cl = helpers.Client(O1, 20, hamming_weight=16)
    R2 = run_matmul(O1, cl, X, Wm, None, m, C, 16, 2.0**30, 2.0**30, 3, merged=False)
    assert (R1["y"] == R2["y"]).all()


@pytest.mark.parametrize("N1", [1, 4, 16])
def test_bsgs_split_does_not_change_the_result(N1):
    O = helpers.small_oracle(8, L=3, K=1, dnum=3, qbits=40, pbits=42)
    m, C = 4, 16                                   # n = 128, N_seg = 32: two periods of C
    r = np.random.default_rng(9)
    X = r.uniform(-1, 1, (m, 40))                  # ragged d_in: G = 3, last group partly empty
    Wm = r.uniform(-0.5, 0.5, (40, 20))
    bias = r.uniform(-0.5, 0.5, 20)
    cl = helpers.Client(O, 19, hamming_weight=16)
    R = run_matmul(O, cl, X, Wm, bias, m, C, N1, 2.0**30, 2.0**30, 3)
    y = O.rescale(R["y"], 3)
    scale = 2.0**60 / O.q[2]
    slots = np.stack([cl.decrypt_slots(y[b], 2, scale, nlimbs=2) for b in range(R["B_out"])])
    assert np.abs(E.unpack_columns(slots.real, m, C, 20) - (X @ Wm + bias)).max() < 1e-3


def test_block_subset_equals_full_run(toy_oracle):
    O = helpers.small_oracle(6, L=3, K=1, dnum=3, qbits=40, pbits=42)
    m, C, N1 = 2, 16, 4
    r = np.random.default_rng(3)
    X, Wm = r.uniform(-1, 1, (m, 16)), r.uniform(-1, 1, (16, 48))
    cl = helpers.Client(O, 23, hamming_weight=8)
    R = run_matmul(O, cl, X, Wm, None, m, C, N1, 2.0**30, 2.0**30, 3)
    baby = [helpers.Client(O, 23, 8)]  # fresh client with the same seed reproduces the same keys
    cl2 = baby[0]
    mx = E.encode(E.pack_columns(X, O.n, C) + 0j, 2.0**30, O.N)
    ct_x = np.stack([cl2.encrypt_coeffs(mx[0], 3)])
    bk = [cl2.galois_key(O.galois_elt(q * m)) for q in range(1, N1)]
    gk = [cl2.galois_key(O.galois_elt(p * N1 * m)) for p in range(1, C // N1)]
    part = O.ctpt_matmul(3, m, 1, 3, N1, C // N1, R["diag"], None, 0, ct_x, bk, gk, b_first=1, b_count=1)
    assert (part[1] == R["y"][1]).all() and (part[0] == 0).all() and (part[2] == 0).all()
