"""Pins for complex-pair compression, decomplexification and the fused QK projection (Sec. 3.2, App. A.2)."""
import numpy as np
import pytest

from oracle import encoding as E
from tests import helpers
from tests.test_oracle_keyswitch import int_automorph, ks_bound
from tests.test_oracle_matmul import int_negacyclic


def run_complex(O, cl, X, Wm, bias, m, C, N1, sx, sw, level, per_acc=False):
    """Complexified inputs, halved complex weights, y + conj(y) per output block (per_acc: the real part of
    every giant-step accumulator taken before the fold, the order in which Sec. 3.2 writes it)."""
    N, n = O.N, O.n
    d_in, d_out = Wm.shape
    G, B_out, N2 = -(-d_in // C), -(-d_out // C), C // N1
    U = -(-G // 2)
    mx = E.encode(E.pack_columns_complex(X, n, C), sx, N)
    ct_x = np.stack([cl.encrypt_coeffs(mx[u], level) for u in range(U)])
    diag = E.encode_diagonals_complex(Wm, m, N, C, N1, sw, half=True)
    bias_c = None
    if bias is not None:
        bias_c = np.stack([E.encode(E.bias_slots(bias, m, n, C, b) + 0j, sx, N) for b in range(B_out)])
    baby = [cl.galois_key(O.galois_elt(q * m)) for q in range(1, N1)]
    giant = [cl.galois_key(O.galois_elt(p * N1 * m)) for p in range(1, N2)]
    conj = cl.galois_key(O.galois_elt("conj"))
    y = O.ctpt_matmul(level, m, U, B_out, N1, N2, diag, bias_c, int(sw), ct_x, baby, giant, conj_key=conj,
                      conj_per_acc=per_acc)
    return dict(mx=mx, diag=diag, bias_c=bias_c, y=y, U=U, B_out=B_out, N2=N2, ct_x=ct_x, baby=baby, giant=giant,
                conj=conj)


def test_tiny_ring_against_integer_polynomials():
    """N = 32, m = 2, C = 8, three real input groups -> two complex ciphertexts (the second half empty):
    every step, including y + conj(y), redone over Z[X]/(X^N+1) with Python ints."""
    O = helpers.small_oracle(5, L=3, K=1, dnum=3, qbits=30, pbits=33)
    N, m, C, N1 = O.N, 2, 8, 4
    r = np.random.default_rng(78)
    X = r.uniform(-1, 1, (m, 20))
    Wm = r.uniform(-1, 1, (20, 13))
    bias = r.uniform(-1, 1, 13)
    sx, sw, hw = 2.0**25, 2.0**20, 8
    cl = helpers.Client(O, 6, hamming_weight=hw)
    R = run_complex(O, cl, X, Wm, bias, m, C, N1, sx, sw, 3)
    U, B_out, N2 = R["U"], R["B_out"], R["N2"]
    assert (U, B_out, N2) == (2, 2, 2)
    Q = O.q[0] * O.q[1] * O.q[2]
    ksb = ks_bound(O, 3, hw)
    wmax = int(np.abs(R["diag"]).max())
    bound = 2 * (U * N1 * N * wmax * (19 + ksb) + N2 * ksb) + ksb
    mx = [[int(v) for v in R["mx"][u]] for u in range(U)]
    conj_g = O.galois_elt("conj")
    for b in range(B_out):
        total = [0] * N
        for p in range(N2):
            acc = [0] * N
            for u in range(U):
                for q in range(N1):
                    xr = int_automorph(mx[u], O.galois_elt(q * m), N)
                    acc = [a + c for a, c in zip(acc, int_negacyclic(xr, [int(v) for v in R["diag"][b, p, u, q]], N))]
            total = [a + c for a, c in zip(total, int_automorph(acc, O.galois_elt(p * N1 * m), N))]
        total = [a + c for a, c in zip(total, int_automorph(total, conj_g, N))]
        total = [a + int(c) * int(sw) for a, c in zip(total, R["bias_c"][b])]
        got = O.decrypt_centred(R["y"][b], 3, cl.s, 3)
        err = max(abs(((a - c + Q // 2) % Q) - Q // 2) for a, c in zip(got, total))
        assert err <= bound
        assert max(abs(v) for v in total) > 64 * bound
    slots = np.stack([E.decode(O.decrypt_centred(R["y"][b], 3, cl.s, 3), sx * sw, N) for b in range(B_out)])
    assert np.abs(E.unpack_columns(slots.real, m, C, 13) - (X @ Wm + bias)).max() < 1e-3
    assert np.abs(slots.imag).max() < 1e-3              # the imaginary parts cancel


@pytest.mark.parametrize("d_in", [32, 40, 64])
def test_complexified_projection_decodes_to_the_product(d_in):
    """Even and odd numbers of real groups (G = 2, 3, 4) at n = 128, C = 16."""
    O = helpers.small_oracle(8, L=3, K=1, dnum=3, qbits=40, pbits=42)
    m, C, N1 = 4, 16, 4
    r = np.random.default_rng(d_in)
    X = r.uniform(-1, 1, (m, d_in))
    Wm = r.uniform(-0.5, 0.5, (d_in, 20))
    bias = r.uniform(-0.5, 0.5, 20)
    cl = helpers.Client(O, 31, hamming_weight=16)
    R = run_complex(O, cl, X, Wm, bias, m, C, N1, 2.0**30, 2.0**30, 3)
    assert R["U"] == -(-(-(-d_in // C)) // 2)
    y = O.rescale(R["y"], 3)
    slots = np.stack([cl.decrypt_slots(y[b], 2, 2.0**60 / O.q[2], nlimbs=2) for b in range(R["B_out"])])
    assert np.abs(E.unpack_columns(slots.real, m, C, 20) - (X @ Wm + bias)).max() < 1e-3
    assert np.abs(slots.imag).max() < 1e-3


def test_fused_qk_projection_and_score_friendly_order():
    """W_Q + i W_K on a real-packed input: Q in the real parts, K in the imaginary parts, columns already in
    the order pi_S(h,u) = u*H + h."""
    O = helpers.small_oracle(8, L=3, K=1, dnum=3, qbits=40, pbits=42)
    m, C, N1, H, d_h = 4, 16, 4, 4, 4
    r = np.random.default_rng(5)
    X = r.uniform(-1, 1, (m, 24))
    WQ, WK = r.uniform(-0.5, 0.5, (24, 16)), r.uniform(-0.5, 0.5, (24, 16))
    perm = E.score_friendly_permutation(H, d_h)
    assert sorted(perm) == list(range(16)) and perm[1 * d_h + 2] == 2 * H + 1
    WQp, WKp = np.zeros_like(WQ), np.zeros_like(WK)
    WQp[:, perm], WKp[:, perm] = WQ, WK
    cl = helpers.Client(O, 33, hamming_weight=16)
    N, n = O.N, O.n
    G, B_out, N2 = 2, 1, C // N1
    mx = E.encode(E.pack_columns(X, n, C) + 0j, 2.0**30, N)
    ct_x = np.stack([cl.encrypt_coeffs(mx[g], 3) for g in range(G)])
    diag = E.encode_diagonals_fused(WQp, WKp, m, N, C, N1, 2.0**30)
    baby = [cl.galois_key(O.galois_elt(q * m)) for q in range(1, N1)]
    giant = [cl.galois_key(O.galois_elt(p * N1 * m)) for p in range(1, N2)]
    y = O.rescale(O.ctpt_matmul(3, m, G, B_out, N1, N2, diag, None, 0, ct_x, baby, giant), 3)
    slots = cl.decrypt_slots(y[0], 2, 2.0**60 / O.q[2], nlimbs=2)[None]
    Qp = E.unpack_columns(slots.real, m, C, 16)
    Kp = E.unpack_columns(slots.imag, m, C, 16)
    Qref, Kref = X @ WQ, X @ WK
    for h in range(H):
        for u in range(d_h):
            assert np.abs(Qp[:, u * H + h] - Qref[:, h * d_h + u]).max() < 1e-3
            assert np.abs(Kp[:, u * H + h] - Kref[:, h * d_h + u]).max() < 1e-3


def test_decomplexification_per_accumulator_is_the_same_polynomial():
    """Sec. 3.2 displays c_p = (c~_p + conj(c~_p))/2 for every giant-step accumulator before the fold over p; App.
    A.2.2 counts one conjugation per output block.  Automorphisms commute, so over Z[X]/(X^N+1) both orders are the
    same polynomial: the per-accumulator variant is pinned to the same Python-integer computation (with the noise of
    its N2 conjugations per block), its residues differ from the other order's, and both decode to the product."""
    O = helpers.small_oracle(5, L=3, K=1, dnum=3, qbits=30, pbits=33)
    N, m, C, N1 = O.N, 2, 8, 4
    r = np.random.default_rng(78)
    X = r.uniform(-1, 1, (m, 20))
    Wm = r.uniform(-1, 1, (20, 13))
    bias = r.uniform(-1, 1, 13)
    sx, sw, hw = 2.0**25, 2.0**20, 8
    R0 = run_complex(O, helpers.Client(O, 6, hamming_weight=hw), X, Wm, bias, m, C, N1, sx, sw, 3)
    cl = helpers.Client(O, 6, hamming_weight=hw)
    R = run_complex(O, cl, X, Wm, bias, m, C, N1, sx, sw, 3, per_acc=True)
    assert np.array_equal(R0["ct_x"], R["ct_x"]) and not np.array_equal(R0["y"], R["y"])
    U, B_out, N2 = R["U"], R["B_out"], R["N2"]
    Q = O.q[0] * O.q[1] * O.q[2]
    ksb = ks_bound(O, 3, hw)
    wmax = int(np.abs(R["diag"]).max())
    # every accumulator: inputs' noise through the weights, doubled by c + conj(c), one switch for the conjugation and
    # one for the giant rotation
    bound = N2 * (2 * U * N1 * N * wmax * (19 + ksb) + 2 * ksb)
    mx = [[int(v) for v in R["mx"][u]] for u in range(U)]
    conj_g = O.galois_elt("conj")
    for b in range(B_out):
        total = [0] * N
        for p in range(N2):
            acc = [0] * N
            for u in range(U):
                for q in range(N1):
                    xr = int_automorph(mx[u], O.galois_elt(q * m), N)
                    acc = [a + c for a, c in zip(acc, int_negacyclic(xr, [int(v) for v in R["diag"][b, p, u, q]], N))]
            acc = [a + c for a, c in zip(acc, int_automorph(acc, conj_g, N))]          # real part first
            total = [a + c for a, c in zip(total, int_automorph(acc, O.galois_elt(p * N1 * m), N))]
        total = [a + int(c) * int(sw) for a, c in zip(total, R["bias_c"][b])]
        got = O.decrypt_centred(R["y"][b], 3, cl.s, 3)
        err = max(abs(((a - c + Q // 2) % Q) - Q // 2) for a, c in zip(got, total))
        assert err <= bound
        assert max(abs(v) for v in total) > 32 * bound
    slots = np.stack([E.decode(O.decrypt_centred(R["y"][b], 3, cl.s, 3), sx * sw, N) for b in range(B_out)])
    assert np.abs(E.unpack_columns(slots.real, m, C, 13) - (X @ Wm + bias)).max() < 1e-3
    assert np.abs(slots.imag).max() < 1e-3
