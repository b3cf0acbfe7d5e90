"""fp64 side of the oracle (TEST INFRASTRUCTURE ONLY): complex-slot encode/decode,
CRT lifting, segment-column packing and the plaintext diagonals of the
projection kernel, in plain numpy.

Slot convention (reading; the paper only says n = N/2 complex slots are packed
by an approximate encoding map, Sec. 2.2): slot j is the value of the plaintext
polynomial at zeta^(5^j), zeta = exp(i*pi/N), so that the Galois map
X -> X^(5^r) is the cyclic LEFT shift by r of Sec. 3.1 and X -> X^(-1) is
conjugation.
"""
import numpy as np


def slot_exponents(N):
    """e_j = 5^j mod 2N, j < N/2."""
    n = N // 2
    e = np.empty(n, dtype=np.int64)
    cur = 1
    for j in range(n):
        e[j] = cur
        cur = (cur * 5) % (2 * N)
    return e


def encode_direct(z, scale, N):
    """m_k = round_half_even(scale * (2/N) * Re sum_j z_j * zeta_j^(-k)); O(N*n), small N only.

    Follows from m(zeta_j) = z_j and m(conj zeta_j) = conj z_j for a real polynomial of degree < N.
    """
    z = np.asarray(z, dtype=np.complex128)
    e = slot_exponents(N)
    k = np.arange(N)
    ang = -np.pi * ((e[:, None] * k[None, :]) % (2 * N)) / N
    s = (z[:, None] * np.exp(1j * ang)).sum(axis=0)
    return np.rint(scale * (2.0 / N) * s.real).astype(np.int64)


def encode(z, scale, N):
    """Same map through one length-N FFT.  z [..., n] complex -> int64 [..., N]."""
    z = np.asarray(z, dtype=np.complex128)
    e = slot_exponents(N)
    v = np.zeros(z.shape[:-1] + (N,), dtype=np.complex128)
    v[..., (e - 1) // 2] = z
    v[..., (2 * N - e - 1) // 2] = np.conj(z)
    k = np.arange(N)
    f = np.fft.fft(v, axis=-1) * np.exp(-1j * np.pi * k / N)
    return np.rint(scale * f.real / N).astype(np.int64)


def decode(m, scale, N):
    """z_j = m(zeta^(5^j)) / scale.  m: N integers (int64 array or Python ints)."""
    mf = np.array([float(x) for x in m], dtype=np.float64) if not isinstance(m, np.ndarray) else m.astype(np.float64)
    k = np.arange(N)
    t = np.fft.ifft(mf * np.exp(1j * np.pi * k / N)) * N
    e = slot_exponents(N)
    return t[(e - 1) // 2] / scale


def decode_direct(m, scale, N):
    """O(N*n) evaluation, small N only."""
    mf = np.array([float(x) for x in m], dtype=np.float64)
    e = slot_exponents(N)
    k = np.arange(N)
    ang = np.pi * ((e[:, None] * k[None, :]) % (2 * N)) / N
    return (mf[None, :] * np.exp(1j * ang)).sum(axis=1) / scale


def crt_centre(res, moduli):
    """res [nl][N] canonical residues -> list of N centred Python ints in (-M/2, M/2]."""
    M = 1
    for q in moduli:
        M *= int(q)
    coef = []
    for q in moduli:
        Mi = M // int(q)
        coef.append(Mi * pow(Mi % int(q), -1, int(q)))
    out = []
    cols = [[int(x) for x in res[i]] for i in range(len(moduli))]
    for x in range(len(cols[0])):
        v = 0
        for i in range(len(moduli)):
            v += cols[i][x] * coef[i]
        v %= M
        if v > M // 2:
            v -= M
        out.append(v)
    return out


# ---------------------------------------------------------------------------
# segment-column packing (Sec. 3.2) and the weight diagonals (App. A.2.1)
# ---------------------------------------------------------------------------
def pack_columns(X, n, C):
    """X [m][d_in] -> slots [G][n]: in ciphertext g, segment c' holds column g*C + (c' mod C).

    The paper activates the first C segments; here C divides N_seg = n/m and the
    C columns repeat with period C over all N_seg segments, so that a plain
    rotation by whole segments is already cyclic over the C active columns
    (reading for C < N_seg; with C = N_seg it is the paper's layout itself).
    Columns beyond d_in are zero.
    """
    m, d_in = X.shape
    nseg = n // m
    assert nseg % C == 0
    G = -(-d_in // C)
    Xp = np.zeros((m, G * C))
    Xp[:, :d_in] = X
    out = np.zeros((G, n))
    for g in range(G):
        for cp in range(nseg):
            out[g, cp * m:(cp + 1) * m] = Xp[:, g * C + cp % C]
    return out


def unpack_columns(slots, m, C, d_out):
    """slots [B][n] -> Y [m][d_out] read from the first C segments of each block."""
    B = slots.shape[0]
    Y = np.zeros((m, B * C), dtype=slots.dtype)
    for b in range(B):
        for c in range(C):
            Y[:, b * C + c] = slots[b, c * m:(c + 1) * m]
    return Y[:, :d_out]


def weight_diagonal(W, m, n, C, N1, b, p, g, q):
    """Slot vector of the plaintext for (output block b, giant p, input group g, baby q).

    Segment c' (c = c' mod C) holds, in all of its m slots,
        W[g*C + (c+q) mod C,  b*C + (c - p*N1) mod C]
    -- the real part of the weight formula of App. A.2.1 -- and zero outside W.
    """
    d_in, d_out = W.shape
    nseg = n // m
    c = np.arange(nseg) % C
    row = g * C + (c + q) % C
    col = b * C + (c - p * N1) % C
    ok = (row < d_in) & (col < d_out)
    val = np.zeros(nseg)
    val[ok] = W[row[ok], col[ok]]
    return np.repeat(val, m)


def bias_slots(bias, m, n, C, b):
    """Slot vector of the bias for output block b: segment c' holds bias[b*C + c' mod C]."""
    nseg = n // m
    col = b * C + np.arange(nseg) % C
    val = np.zeros(nseg)
    ok = col < len(bias)
    val[ok] = bias[col[ok]]
    return np.repeat(val, m)


def encode_diagonals(W, m, N, C, N1, scale, blocks=None):
    """int64 [B_out][N2][G][N1][N] coefficient encodings of every diagonal (blocks: subset of b kept, others zero)."""
    n = N // 2
    d_in, d_out = W.shape
    G, B_out, N2 = -(-d_in // C), -(-d_out // C), C // N1
    out = np.zeros((B_out, N2, G, N1, N), dtype=np.int64)
    for b in range(B_out):
        if blocks is not None and b not in blocks:
            continue
        for p in range(N2):
            z = np.stack([weight_diagonal(W, m, n, C, N1, b, p, g, q) for g in range(G) for q in range(N1)])
            out[b, p] = encode(z, scale, N).reshape(G, N1, N)
    return out


# ---------------------------------------------------------------------------
# complex-pair compression and the fused QK projection (Sec. 3.2, App. A.2.1 / A.2.3)
# ---------------------------------------------------------------------------
def pack_columns_complex(X, n, C):
    """Complexified inputs: ciphertext u holds x^(2u) + i*x^(2u+1), the real groups of pack_columns
    (an odd last group has imaginary part zero).  [U][n] complex."""
    real = pack_columns(X, n, C)
    G = real.shape[0]
    U = -(-G // 2)
    out = np.zeros((U, n), dtype=np.complex128)
    for u in range(U):
        out[u] = real[2 * u]
        if 2 * u + 1 < G:
            out[u] = out[u] + 1j * real[2 * u + 1]
    return out


def weight_diagonal_complex(W, m, n, C, N1, b, p, u, q, half=True):
    """Complex plaintext of App. A.2.1 for pair u: segment c holds
        W[(2u)C + (c+q) mod C, bC + (c - p*N1) mod C] - i * W[(2u+1)C + (c+q) mod C, bC + (c - p*N1) mod C],
    times 1/2 when the result is to be recovered as y + conj(y)."""
    re = weight_diagonal(W, m, n, C, N1, b, p, 2 * u, q)
    G = -(-W.shape[0] // C)
    im = weight_diagonal(W, m, n, C, N1, b, p, 2 * u + 1, q) if 2 * u + 1 < G else np.zeros(n)
    z = re - 1j * im
    return 0.5 * z if half else z


def encode_diagonals_complex(W, m, N, C, N1, scale, half=True, blocks=None):
    """int64 [B_out][N2][U][N1][N] encodings of the complexified diagonals (blocks: subset of b kept, others zero)."""
    n = N // 2
    d_in, d_out = W.shape
    G, B_out, N2 = -(-d_in // C), -(-d_out // C), C // N1
    U = -(-G // 2)
    out = np.zeros((B_out, N2, U, N1, N), dtype=np.int64)
    for b in range(B_out):
        if blocks is not None and b not in blocks:
            continue
        for p in range(N2):
            z = np.stack([weight_diagonal_complex(W, m, n, C, N1, b, p, u, q, half) for u in range(U) for q in range(N1)])
            out[b, p] = encode(z, scale, N).reshape(U, N1, N)
    return out


def encode_diagonals_fused(WQ, WK, m, N, C, N1, scale):
    """Fused QK projection (App. A.2.3): one projection with the complex weights W_Q + i*W_K on a REAL-packed
    input yields Q in the real parts and K in the imaginary parts.  int64 [B_out][N2][G][N1][N]."""
    n = N // 2
    d_in, d_out = WQ.shape
    G, B_out, N2 = -(-d_in // C), -(-d_out // C), C // N1
    out = np.zeros((B_out, N2, G, N1, N), dtype=np.int64)
    for b in range(B_out):
        for p in range(N2):
            z = np.stack([weight_diagonal(WQ, m, n, C, N1, b, p, g, q) + 1j * weight_diagonal(WK, m, n, C, N1, b, p, g, q)
                          for g in range(G) for q in range(N1)])
            out[b, p] = encode(z, scale, N).reshape(G, N1, N)
    return out


def score_friendly_permutation(H, d_h):
    """pi_S of App. A.2.1: column k(h,u) = h*d_h + u of W_Q / W_K moves to position u*H + h.
    Returns `perm` with W_perm[:, perm[k]] = W[:, k]."""
    perm = np.empty(H * d_h, dtype=np.int64)
    for h in range(H):
        for u in range(d_h):
            perm[h * d_h + u] = u * H + h
    return perm


# ---------------------------------------------------------------------------
# restricted rotations (App. A.1)
# ---------------------------------------------------------------------------
def rot_first_masks(n, L, tau):
    """a_{L,tau} = 1{0 <= i < L - tau}, b_{L,tau} = 1{L - tau <= i < L} and the two rotation steps
    (tau, (tau - L) mod n) of RotFirst_L(.; tau)."""
    tau %= L
    i = np.arange(n)
    a = ((i >= 0) & (i < L - tau)).astype(np.float64)
    b = ((i >= L - tau) & (i < L)).astype(np.float64)
    return a, b, (tau, (tau - L) % n)


def psi_masks(n, m, t):
    """Masks and rotation steps of the intra-segment shift Psi^t (App. A.1): H_{r,s} = 1{0 <= r < m - t},
    U_{r,s} = 1{m - t <= r < m} on slot s*m + r, steps (t, (t - m) mod n) with t taken mod m."""
    t %= m
    r = np.arange(n) % m
    return (r < m - t).astype(np.float64), (r >= m - t).astype(np.float64), (t, (t - m) % n)


def psi_shift(x, m, t):
    """Psi^t on a slot vector by its definition (Sec. 3.1): slot s*m + r takes the value of slot s*m + (r+t) mod m."""
    n = len(x)
    X = np.asarray(x).reshape(n // m, m)          # X[s][r]
    return np.roll(X, -(t % m), axis=1).reshape(n)
