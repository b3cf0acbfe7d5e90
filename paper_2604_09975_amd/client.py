"""Key holder's helper around the library's ckks_client_* calls: complex-slot
encode / decode on the host (numpy fp64), segment-column packing, the plaintext
diagonals of the projection, and a `Client` that draws its randomness from the
seeded generators in `workload`.  Off the server's path: the benchmark uses it
to make valid keys, ciphertexts and weights and to check decrypted results.

Slot j of a plaintext m(X) is m(zeta^(5^j)) with zeta = exp(i*pi/N); rotations
by r are then X -> X^(5^r) and act as the cyclic left shift of Sec. 3.1.
"""
import numpy as np
import torch

from . import binding as B
from . import workload as W


class Encoder:
    """Canonical-embedding encoder for ring degree N (tables built once)."""

    def __init__(self, N):
        self.N, self.n = N, N // 2
        e = np.empty(self.n, dtype=np.int64)
        x = 1
        for j in range(self.n):
            e[j] = x
            x = x * 5 % (2 * N)
        self.pos = (e - 1) >> 1                     # FFT bin of slot j (odd exponent e = 2t+1)
        self.neg = (2 * N - e - 1) >> 1             # bin of the conjugate root
        self.twist = np.exp(-1j * np.pi * np.arange(N) / N)

    def encode(self, z, scale):
        """z [..., n] complex (or real) -> int64 [..., N]: nearest integers to scale * m, m the real
        polynomial with m(zeta_j) = z_j."""
        z = np.asarray(z)
        v = np.zeros(z.shape[:-1] + (self.N,), dtype=np.complex128)
        v[..., self.pos] = z
        v[..., self.neg] = np.conj(z)
        m = (np.fft.fft(v, axis=-1) * self.twist).real * (scale / self.N)
        m = np.rint(m).astype(np.int64)
        # a real slot vector is fixed by conjugation, so m(X) = m(1/X): m[N-j] = -m[j] exactly.  The FFT only
        # gives that up to rounding; enforcing it (for every vector whose imaginary parts are all zero, also
        # inside a complex batch) lets the library read half of every such weight limb.
        h = self.N // 2
        if np.isrealobj(z):
            m[..., h + 1:] = -m[..., 1:h][..., ::-1]
            m[..., h] = 0
        else:
            real_rows = ~np.any(z.imag != 0, axis=-1)
            if np.any(real_rows):
                sub = m[real_rows]
                sub[..., h + 1:] = -sub[..., 1:h][..., ::-1]
                sub[..., h] = 0
                m[real_rows] = sub
        return m

    def decode(self, m, scale):
        """m: N centred integers (array of Python ints or floats) -> n complex slots."""
        mf = np.asarray([float(x) for x in m]) if not isinstance(m, np.ndarray) or m.dtype == object else m.astype(np.float64)
        t = np.fft.ifft(mf * np.conj(self.twist)) * self.N
        return t[self.pos] / scale


def centred_crt(res, moduli):
    """res [nl][N] uint64 residues (nl <= 3) -> list of centred Python ints."""
    M = 1
    for q in moduli:
        M *= int(q)
    acc = [0] * res.shape[1]
    for i, q in enumerate(moduli):
        Mi = M // int(q)
        c = Mi * pow(Mi, -1, int(q))
        acc = [a + int(r) * c for a, r in zip(acc, res[i].tolist())]
    half = M // 2
    return [(a % M) - M if (a % M) > half else (a % M) for a in acc]


def pack_columns(X, n, C):
    """Segment-column packing (Sec. 3.2): ciphertext g, segment c' holds column g*C + (c' mod C)."""
    m, d_in = X.shape
    nseg = n // m
    G = -(-d_in // C)
    Xp = np.zeros((m, G * C))
    Xp[:, :d_in] = X
    cols = (np.arange(G)[:, None] * C + (np.arange(nseg) % C)[None, :])        # [G][nseg]
    return Xp[:, cols].transpose(1, 2, 0).reshape(G, n)                         # slot = seg*m + row


def unpack_columns(slots, m, C, d_out):
    Bn = slots.shape[0]
    Y = slots.reshape(Bn, -1, m)[:, :C, :]          # [B][C][m] (real or complex)
    return Y.transpose(2, 0, 1).reshape(m, Bn * C)[:, :d_out]


def diagonal_slots(Wm, m, n, C, N1, b, p):
    """[G][N1][n] slot vectors of the plaintexts of output block b, giant step p (App. A.2.1, real part):
    segment c holds W[g*C + (c+q) mod C, b*C + (c - p*N1) mod C]."""
    d_in, d_out = Wm.shape
    nseg = n // m
    G = -(-d_in // C)
    Wp = np.zeros((G * C, (-(-d_out // C)) * C), dtype=Wm.dtype)
    Wp[:d_in, :d_out] = Wm
    c = np.arange(nseg) % C
    col = b * C + (c - p * N1) % C                                               # [nseg]
    row = (np.arange(G)[:, None, None] * C + (c[None, None, :] + np.arange(N1)[None, :, None]) % C)   # [G][N1][nseg]
    vals = Wp[row, col[None, None, :]]
    return np.repeat(vals, m, axis=-1)


def pack_columns_complex(X, n, C):
    """Complex-pair compression (Sec. 3.2): ciphertext u holds x^(2u) + i*x^(2u+1)."""
    real = pack_columns(X, n, C)
    if real.shape[0] % 2:
        real = np.concatenate([real, np.zeros((1, n))])
    return real[0::2] + 1j * real[1::2]


def diagonal_slots_complex(Wm, m, n, C, N1, b, p, half=True):
    """[U][N1][n] complex plaintexts of App. A.2.1: W[(2u)C + .., ..] - i*W[(2u+1)C + .., ..] (times 1/2 when the
    real part is recovered as y + conj(y))."""
    d = diagonal_slots(Wm, m, n, C, N1, b, p)                       # [G][N1][n]
    if d.shape[0] % 2:
        d = np.concatenate([d, np.zeros((1,) + d.shape[1:])])
    z = d[0::2] - 1j * d[1::2]
    return 0.5 * z if half else z


def rot_first_masks(n, L, tau):
    """Masks and rotation steps of RotFirst_L(.; tau) (App. A.1): first L - tau slots from the plain rotation,
    the next tau from the wrapped one.  -> (a [n], b [n], (step_tau, step_wrap))."""
    t = tau % L
    i = np.arange(n)
    return (i < L - t).astype(np.float64), ((i >= L - t) & (i < L)).astype(np.float64), (t, (t - L) % n)


def psi_masks(n, m, t):
    """Masks and rotation steps of the intra-segment shift Psi^t (App. A.1) on slots s*m + r:
    H = 1{r < m - t}, U = 1{r >= m - t}, steps (t, (t - m) mod n), t taken mod m."""
    t %= m
    r = np.arange(n) % m
    return (r < m - t).astype(np.float64), (r >= m - t).astype(np.float64), (t, (t - m) % n)


class Client:
    """Secret-key holder bound to one parameter set."""

    def __init__(self, P, seed, hamming_weight=64):
        self.P = P
        self.r = W.rng(seed)
        self.s = W.ternary_secret(self.r, P.N, hamming_weight)
        self.S = B.ckks_client_secret_load(P, self.s)
        self.enc = Encoder(P.N)
        self.moduli = P.q + P.p

    def _dev(self, a):
        a = np.ascontiguousarray(a)
        return torch.from_numpy(a.view(np.int64) if a.dtype == np.uint64 else a).cuda()

    def galois_key(self, step):
        """Library key handle for a rotation step (or "conj")."""
        P = self.P
        g = B.ckks_galois_elt(P, step)
        a = W.uniform_residues(self.r, self.moduli, P.N, lead=(P.dnum,))
        e = W.gaussian_error(self.r, (P.dnum, P.N))
        d_key = B.ckks_client_galois_keygen(P, self.S, g, self._dev(a), self._dev(e))
        h = B.ckks_galois_key_load(P, g, d_key)
        torch.cuda.synchronize()
        return h

    def relin_key(self):
        """Library handle of the relinearisation key."""
        P = self.P
        a = W.uniform_residues(self.r, self.moduli, P.N, lead=(P.dnum,))
        e = W.gaussian_error(self.r, (P.dnum, P.N))
        h = B.ckks_relin_key_load(P, B.ckks_client_relin_keygen(P, self.S, self._dev(a), self._dev(e)))
        torch.cuda.synchronize()
        return h

    def encrypt_slots(self, z, scale, level):
        P = self.P
        m = self.enc.encode(z, scale)
        a = W.uniform_residues(self.r, P.q[:level], P.N)
        e = W.gaussian_error(self.r, (P.N,))
        return B.ckks_client_encrypt(P, self.S, level, self._dev(m), self._dev(a), self._dev(e))

    def decrypt_slots(self, d_ct, level, scale, nlimbs=2):
        P = self.P
        nlimbs = min(nlimbs, level)
        res = B.ckks_client_decrypt(P, self.S, d_ct, level, nlimbs).cpu().numpy().view(np.uint64)
        return self.enc.decode(centred_crt(res, P.q[:nlimbs]), scale)
