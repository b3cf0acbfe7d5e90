"""Key holder's helper around the library's ckks_client_* / ckks_encode / ckks_decode calls: segment-column
packing and the plaintext slot vectors of the projection on the host (numpy, data layout only), and a `Client`
that draws its randomness from the seeded generators in `workload`.  Off the server's path: the benchmark uses it
to make valid keys, ciphertexts and weights and to check decrypted results.

Slot j of a plaintext m(X) is m(zeta^(5^j)) with zeta = exp(i*pi/N); rotations
by r are then X -> X^(5^r) and act as the cyclic left shift of Sec. 3.1.
"""
import numpy as np
import torch

from . import binding as B
from . import workload as W


class Encoder:
    """Complex-slot encode / decode of one parameter set, on the device (ckks_encode / ckks_decode)."""

    def __init__(self, P):
        self.P, self.N, self.n = P, P.N, P.N // 2

    def encode(self, z, scale):
        """z [..., n] complex or real (numpy) -> int64 device tensor [..., N]: nearest integers to scale * m, m
        the real polynomial with m(zeta_j) = z_j.  Vectors whose imaginary parts are all zero get exactly
        antisymmetric coefficients (m[N-j] = -m[j]), which lets the weight store keep half of every limb."""
        z = np.asarray(z)
        lead = z.shape[:-1]
        if np.isrealobj(z):
            d = torch.from_numpy(np.ascontiguousarray(z.reshape(-1, self.n), dtype=np.float64)).cuda().to(torch.complex128)
            return B.ckks_encode(self.P, d, scale, B.ENCODE_REAL).reshape(lead + (self.N,))
        flat = z.reshape(-1, self.n)
        d = torch.from_numpy(np.ascontiguousarray(flat, dtype=np.complex128)).cuda()
        out = B.ckks_encode(self.P, d, scale)
        real_rows = np.flatnonzero(~np.any(flat.imag != 0, axis=-1))
        if real_rows.size:
            idx = torch.from_numpy(real_rows).cuda()
            out[idx] = B.ckks_encode(self.P, d[idx].contiguous(), scale, B.ENCODE_REAL)
        return out.reshape(lead + (self.N,))

    def decode(self, d_res, nlimbs, scale):
        """d_res device [nlimbs][N] coefficient-domain residues (nlimbs <= 2) -> n complex slots (numpy)."""
        return B.ckks_decode(self.P, d_res.reshape(1, nlimbs, self.N), nlimbs, scale)[0].cpu().numpy()


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


def score_friendly_permutation(H, d_h):
    """pi_S of App. A.2.1: the head-major column k(h,u) = h*d_h + u of W_Q / W_K goes to position u*H + h, so that the
    projection emits Q and K in the segment order the score kernel consumes.  Returns `perm` with
    perm[k(h,u)] = u*H + h (a bijection of range(H*d_h))."""
    h, u = np.divmod(np.arange(H * d_h), d_h)
    return u * H + h


def permute_columns(Wm, perm, bias=None):
    """W^pi with W^pi[:, perm[k]] = W[:, k] (and the bias moved the same way): a plaintext-side reordering of the
    weight matrix before its diagonals are encoded, no homomorphic cost.  pi_V of App. A.2.1 is the identity
    (W_V stays head-major), so only W_Q and W_K pass through here."""
    perm = np.asarray(perm)
    if sorted(perm.tolist()) != list(range(Wm.shape[1])):
        raise ValueError("perm must be a bijection of the columns")
    Wp = np.empty_like(Wm)
    Wp[:, perm] = Wm
    if bias is None:
        return Wp
    bp = np.empty_like(bias)
    bp[perm] = bias
    return Wp, bp


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
        self.enc = Encoder(P)
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
        h = B.ckks_galois_key_adopt(P, g, d_key)      # the generated buffer becomes the library's key: no second copy
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
        return B.ckks_client_encrypt(P, self.S, level, m, self._dev(a), self._dev(e))

    def decrypt_slots(self, d_ct, level, scale, nlimbs=2):
        P = self.P
        nlimbs = min(nlimbs, level)
        return self.enc.decode(B.ckks_client_decrypt(P, self.S, d_ct, level, nlimbs), nlimbs, scale)
