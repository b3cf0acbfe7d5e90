"""Seeded synthetic inputs for the CKKS ct x pt matmul path.

This module holds no arithmetic of the method: it only draws random numbers
(numpy PCG64 through `numpy.random.default_rng(seed)`) with the shapes and
value distributions of the benchmark configurations and describes those
configurations as plain data.  Both the GPU library's callers and the tests'
CPU checker take their raw inputs from here, so the two sides see identical
matrices, secrets, errors and uniform residues.
"""
from dataclasses import dataclass, field

import numpy as np

SEED_BASE = 20260409


@dataclass(frozen=True)
class RingSpec:
    """Which primes to search for (the search itself is done by each consumer)."""
    logN: int
    q_bits: tuple          # bit size of each ciphertext prime, q_0 first
    p_bits: tuple          # bit size of each special prime
    dnum: int
    log_scale: int
    # (bits -> which hits of the descending search go to p first); p takes the
    # earliest hits of its bit size so that P exceeds every digit product
    name: str = ""


@dataclass(frozen=True)
class MatmulSpec:
    ring: RingSpec
    m: int                 # sequence length = segment length
    d_in: int
    d_out: int
    C: int                 # active columns per ciphertext
    N1: int                # baby steps
    x_dist: str = "normal_clip4"
    w_std: float = 0.02
    bias: bool = True
    seed: int = SEED_BASE
    name: str = ""


TOY_RING = RingSpec(logN=12, q_bits=(40, 30, 30), p_bits=(40,), dnum=3, log_scale=30, name="toy")
BIG_RING = RingSpec(logN=16, q_bits=(50,) * 24, p_bits=(60,) * 8, dnum=3, log_scale=40, name="n16_l24_k8")
NTT_RING = RingSpec(logN=16, q_bits=(50,) * 24, p_bits=(), dnum=3, log_scale=40, name="ntt_n16_l24")

TOY_MATMUL = MatmulSpec(ring=TOY_RING, m=16, d_in=64, d_out=64, C=64, N1=64, x_dist="uniform1", w_std=0.0,
                        bias=False, seed=SEED_BASE + 0, name="toy_16x64x64")
BERT_QKV = MatmulSpec(ring=BIG_RING, m=128, d_in=768, d_out=2304, C=256, N1=32, seed=SEED_BASE + 3,
                      name="bert_base_qkv_128x768x2304")
GPT2_LAYERS = (
    MatmulSpec(ring=BIG_RING, m=128, d_in=768, d_out=2304, C=256, N1=32, seed=SEED_BASE + 40, name="gpt2_qkv"),
    MatmulSpec(ring=BIG_RING, m=128, d_in=768, d_out=768, C=256, N1=16, seed=SEED_BASE + 41, name="gpt2_attn_out"),
    MatmulSpec(ring=BIG_RING, m=128, d_in=768, d_out=3072, C=256, N1=32, seed=SEED_BASE + 42, name="gpt2_ffn_up"),
    MatmulSpec(ring=BIG_RING, m=128, d_in=3072, d_out=768, C=256, N1=8, seed=SEED_BASE + 43, name="gpt2_ffn_down"),
)

# hoisted-rotation batch: the 26 non-trivial listed steps, conjugation, and the
# full-turn step 2^15 (= identity at N = 2^16), see the design notes
CONJ = "conj"
HOISTED_STEPS = tuple(range(1, 17)) + tuple(1 << k for k in range(5, 16)) + (CONJ,)
HOISTED_SEED = SEED_BASE + 2
NTT_SEED = SEED_BASE + 1
NTT_BATCH = 64


def rng(seed):
    return np.random.default_rng(int(seed))


def ternary_secret(r, N, hamming_weight=64):
    """Ternary secret with exactly `hamming_weight` non-zeros, signs uniform."""
    s = np.zeros(N, dtype=np.int8)
    pos = r.choice(N, size=min(hamming_weight, N), replace=False)
    s[pos] = r.choice(np.array([-1, 1], dtype=np.int8), size=len(pos))
    return s


def gaussian_error(r, shape, sigma=3.2):
    """round(sigma*z), |e| <= 6*sigma by rejection."""
    e = np.rint(sigma * r.standard_normal(shape))
    bound = np.floor(6 * sigma)
    bad = np.abs(e) > bound
    while bad.any():
        e[bad] = np.rint(sigma * r.standard_normal(int(bad.sum())))
        bad = np.abs(e) > bound
    return e.astype(np.int64)


def uniform_residues(r, moduli, N, lead=()):
    """uint64 [*lead][len(moduli)][N], limb i uniform in [0, moduli[i])."""
    out = np.empty(tuple(lead) + (len(moduli), N), dtype=np.uint64)
    for i, q in enumerate(moduli):
        out[..., i, :] = r.integers(0, int(q), size=tuple(lead) + (N,), dtype=np.uint64)
    return out


def unit_disk_slots(r, n):
    """n complex values uniform on the unit disk."""
    rad = np.sqrt(r.random(n))
    th = 2 * np.pi * r.random(n)
    return rad * np.exp(1j * th)


def matmul_inputs(spec: MatmulSpec):
    """X [m][d_in], W [d_in][d_out], bias [d_out] or None, all fp64."""
    r = rng(spec.seed)
    if spec.x_dist == "uniform1":
        X = r.uniform(-1.0, 1.0, size=(spec.m, spec.d_in))
        W = r.uniform(-0.1, 0.1, size=(spec.d_in, spec.d_out))
    else:
        X = np.clip(r.standard_normal((spec.m, spec.d_in)), -4.0, 4.0)
        W = spec.w_std * r.standard_normal((spec.d_in, spec.d_out))
    b = spec.w_std * r.standard_normal(spec.d_out) if spec.bias else None
    return X, W, b


def plan(spec: MatmulSpec):
    """Block counts of the projection: G input groups, B_out output blocks, N2 giant steps."""
    G = -(-spec.d_in // spec.C)
    B_out = -(-spec.d_out // spec.C)
    assert spec.C % spec.N1 == 0
    return G, B_out, spec.C // spec.N1
