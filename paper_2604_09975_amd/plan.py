"""Host-side planning of the baby-step / giant-step split of a projection (Sec. 3.2: "choose N1 | C").

The rotation counts are those of App. A.2.2: G*(N1-1) baby-step key switches, all of one input hoisted from one
decomposition, and B_out*(N2-1) giant-step key switches, each on its own accumulator.  The two kinds do not cost
the same on the GPU, so the split is chosen by a two-term cost model rather than by the plain count; the
default unit costs are the measured microseconds per key switch of the N = 2^16, 24+8-limb ring (a hoisted
switch; a giant-step switch of the merged form including its decomposition)."""

BABY_US = 72.0
GIANT_US = 84.0


def divisors(C):
    return [d for d in range(1, C + 1) if C % d == 0]


def key_switches(G, B_out, C, N1):
    """(baby, giant) key-switch counts of the split N1 * N2 = C."""
    return G * (N1 - 1), B_out * (C // N1 - 1)


def choose_n1(G, B_out, C, baby_cost=BABY_US, giant_cost=GIANT_US):
    """The divisor N1 of C with the smallest modelled rotation time; ties go to the larger N1 (fewer
    accumulators to hold)."""
    best = None
    for N1 in divisors(C):
        nb, ng = key_switches(G, B_out, C, N1)
        cost = nb * baby_cost + ng * giant_cost
        if best is None or cost < best[0] - 1e-9 or (abs(cost - best[0]) <= 1e-9 and N1 > best[1]):
            best = (cost, N1)
    return best[1]


def ciphertext_bytes(N, L):
    """Serialized size of a ciphertext with L RNS limbs (Sec. 5): two polynomials of N 8-byte residues per limb."""
    return 2 * N * L * 8


def blocks(d, C):
    """Ciphertext blocks of a d-column object with C active columns per ciphertext (Sec. 3.2): ceil(d / C)."""
    return -(-d // C)


def segments(n, m):
    """N_seg of Sec. 3.1: n = m * N_seg slots."""
    assert n % m == 0
    return n // m


def complex_pairs(G):
    """U = ceil(G / 2) complexified inputs x^(2u) + i x^(2u+1) (Sec. 3.2)."""
    return -(-G // 2)
