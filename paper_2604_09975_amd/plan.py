"""Host-side planning of the baby-step / giant-step split of a projection (Sec. 3.2: "choose N1 | C").

The rotation counts are those of App. A.2.2: G*(N1-1) baby-step key switches, all of one input hoisted from one
decomposition, and B_out*(N2-1) giant-step key switches, each on its own accumulator.  The two kinds do not cost
the same on the GPU, so the split is chosen by a two-term cost model rather than by the plain count; the
default unit costs are the measured microseconds per key switch of the N = 2^16, 24+8-limb ring (a hoisted
switch; a giant-step switch of the merged form including its decomposition)."""

BABY_US = 49.0
GIANT_US = 75.0


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
