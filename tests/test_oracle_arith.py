"""Pins for the oracle's scalar arithmetic, primes and roots."""
import math
import random

import numpy as np
import pytest

import oracle
from tests import helpers
from paper_2604_09975_amd import workload as W


def test_mulmod_against_python_ints():
    rnd = random.Random(7)
    for bits in (30, 40, 50, 60, 62):
        q = oracle.find_primes(bits, 12, 1)[0]
        cases = [(0, 0), (0, q - 1), (1, q - 1), (q - 1, q - 1), (q - 1, 1)]
        cases += [(rnd.randrange(q), rnd.randrange(q)) for _ in range(200)]
        for a, b in cases:
            assert oracle.mulmod(a, b, q) == (a * b) % q


def _trial_division_is_prime(n):
    """Independent of the oracle's Miller-Rabin: divide by every odd number up to sqrt(n)."""
    if n < 2 or n % 2 == 0:
        return n == 2
    lim = math.isqrt(n)
    step = 1 << 22
    for lo in range(3, lim + 1, 2 * step):
        d = np.arange(lo, min(lo + 2 * step, lim + 1), 2, dtype=np.uint64)
        if d.size and (np.uint64(n) % d == 0).any():
            return False
    return True


def _python_miller_rabin(n, rounds=24):
    rnd = random.Random(n)
    d, r = n - 1, 0
    while d % 2 == 0:
        d //= 2
        r += 1
    for _ in range(rounds):
        a = rnd.randrange(2, n - 1)
        x = pow(a, d, n)
        if x in (1, n - 1):
            continue
        for _ in range(r - 1):
            x = x * x % n
            if x == n - 1:
                break
        else:
            return False
    return True


@pytest.mark.parametrize("bits,logN,count", [(30, 12, 2), (40, 12, 2), (50, 16, 24)])
def test_prime_rule_trial_division(bits, logN, count):
    """Every hit is prime and of the form 2^bits - k*2N + 1; every skipped candidate is composite."""
    primes = oracle.find_primes(bits, logN, count)
    twoN = 2 << logN
    assert len(set(primes)) == count
    ks = []
    for p in primes:
        assert p % twoN == 1 and p.bit_length() == bits
        assert _trial_division_is_prime(p)
        ks.append(((1 << bits) + 1 - p) // twoN)
    assert ks == sorted(ks)
    # small bit sizes: check the skipped candidates too (they must be composite)
    if bits <= 40:
        hit = set(ks)
        for k in range(1, ks[-1]):
            if k not in hit:
                assert not _trial_division_is_prime((1 << bits) - k * twoN + 1)


def test_prime_rule_60_bit():
    """60-bit special primes: trial division to 2^30 is too slow here; an independent
    pure-Python Miller-Rabin with random bases confirms hits and rejects the skipped candidates."""
    primes = oracle.find_primes(60, 16, 8)
    twoN = 2 << 16
    ks = [((1 << 60) + 1 - p) // twoN for p in primes]
    assert ks == sorted(ks) and len(set(ks)) == 8
    for p in primes:
        assert p % twoN == 1 and p.bit_length() == 60 and _python_miller_rabin(p)
    for k in range(1, ks[-1]):
        if k not in set(ks):
            assert not _python_miller_rabin((1 << 60) - k * twoN + 1)


def test_is_prime_small_numbers():
    sieve = [True] * 2000
    sieve[0] = sieve[1] = False
    for i in range(2, 2000):
        if sieve[i]:
            for j in range(i * i, 2000, i):
                sieve[j] = False
    for n in range(2000):
        assert oracle.is_prime(n) == sieve[n]
    # Carmichael numbers and strong pseudoprimes to small bases
    for n in (561, 1105, 1729, 2047, 3215031751, 3825123056546413051):
        assert not oracle.is_prime(n)


@pytest.mark.parametrize("logN", [2, 3, 4, 5])
def test_min_root_exhaustive(logN):
    N = 1 << logN
    for q in oracle.find_primes(14, logN, 3) + oracle.find_primes(20, logN, 2):
        psi = oracle.min_root(q, logN)
        assert pow(psi, N, q) == q - 1
        for x in range(1, psi):
            assert pow(x, N, q) != q - 1


def test_min_root_big_ring():
    O = helpers.make_oracle(W.BIG_RING)
    for i, q in enumerate(O.moduli):
        psi = O.psi(i)
        assert pow(psi, O.N, q) == q - 1
        assert psi == oracle.min_root(q, 16)
