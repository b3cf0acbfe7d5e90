"""CPU-only checks of the C-ABI library: it loads, exports every declared symbol, and its host-side
argument validation and prime search work without a GPU."""
import ctypes as C
import os
import re

import pytest

import oracle
from paper_2604_09975_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    syms = set()
    for name in sorted(os.listdir(os.path.join(ROOT, "include"))):
        if not name.endswith(".h"):
            continue
        text = open(os.path.join(ROOT, "include", name)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        syms |= set(re.findall(r"\b(ckks_[a-z_0-9]+)\s*\(", text))
    return sorted(syms)


def test_every_declared_symbol_is_exported():
    syms = declared_symbols()
    assert len(syms) >= 40
    for s in syms:
        assert hasattr(B.lib, s), s


@pytest.mark.parametrize("bits,logN,count", [(30, 12, 2), (40, 12, 2), (50, 16, 24), (60, 16, 8), (33, 10, 5)])
def test_prime_search_agrees_with_oracle(bits, logN, count):
    assert B.ckks_find_primes(bits, logN, count) == oracle.find_primes(bits, logN, count)


def test_prime_search_rejects_bad_arguments():
    with pytest.raises(B.CkksError) as e:
        B.ckks_find_primes(62, 12, 1)
    assert e.value.code == -1
    with pytest.raises(B.CkksError):
        B.ckks_find_primes(13, 12, 1)


def _create(logN, q, p, dnum):
    return B.ckks_params_create(logN, q, p, dnum)


def test_params_validation_needs_no_gpu():
    q = oracle.find_primes(30, 12, 3)
    p = oracle.find_primes(40, 12, 1)
    bad = [
        (12, [q[0], q[1], q[2] + 2], p, 3),          # not prime / not 1 mod 2N
        (12, q, p, 2),                                # L % dnum != 0
        (12, [q[0], q[0], q[1]], p, 3),               # repeated
        (9, q, p, 3),                                 # logN out of range
        (18, q, p, 3),
        (12, q, [q[0]], 3),                           # special prime repeats a ciphertext prime
        (12, q, p, 0),
    ]
    for args in bad:
        with pytest.raises(B.CkksError) as e:
            _create(*args)
        assert e.value.code == -1, args
        assert "ckks_params_create" in str(e.value)
    # a composite that is 1 mod 2N must be refused too
    c = next(v for v in range((1 << 30) + 1, (1 << 31), 8192) if not oracle.is_prime(v))
    with pytest.raises(B.CkksError):
        _create(12, [q[0], q[1], c], p, 3)


def test_null_arguments_are_errors_not_crashes():
    assert B.lib.ckks_params_create(12, None, 3, None, 0, 3, None) == -1
    h = C.c_void_p()
    assert B.lib.ckks_params_create(12, None, 3, None, 0, 3, C.byref(h)) == -1
    assert B.lib.ckks_ntt(None, None, None, 0, 0, None) == -1
    assert B.lib.ckks_rescale(None, None, 2, 1, None, None) == -1
    assert B.lib.ckks_rotate_hoisted(None, None, 1, None, 0, None, None, None) == -1
    assert B.lib.ckks_ctpt_matmul(None, None, None, None, None, None, 0, None, None, None) == -1
    assert B.lib.ckks_weights_create(None, 1, 1, 1, 1, 1, 1, C.byref(h)) == -1
    assert B.lib.ckks_galois_key_load(None, 3, None, None, C.byref(h)) == -1
    B.lib.ckks_params_destroy(None)
    B.lib.ckks_galois_key_destroy(None)
    B.lib.ckks_weights_destroy(None)
    assert b"null" in B.lib.ckks_last_error()
