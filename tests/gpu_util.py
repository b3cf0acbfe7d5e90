"""Helpers for the GPU parity tests: numpy <-> device tensors and matching parameter sets."""
import numpy as np
import torch

from tests import helpers


def to_dev(a):
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint64:
        a = a.view(np.int64)
    return torch.from_numpy(a).cuda()


def to_host(t):
    return t.cpu().numpy().view(np.uint64)


def make_pair(spec_or_oracle):
    """(oracle, library params) on the same primes; the primes come from the oracle's search and are
    checked against the library's own search in test_gpu_ntt."""
    from paper_2604_09975_amd import binding as B
    O = spec_or_oracle if hasattr(spec_or_oracle, "moduli") else helpers.make_oracle(spec_or_oracle)
    P = B.ckks_params_create(O.logN, O.q, O.p, O.dnum)
    return O, P


def load_keys(P, O, client, steps):
    """Oracle-side keys for `steps` and their library handles (None for identity steps)."""
    from paper_2604_09975_amd import binding as B
    np_keys, handles = [], []
    for st in steps:
        g = O.galois_elt(st)
        assert g == B.ckks_galois_elt(P, st)
        if g == 1:
            np_keys.append(None)
            handles.append(None)
            continue
        k = client.galois_key(g)
        np_keys.append(k)
        handles.append(B.ckks_galois_key_load(P, g, to_dev(k)))
    torch.cuda.synchronize()
    return np_keys, handles
