"""GPU: ckks_rescale_static (the entry point for callers that cannot allocate) against ckks_rescale, through the
C ABI: two calls in a row on one parameter set, the second with a smaller input, every residue equal; the size limit
and the other argument checks return errors without launching anything."""
import numpy as np
import pytest
import torch

from tests import helpers
from tests.gpu_util import make_pair, to_dev, to_host
from paper_2604_09975_amd import workload as W

pytestmark = pytest.mark.gpu


def _random_cts(O, r, n_ct, level):
    return np.stack([np.stack([W.uniform_residues(r, O.q[:level], O.N) for _ in range(2)]) for _ in range(n_ct)])


@pytest.mark.parametrize("ring,first,second", [("big", (4, 24), (1, 7)), ("toy", (5, 3), (2, 2))])
def test_two_calls_in_a_row_match_ckks_rescale_and_the_oracle(ring, first, second):
    from paper_2604_09975_amd import binding as B
    O, P = make_pair(W.BIG_RING if ring == "big" else W.TOY_RING)
    r = W.rng(8128)
    for n_ct, level in (first, second):
        ct = _random_cts(O, r, n_ct, level)
        d_in = to_dev(ct)
        want = B.ckks_rescale(P, d_in, level, n_ct)
        out = torch.full((n_ct, 2, level - 1, O.N), -1, dtype=torch.int64, device="cuda")
        torch.cuda.synchronize()
        free_before = torch.cuda.mem_get_info()[0]          # device-wide: sees the library's own allocations too
        got = B.ckks_rescale_static(P, d_in, level, n_ct, out)
        torch.cuda.synchronize()
        assert torch.cuda.mem_get_info()[0] >= free_before
        assert torch.equal(got, want), (n_ct, level)
        assert (to_host(got) == O.rescale(ct, level)).all(), (n_ct, level)


def test_limits_are_errors():
    from paper_2604_09975_amd import binding as B
    O, P = make_pair(W.BIG_RING)
    level = 3
    n_big = 9                                    # 2 * 9 * 2^16 words exceed the 2^20-word buffer
    d_in = torch.zeros((n_big, 2, level, O.N), dtype=torch.int64, device="cuda")
    d_out = torch.zeros((n_big, 2, level - 1, O.N), dtype=torch.int64, device="cuda")
    with pytest.raises(B.CkksError) as e:
        B.ckks_rescale_static(P, d_in, level, n_big, d_out)
    assert e.value.code == -1 and "static buffer" in str(e.value)
    assert B.lib.ckks_rescale_static(P.h, d_in.data_ptr(), 1, 1, d_out.data_ptr(), None) == -2      # level 1
    assert B.lib.ckks_rescale_static(P.h, d_in.data_ptr(), O.L + 1, 1, d_out.data_ptr(), None) == -2
    assert B.lib.ckks_rescale_static(P.h, None, level, 1, d_out.data_ptr(), None) == -1
    with pytest.raises(B.CkksError) as e:        # output inside the input
        rc = B.lib.ckks_rescale_static(P.h, d_in.data_ptr(), level, 1, d_in.data_ptr() + 8 * O.N, None)
        B._check(rc)
    assert e.value.code == -1 and "overlaps" in str(e.value)
    torch.cuda.synchronize()
