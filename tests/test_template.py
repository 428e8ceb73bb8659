"""tlt_template_build (host side of sampled drafting) against the oracle's template, through the C ABI."""
import ctypes as C

import numpy as np
import pytest

from oracle import sample_draft as osd
from paper_2511_16665_amd import binding as tlt


@pytest.mark.parametrize("K,D,N", [(1, 4, 3), (2, 2, 4), (2, 2, 5), (2, 4, 8), (3, 3, 10), (3, 4, 25), (8, 6, 48), (10, 8, 64),
                                   (4, 2, 64), (3, 3, 1), (16, 16, 64), (2, 16, 64), (5, 1, 64)])
def test_template_equals_the_oracles(K, D, N):
    p, r, d = tlt.template_build(K, D, N)
    op, orr, od = osd.static_template(K, D, N)
    np.testing.assert_array_equal(p, op)
    np.testing.assert_array_equal(r, orr)
    np.testing.assert_array_equal(d, od)


def test_template_rejects_bad_arguments():
    lib = tlt.load()
    a = (C.c_int32 * 64)()
    n = C.c_int32(0)
    for K, D, N in [(0, 2, 4), (17, 2, 4), (2, -1, 4), (2, 17, 4), (2, 2, 0), (2, 2, 65)]:
        assert lib.tlt_template_build(K, D, N, a, a, a, C.byref(n)) == -1
    assert lib.tlt_template_build(2, 2, 4, None, a, a, C.byref(n)) == -1
    # (-1 = TLT_EINVAL)  depth 0: the root alone
    assert lib.tlt_template_build(2, 0, 4, a, a, a, C.byref(n)) == 0 and n.value == 1 and a[0] in (-1, 0)
