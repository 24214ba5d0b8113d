"""rbe_search_static: the search entry point that allocates nothing (fixed scratch array inside the library),
against rbe_search on the same index, twice in a row, the second call with a smaller input."""
import numpy as np
import pytest

import paper_1802_06466_amd as rbe
from parity import check_batch, check_nearlossless
from test_gpu_parity import clustered, load_with_ratio

pytestmark = pytest.mark.gpu


def test_static_scratch_search_equals_rbe_search_on_two_calls_in_a_row():
    N, d, P, k = 300_011, 64, 3, 200
    planes, scales, qp, qs = clustered(N, d, P, 512, 0.3, 4, P, seed=340)
    big = load_with_ratio(planes, scales, 8)
    n2, k2 = 40_003, 17
    small = load_with_ratio(np.ascontiguousarray(planes[:, :n2]), np.ascontiguousarray(scales[:, :n2]), 8)
    # first call: 4 queries, k = 200, 300 011 items; second: 1 query, k = 17, 40 003 items (the array keeps the first
    # call's contents: counters, thresholds and lists must not leak into the second)
    got_a = rbe.rbe_search_static(big, qp, qs, k)
    got_b = rbe.rbe_search_static(small, qp[2:3], qs[2:3], k2)
    ref_a = rbe.rbe_search(big, qp, qs, k)
    ref_b = rbe.rbe_search(small, qp[2:3], qs[2:3], k2)
    for got, ref in ((got_a, ref_a), (got_b, ref_b)):
        np.testing.assert_array_equal(got[0], ref[0]); np.testing.assert_array_equal(got[1], ref[1])
    check_batch(planes, scales, qp, qs, k, got_a[0], got_a[1])
    check_batch(planes[:, :n2], scales[:, :n2], qp[2:3], qs[2:3], k2, got_b[0], got_b[1])
    # and once more in the other order, near-lossless mode in between
    got_n = rbe.rbe_search_static(big, qp[:2], qs[:2], k, mode=rbe.RBE_SELECT_NEARLOSSLESS, group_size_I=8)
    for q in range(2):
        check_nearlossless(planes, scales, qp[q], qs[q], k, 8, got_n[0][q], got_n[1][q])
    got_b2 = rbe.rbe_search_static(small, qp[2:3], qs[2:3], k2)
    np.testing.assert_array_equal(got_b2[0], ref_b[0]); np.testing.assert_array_equal(got_b2[1], ref_b[1])
    # beyond the array's size: refused, nothing run
    assert rbe.rbe_workspace_bytes(big, 64, 4096) > rbe.RBE_STATIC_SCRATCH_BYTES
    q64 = np.repeat(qp[:1], 64, axis=0); s64 = np.repeat(qs[:1], 64, axis=0)
    with pytest.raises(rbe.RbeError) as e:
        rbe.rbe_search_static(big, q64, s64, 4096)
    assert e.value.code == rbe.RBE_EINVAL
    assert rbe.rbe_workspace_bytes(big, 4, 1000) <= rbe.RBE_STATIC_SCRATCH_BYTES
    assert rbe.rbe_workspace_bytes(big, 1, 4096) <= rbe.RBE_STATIC_SCRATCH_BYTES
    rbe.rbe_free(big); rbe.rbe_free(small)
