"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on
the same seeded inputs."""
import numpy as np
import pytest

import oracle
import paper_1802_06466_amd as rbe
import rbe_synth
from parity import check_batch, check_nearlossless, check_topk, score_tolerance

pytestmark = pytest.mark.gpu


def random_corpus(rng, N, d, P):
    planes = rng.integers(0, 2**64, size=(P, N, d // 64), dtype=np.uint64)
    scales = rng.uniform(0.01, 1.0, size=(P, N)).astype(np.float32)
    return planes, scales


def random_queries(rng, Q, d, Pq):
    return (rng.integers(0, 2**64, size=(Q, Pq, d // 64), dtype=np.uint64),
            rng.uniform(0.01, 1.0, size=(Q, Pq)).astype(np.float32))


def clustered(N, d, P, n_clusters, sigma, Q, Pq, seed=0, sort_by_cluster=False):
    c = rbe_synth.centres_numpy(n_clusters, d)
    x = rbe_synth.vectors_numpy(N, c, sigma, seed=rbe_synth.SEED_ITEMS + seed, sort_by_cluster=sort_by_cluster)
    q = rbe_synth.vectors_numpy(Q, c, sigma, seed=rbe_synth.SEED_QUERIES + seed)
    planes, scales = oracle.encode(x, P)
    qp, qs = oracle.encode(q, Pq)
    return planes, scales, np.ascontiguousarray(qp.transpose(1, 0, 2)), np.ascontiguousarray(qs.T)


NL_STATS = {}     # search statistics of the last nl_search, per path


def nl_search(ix, qp, qs, k, mode=None, group_size_I=0):
    """A near-lossless search both ways -- the exact scans followed by selection by groups (the default) and the
    scan that keeps one queue per thread as Algorithm 1 is written -- which must agree bit for bit; returns the
    default path's result."""
    mode = rbe.RBE_SELECT_NEARLOSSLESS if mode is None else mode
    rbe.rbe_debug_set_nearlossless_path(ix, 1)
    ids_q, sc_q = rbe.rbe_search(ix, qp, qs, k, mode=mode, group_size_I=group_size_I)
    NL_STATS["queue"] = rbe.rbe_get_search_stats(ix)
    kernels_q = NL_STATS["queue"]["scan_kernel"]
    rbe.rbe_debug_set_nearlossless_path(ix, 0)
    ids, sc = rbe.rbe_search(ix, qp, qs, k, mode=mode, group_size_I=group_size_I)
    NL_STATS["groups"] = rbe.rbe_get_search_stats(ix)
    kernels = NL_STATS["groups"]["scan_kernel"]
    assert all(kn == "scan_groupmax" for kn in kernels_q) and "scan_groupmax" not in kernels
    np.testing.assert_array_equal(ids, ids_q)
    np.testing.assert_array_equal(sc, sc_q)
    return ids, sc


def load_with_ratio(planes, scales, ratio, flags=0):
    P, N, W = planes.shape
    ix = rbe.rbe_index_create_ex(N, 64 * W, P, flags, ratio)
    rbe.rbe_load_chunk(ix, 0, planes, scales)
    rbe.rbe_finalize(ix)
    return ix


# ------------------------------------------------------------------ binary dot products: bit-exact
@pytest.mark.parametrize("N,d,P,Pq", [(1, 64, 1, 1), (63, 64, 3, 3), (1025, 64, 3, 2), (5000, 128, 4, 4),
                                      (3000, 128, 2, 3), (2049, 256, 2, 2)])
def test_popcounts_bit_exact(N, d, P, Pq):
    rng = np.random.default_rng(N + d + P + Pq)
    planes, scales = random_corpus(rng, N, d, P)
    qp, _ = random_queries(rng, 1, d, Pq)
    ix = rbe.rbe_load_corpus(planes, scales)
    got = rbe.rbe_debug_popcounts(ix, qp[0], 0, N)
    np.testing.assert_array_equal(got, oracle.popcounts(planes, qp[0]))
    if N > 100:
        part = rbe.rbe_debug_popcounts(ix, qp[0], 37, 50)
        np.testing.assert_array_equal(part, oracle.popcounts(planes[:, 37:87], qp[0]))
    rbe.rbe_free(ix)


# ------------------------------------------------------------------ combined fp32 scores
@pytest.mark.parametrize("N,d,P,Pq", [(777, 64, 1, 1), (4099, 64, 3, 3), (4099, 64, 2, 3), (3001, 128, 4, 4),
                                      (1500, 128, 4, 1), (1030, 256, 3, 2)])
def test_dense_scores_within_tolerance(N, d, P, Pq):
    rng = np.random.default_rng(7 * N + d + P + Pq)
    planes, scales = random_corpus(rng, N, d, P)
    qp, qs = random_queries(rng, 1, d, Pq)
    ix = rbe.rbe_load_corpus(planes, scales)
    got = rbe.rbe_debug_scores(ix, qp[0], qs[0], 0, N).astype(np.float64)
    ref = oracle.scores(planes, scales, qp[0], qs[0])
    assert np.all(np.abs(got - ref) <= score_tolerance(scales, qs[0], d))
    rbe.rbe_free(ix)


def test_dense_scores_on_encoded_corpus_relative():
    planes, scales, qp, qs = clustered(20000, 64, 3, 16, 0.3, 1, 3)
    ix = rbe.rbe_load_corpus(planes, scales)
    got = rbe.rbe_debug_scores(ix, qp[0], qs[0], 0, 20000).astype(np.float64)
    ref = oracle.scores(planes, scales, qp[0], qs[0])
    big = np.abs(ref) > 0.1 * np.abs(ref).max()
    np.testing.assert_allclose(got[big], ref[big], rtol=1e-5)
    rbe.rbe_free(ix)


# ------------------------------------------------------------------ exact search, size sweep
@pytest.mark.parametrize("N", [1, 63, 64, 65, 1000, 1024, 1025, 65537])
@pytest.mark.parametrize("k", [1, 100, 1000])
def test_search_sizes(N, k):
    rng = np.random.default_rng(N * 31 + k)
    planes, scales = random_corpus(rng, N, 64, 3)
    qp, qs = random_queries(rng, 2, 64, 3)
    ix = rbe.rbe_load_corpus(planes, scales)
    ids, sc = rbe.rbe_search(ix, qp, qs, k)
    check_batch(planes, scales, qp, qs, k, ids, sc)
    rbe.rbe_free(ix)


@pytest.mark.parametrize("d,P,Pq,Q,k", [(64, 1, 1, 1, 10), (64, 2, 3, 8, 100), (64, 3, 3, 64, 50), (64, 4, 4, 3, 4096),
                                        (128, 4, 4, 8, 1000), (128, 1, 2, 1, 7), (128, 3, 1, 5, 333), (256, 2, 2, 4, 100)])
def test_search_shapes(d, P, Pq, Q, k):
    N = 30011
    rng = np.random.default_rng(d + 10 * P + 100 * Pq + Q + k)
    planes, scales = random_corpus(rng, N, d, P)
    qp, qs = random_queries(rng, Q, d, Pq)
    ix = rbe.rbe_load_corpus(planes, scales)
    ids, sc = rbe.rbe_search(ix, qp, qs, k)
    check_batch(planes, scales, qp, qs, k, ids, sc)
    rbe.rbe_free(ix)


def test_k_larger_than_corpus():
    rng = np.random.default_rng(5)
    planes, scales = random_corpus(rng, 300, 64, 2)
    qp, qs = random_queries(rng, 3, 64, 2)
    ix = rbe.rbe_load_corpus(planes, scales)
    ids, sc = rbe.rbe_search(ix, qp, qs, 301)
    check_batch(planes, scales, qp, qs, 301, ids, sc)
    assert np.all(ids[:, 300] == -1)
    ids, sc = rbe.rbe_search(ix, qp, qs, 300)
    check_batch(planes, scales, qp, qs, 300, ids, sc)
    rbe.rbe_free(ix)


# ------------------------------------------------------------------ multi-level plan and the slow path
def test_multi_level_plan_small_capacity():
    planes, scales, qp, qs = clustered(300_000, 64, 3, 64, 0.3, 4, 3, seed=1)
    ix = load_with_ratio(planes, scales, 8)
    rbe.rbe_set_tuning(ix, cand_capacity=6144)
    ids, sc = rbe.rbe_search(ix, qp, qs, 100)
    st = rbe.rbe_get_search_stats(ix)
    assert st["n_levels"] >= 3 and not st["fallback"]
    check_batch(planes, scales, qp, qs, 100, ids, sc)
    rbe.rbe_free(ix)


def test_overflow_takes_bounded_segment_path_and_stays_exact():
    # every tile the coarse levels sample holds only weak items, so their threshold
    # prunes nothing and the finer level overflows the (tiny) candidate list
    rng = np.random.default_rng(6)
    N = 200_000
    planes, scales = random_corpus(rng, N, 64, 2)
    tile = np.arange(N) // 1024
    scales[:, tile % 8 == 0] *= np.float32(1e-3)
    qp, qs = random_queries(rng, 2, 64, 2)
    ix = load_with_ratio(planes, scales, 8)
    rbe.rbe_set_tuning(ix, cand_capacity=6144)
    ids, sc = rbe.rbe_search(ix, qp, qs, 50)
    assert rbe.rbe_get_search_stats(ix)["fallback"] == 1
    check_batch(planes, scales, qp, qs, 50, ids, sc)
    rbe.rbe_free(ix)


@pytest.mark.parametrize("ratio,cap", [(2, 2048), (3, 4096), (16, 8192), (64, 0), (4096, 0)])
def test_sample_ratios(ratio, cap):
    planes, scales, qp, qs = clustered(150_001, 64, 3, 32, 0.3, 3, 3, seed=8)
    ix = load_with_ratio(planes, scales, ratio)
    if cap:
        rbe.rbe_set_tuning(ix, cand_capacity=cap)
    ids, sc = rbe.rbe_search(ix, qp, qs, 64)
    check_batch(planes, scales, qp, qs, 64, ids, sc)
    got = rbe.rbe_debug_popcounts(ix, qp[0], 0, 150_001)
    np.testing.assert_array_equal(got, oracle.popcounts(planes, qp[0]))
    rbe.rbe_free(ix)


# ------------------------------------------------------------------ adversarial orders and ties
def test_all_items_identical():
    N, k = 50_000, 200
    one_p = np.array([0x0123456789ABCDEF], dtype=np.uint64)
    planes = np.broadcast_to(one_p, (3, N, 1)).copy()
    scales = np.full((3, N), 0.25, dtype=np.float32)
    qp = planes[:, :1].transpose(1, 0, 2).copy()
    qs = np.full((1, 3), 0.5, dtype=np.float32)
    ix = rbe.rbe_load_corpus(planes, scales)
    ids, sc = rbe.rbe_search(ix, qp, qs, k)
    np.testing.assert_array_equal(ids[0], np.arange(k))        # all tie: lowest ids win, in order
    assert np.all(sc[0] == sc[0][0])
    rbe.rbe_free(ix)


@pytest.mark.parametrize("order", ["ascending", "descending"])
def test_items_sorted_by_score(order):
    planes, scales, qp, qs = clustered(120_000, 64, 3, 32, 0.3, 1, 3, seed=2)
    s = oracle.scores(planes, scales, qp[0], qs[0])
    perm = np.argsort(s if order == "ascending" else -s, kind="stable")
    planes, scales = np.ascontiguousarray(planes[:, perm]), np.ascontiguousarray(scales[:, perm])
    ix = rbe.rbe_load_corpus(planes, scales)
    ids, sc = rbe.rbe_search(ix, qp, qs, 500)
    check_batch(planes, scales, qp, qs, 500, ids, sc)
    rbe.rbe_free(ix)


def test_topk_inside_one_wave_row():
    rng = np.random.default_rng(8)
    N, k = 100_000, 100
    planes, scales = random_corpus(rng, N, 64, 3)
    qp, qs = random_queries(rng, 1, 64, 3)
    # plant k near-copies of the query in one 256-item row that no coarse level samples
    start = 1024 * 37 + 256 * 2
    planes[:, start:start + k, 0] = qp[0][:, None, 0][:3]
    scales[:, start:start + k] = rng.uniform(2.0, 3.0, size=(3, k)).astype(np.float32)
    ix = rbe.rbe_load_corpus(planes, scales)
    ids, sc = rbe.rbe_search(ix, qp, qs, k)
    assert set(ids[0].tolist()) == set(range(start, start + k))
    check_batch(planes, scales, qp, qs, k, ids, sc)
    rbe.rbe_free(ix)


def test_duplicates_and_permutation_invariance():
    x = rbe_synth.near_duplicates_numpy(40_000, 64, 50, seed=3)
    planes, scales = oracle.encode(x, 3)
    qp, qs = oracle.encode(x[:2], 3)
    qp, qs = np.ascontiguousarray(qp.transpose(1, 0, 2)), np.ascontiguousarray(qs.T)
    ix = rbe.rbe_load_corpus(planes, scales)
    ids, sc = rbe.rbe_search(ix, qp, qs, 1500)
    check_batch(planes, scales, qp, qs, 1500, ids, sc)
    rbe.rbe_free(ix)
    perm = np.random.default_rng(9).permutation(40_000)
    ix2 = rbe.rbe_load_corpus(np.ascontiguousarray(planes[:, perm]), np.ascontiguousarray(scales[:, perm]))
    ids2, sc2 = rbe.rbe_search(ix2, qp, qs, 1500)
    np.testing.assert_array_equal(sc2, sc)                      # same multiset of scores, bit for bit
    rbe.rbe_free(ix2)


# ------------------------------------------------------------------ loading paths
def test_chunked_and_device_loading():
    import torch
    rng = np.random.default_rng(10)
    N = 10_000
    planes, scales = random_corpus(rng, N, 128, 3)
    qp, qs = random_queries(rng, 2, 128, 3)
    ix = rbe.rbe_index_create(N, 128, 3)
    with pytest.raises(rbe.RbeError):
        rbe.rbe_search(ix, qp, qs, 5)                            # not finalized
    cuts = [0, 1, 1023, 4096, 7777, N]
    for a, b in zip(cuts[:-1], cuts[1:]):
        if (a // 1000) % 2:
            rbe.rbe_load_chunk(ix, a, planes[:, a:b], scales[:, a:b])
        else:
            tp = torch.from_numpy(planes[:, a:b].view(np.int64).copy()).cuda()
            ts = torch.from_numpy(scales[:, a:b].copy()).cuda()
            rbe.rbe_load_chunk(ix, a, tp, ts)
    with pytest.raises(rbe.RbeError):
        rbe.rbe_load_chunk(ix, N - 5, planes[:, :10], scales[:, :10])   # out of range
    rbe.rbe_finalize(ix)
    with pytest.raises(rbe.RbeError):
        rbe.rbe_load_chunk(ix, 0, planes[:, :10], scales[:, :10])       # after finalize
    ids, sc = rbe.rbe_search(ix, qp, qs, 64)
    check_batch(planes, scales, qp, qs, 64, ids, sc)
    rbe.rbe_free(ix)


def test_cosine_flag_folds_item_norm():
    planes, scales, qp, qs = clustered(30_000, 64, 3, 16, 0.3, 2, 3, seed=4)
    scales = (scales * np.random.default_rng(11).uniform(0.2, 5.0, size=scales.shape[1]).astype(np.float32)[None])
    ix = rbe.rbe_load_corpus(planes, scales, flags=rbe.RBE_COSINE)
    folded = oracle.fold_cosine(planes, scales)
    np.testing.assert_allclose(rbe.rbe_debug_read_scales(ix, 0, 30_000), folded, rtol=2e-7)
    ids, sc = rbe.rbe_search(ix, qp, qs, 100)
    check_batch(planes, folded, qp, qs, 100, ids, sc)
    rbe.rbe_free(ix)


def test_paper_operating_point_dyadic_weights_asymmetric():
    """rbe*: 3 query vectors, 2 keyword vectors, weights 2^-t, stored inverse norm."""
    rng = np.random.default_rng(12)
    N = 150_000
    planes = rng.integers(0, 2**64, size=(2, N, 1), dtype=np.uint64)
    weights = np.array([[1.0], [0.5]], dtype=np.float32) * np.ones((2, N), dtype=np.float32)
    qp = rng.integers(0, 2**64, size=(4, 3, 1), dtype=np.uint64)
    qs = np.tile(np.array([1.0, 0.5, 0.25], dtype=np.float32), (4, 1))
    ix = rbe.rbe_load_corpus(planes, weights, flags=rbe.RBE_COSINE)
    ids, sc = rbe.rbe_search(ix, qp, qs, 1000)
    check_batch(planes, oracle.fold_cosine(planes, weights), qp, qs, 1000, ids, sc)
    rbe.rbe_free(ix)
    # without the norm the scores are small dyadic rationals: massive exact ties
    ix = rbe.rbe_load_corpus(planes, weights)
    ids, sc = rbe.rbe_search(ix, qp, qs, 1000)
    check_batch(planes, weights, qp, qs, 1000, ids, sc)
    for q in range(4):      # exact arithmetic on both sides: identical ids
        o_ids, o_sc = oracle.topk(planes, weights, qp[q], qs[q], 1000)
        np.testing.assert_array_equal(ids[q], o_ids)
        np.testing.assert_array_equal(sc[q].astype(np.float64), o_sc)
    rbe.rbe_free(ix)


# ------------------------------------------------------------------ paper-shaped configurations
def test_config_1M_d64_k100():
    planes, scales, qp, qs = clustered(1_000_000, 64, 3, 256, 0.3, 1, 3)
    ix = rbe.rbe_load_corpus(planes, scales)
    ids, sc = rbe.rbe_search(ix, qp, qs, 100)
    check_batch(planes, scales, qp, qs, 100, ids, sc)
    assert not rbe.rbe_get_search_stats(ix)["fallback"]
    rbe.rbe_free(ix)


def test_config_1M_cluster_sorted_ids():
    planes, scales, qp, qs = clustered(1_000_000, 64, 3, 256, 0.3, 4, 3, seed=5, sort_by_cluster=True)
    ix = rbe.rbe_load_corpus(planes, scales)
    ids, sc = rbe.rbe_search(ix, qp, qs, 1000)
    check_batch(planes, scales, qp, qs, 1000, ids, sc)
    rbe.rbe_free(ix)


def test_config_d128_4planes_batch():
    planes, scales, qp, qs = clustered(400_000, 128, 4, 512, 0.3, 16, 4, seed=6)
    ix = rbe.rbe_load_corpus(planes, scales)
    ids, sc = rbe.rbe_search(ix, qp, qs, 1000)
    check_batch(planes, scales, qp, qs, 1000, ids, sc)
    rbe.rbe_free(ix)


def test_near_duplicate_clusters_k4000():
    planes, scales, qp, qs = clustered(600_000, 64, 3, 64, 0.05, 8, 3, seed=7)
    ix = rbe.rbe_load_corpus(planes, scales)
    ids, sc = rbe.rbe_search(ix, qp, qs, 4000)
    check_batch(planes, scales, qp, qs, 4000, ids, sc)
    rbe.rbe_free(ix)


# ------------------------------------------------------------------ near-lossless selection (Algorithm 1, queue length 1)
@pytest.mark.parametrize("N,I,Q,k", [(1000, 1, 1, 50), (1000, 3, 2, 50), (65536, 256, 1, 100), (70001, 256, 3, 300),
                                     (70001, 16, 5, 1000), (300_000, 4, 1, 1000), (300_000, 255, 8, 64),
                                     (5000, 256, 2, 300)])
def test_nearlossless_matches_oracle(N, I, Q, k):
    rng = np.random.default_rng(N + I + Q + k)
    planes, scales = random_corpus(rng, N, 64, 3)
    qp, qs = random_queries(rng, Q, 64, 3)
    ix = rbe.rbe_load_corpus(planes, scales)
    ids, sc = nl_search(ix, qp, qs, k, group_size_I=I)
    for q in range(Q):
        check_nearlossless(planes, scales, qp[q], qs[q], k, I, ids[q], sc[q])
    if I == 1:      # every item is its own group: the selector is exact
        check_batch(planes, scales, qp, qs, k, ids, sc)
    rbe.rbe_free(ix)


@pytest.mark.parametrize("d,P,Pq", [(128, 4, 4), (128, 2, 3), (256, 2, 2), (64, 1, 1)])
def test_nearlossless_shapes(d, P, Pq):
    planes, scales, qp, qs = clustered(200_003, d, P, 64, 0.3, 6, Pq, seed=9)
    ix = rbe.rbe_load_corpus(planes, scales)
    ids, sc = nl_search(ix, qp, qs, 200)   # I = 256 by default
    for q in range(6):
        check_nearlossless(planes, scales, qp[q], qs[q], 200, 256, ids[q], sc[q])
    rbe.rbe_free(ix)


def test_nearlossless_exact_ties_pick_lowest_id():
    N = 100_000
    one = np.array([0x0F0F0F0F0F0F0F0F], dtype=np.uint64)
    planes = np.broadcast_to(one, (2, N, 1)).copy()
    scales = np.full((2, N), 0.5, dtype=np.float32)
    qp = planes[:, :1].transpose(1, 0, 2).copy()
    qs = np.ones((1, 2), dtype=np.float32)
    ix = rbe.rbe_load_corpus(planes, scales)
    ids, sc = nl_search(ix, qp, qs, 300, group_size_I=256)
    o_ids, _ = oracle.nearlossless(planes, scales, qp[0], qs[0], 300, I=256)
    np.testing.assert_array_equal(ids[0], o_ids)     # all scores equal and exact: winners are the lowest ids
    rbe.rbe_free(ix)


def test_nearlossless_multi_level_and_slow_path():
    planes, scales, qp, qs = clustered(1_200_000, 64, 3, 128, 0.3, 2, 3, seed=10)
    ix = load_with_ratio(planes, scales, 8)
    rbe.rbe_set_tuning(ix, cand_capacity=6144)
    ids, sc = nl_search(ix, qp, qs, 100, group_size_I=16)
    # 6144 slots: the per-thread-queue scan samples super-blocks and gets by in several levels; the coarsest tile
    # sample of the exact plan (19 tiles) does not fit, so selection by groups runs on the bounded-segment path
    assert NL_STATS["queue"]["n_levels"] >= 2 and not NL_STATS["queue"]["fallback"]
    assert NL_STATS["groups"]["fallback"] == 1
    for q in range(2):
        check_nearlossless(planes, scales, qp[q], qs[q], 100, 16, ids[q], sc[q])
    rbe.rbe_set_tuning(ix, cand_capacity=32768)          # room for the plan: several levels, each reduced by groups
    ids, sc = nl_search(ix, qp, qs, 100, group_size_I=16)
    assert NL_STATS["groups"]["n_levels"] >= 3 and not NL_STATS["groups"]["fallback"]
    for q in range(2):
        check_nearlossless(planes, scales, qp[q], qs[q], 100, 16, ids[q], sc[q])
    # a corpus whose sampled super-blocks are all weak: the threshold prunes nothing -> slow path
    rng = np.random.default_rng(13)
    N = 600_000
    planes, scales = random_corpus(rng, N, 64, 2)
    sb = np.arange(N) // (256 * 4)
    scales[:, sb % 8 == 0] *= np.float32(1e-3)
    qp, qs = random_queries(rng, 2, 64, 2)
    ix2 = load_with_ratio(planes, scales, 8)
    rbe.rbe_set_tuning(ix2, cand_capacity=6144)
    ids, sc = nl_search(ix2, qp, qs, 50, group_size_I=4)
    assert NL_STATS["queue"]["fallback"] == 1 and NL_STATS["groups"]["fallback"] == 1
    for q in range(2):
        check_nearlossless(planes, scales, qp[q], qs[q], 50, 4, ids[q], sc[q])
    rbe.rbe_free(ix); rbe.rbe_free(ix2)


@pytest.mark.parametrize("Q", [1, 3])
def test_nearlossless_many_super_blocks_per_workgroup(Q):
    """More super-blocks than workgroups and a large k: every wave forwards group winners over
    many iterations, so its per-query staging queues fill up and are flushed in the middle of
    the kernel, with one query (wave-uniform queue index) and with several."""
    N, I, k = 6_000_123, 2, 4000
    rng = np.random.default_rng(99 + Q)
    planes, scales = random_corpus(rng, N, 64, 1)
    qp, qs = random_queries(rng, Q, 64, 1)
    ix = rbe.rbe_load_corpus(planes, scales)
    ids, sc = nl_search(ix, qp, qs, k, group_size_I=I)
    assert not rbe.rbe_get_search_stats(ix)["fallback"]
    for q in range(Q):
        check_nearlossless(planes, scales, qp[q], qs[q], k, I, ids[q], sc[q])
    rbe.rbe_free(ix)


def test_nearlossless_recall_tracks_appendix_a():
    """Random-order ids: recall of the GPU near-lossless selector against the GPU exact
    selector, averaged over queries, agrees with E[M]/N of Appendix A."""
    N, I, k, Q = 2_097_152, 256, 1000, 32
    planes, scales, qp, qs = clustered(N, 64, 3, 256, 0.3, Q, 3, seed=11)
    ix = rbe.rbe_load_corpus(planes, scales)
    exact, _ = rbe.rbe_search(ix, qp, qs, k)
    near, _ = nl_search(ix, qp, qs, k, group_size_I=I)
    rec = np.mean([oracle.recall(near[q], exact[q]) for q in range(Q)])
    expect = oracle.expected_recall(k, N, I)
    assert abs(rec - expect) < 4 * np.sqrt(expect * (1 - expect) / (k * Q)) + 2e-3, (rec, expect)
    rbe.rbe_free(ix)


# ------------------------------------------------------------------ the paper's own representation (RBE_DYADIC)
def dyadic_weights(P, N):
    return (np.array([2.0 ** -j for j in range(P)], dtype=np.float32)[:, None] * np.ones((P, N), dtype=np.float32))


@pytest.mark.parametrize("d,P,Pq", [(64, 2, 3), (64, 2, 2), (64, 3, 3), (64, 1, 1), (128, 3, 4), (128, 4, 2)])
def test_dyadic_scores_are_exact(d, P, Pq):
    rng = np.random.default_rng(d + P + Pq)
    N = 50_003
    planes = rng.integers(0, 2**64, size=(P, N, d // 64), dtype=np.uint64)
    qp = rng.integers(0, 2**64, size=(3, Pq, d // 64), dtype=np.uint64)
    qs = np.tile(np.array([2.0 ** -i for i in range(Pq)], dtype=np.float32), (3, 1))
    w = dyadic_weights(P, N)
    ix = rbe.rbe_load_corpus(planes, None, flags=rbe.RBE_DYADIC)
    np.testing.assert_array_equal(rbe.rbe_debug_read_scales(ix, 0, N), w)
    np.testing.assert_array_equal(rbe.rbe_debug_popcounts(ix, qp[0], 0, N), oracle.popcounts(planes, qp[0]))
    dense = rbe.rbe_debug_scores(ix, qp[0], None, 0, N)
    np.testing.assert_array_equal(dense.astype(np.float64), oracle.scores(planes, w, qp[0], qs[0]))   # exact rationals
    for q_scales in (None, qs):
        ids, sc = rbe.rbe_search(ix, qp, q_scales, 500)
        for q in range(3):
            o_ids, o_sc = oracle.topk(planes, w, qp[q], qs[q], 500)
            np.testing.assert_array_equal(ids[q], o_ids)         # exact arithmetic on both sides, massive ties
            np.testing.assert_array_equal(sc[q].astype(np.float64), o_sc)
    nl, nsc = nl_search(ix, qp[:1], None, 100, group_size_I=16)
    o_ids, o_sc = oracle.nearlossless(planes, w, qp[0], qs[0], 100, I=16)
    np.testing.assert_array_equal(nl[0], o_ids)
    np.testing.assert_array_equal(nsc[0].astype(np.float64), o_sc)
    with pytest.raises(rbe.RbeError):
        rbe.rbe_search(ix, qp, qs * np.float32(1.5), 10)       # query scales must be the dyadic weights
    rbe.rbe_free(ix)


@pytest.mark.parametrize("d,P,Pq", [(64, 2, 3), (128, 3, 3)])
def test_dyadic_with_stored_inverse_norm(d, P, Pq):
    """rbe*-style: weights 2^-t, one stored inverse norm per keyword (Sec. 5.1)."""
    rng = np.random.default_rng(7 * d + P + Pq)
    N = 120_000
    planes = rng.integers(0, 2**64, size=(P, N, d // 64), dtype=np.uint64)
    qp = rng.integers(0, 2**64, size=(5, Pq, d // 64), dtype=np.uint64)
    qs = np.tile(np.array([2.0 ** -i for i in range(Pq)], dtype=np.float32), (5, 1))
    folded = oracle.fold_cosine(planes, dyadic_weights(P, N))
    ix = rbe.rbe_load_corpus(planes, None, flags=rbe.RBE_DYADIC | rbe.RBE_COSINE)
    np.testing.assert_array_equal(rbe.rbe_debug_read_scales(ix, 0, N), folded)    # same double norm, same rounding
    dense = rbe.rbe_debug_scores(ix, qp[0], None, 0, N)
    # an exact integer combination times one fp32 factor: a single rounding on the GPU, none in the oracle
    np.testing.assert_array_equal(dense, oracle.scores(planes, folded, qp[0], qs[0]).astype(np.float32))
    ids, sc = rbe.rbe_search(ix, qp, None, 1000)                 # 5 queries: matrix-core kernel
    check_batch(planes, folded, qp, qs, 1000, ids, sc)
    rbe.rbe_debug_set_batch_path(ix, 1)                          # XOR/popcount kernel for batch and single alike
    ids, sc = rbe.rbe_search(ix, qp, None, 1000)
    check_batch(planes, folded, qp, qs, 1000, ids, sc)
    ids1, sc1 = rbe.rbe_search(ix, qp[:1], None, 1000)
    np.testing.assert_array_equal(ids1[0], ids[0])
    rbe.rbe_debug_set_batch_path(ix, 0)
    nl, nsc = nl_search(ix, qp, None, 200)
    for q in range(5):
        check_nearlossless(planes, folded, qp[q], qs[q], 200, 256, nl[q], nsc[q])
    rbe.rbe_free(ix)


def test_dyadic_unsupported_dim_and_chunked_device_load():
    import torch
    with pytest.raises(rbe.RbeError) as e:
        rbe.rbe_index_create(1000, 256, 2, rbe.RBE_DYADIC)
    assert e.value.code == rbe.RBE_EUNSUPPORTED
    rng = np.random.default_rng(3)
    N = 30_000
    planes = rng.integers(0, 2**64, size=(2, N, 1), dtype=np.uint64)
    ix = rbe.rbe_index_create(N, 64, 2, rbe.RBE_DYADIC | rbe.RBE_COSINE)
    rbe.rbe_load_chunk(ix, 0, torch.from_numpy(planes[:, :12345].view(np.int64).copy()).cuda(), None)
    rbe.rbe_load_chunk(ix, 12345, planes[:, 12345:], None)
    rbe.rbe_finalize(ix)
    qp = rng.integers(0, 2**64, size=(2, 3, 1), dtype=np.uint64)
    qs = np.tile(np.array([1.0, 0.5, 0.25], dtype=np.float32), (2, 1))
    ids, sc = rbe.rbe_search(ix, qp, None, 50)
    check_batch(planes, oracle.fold_cosine(planes, dyadic_weights(2, N)), qp, qs, 50, ids, sc)
    rbe.rbe_free(ix)


# ------------------------------------------------------------------ on-device corpus encoder
@pytest.mark.parametrize("N,d,P", [(1, 64, 1), (1000, 64, 3), (70_001, 64, 3), (33_333, 128, 4), (5_000, 256, 2)])
def test_encode_corpus_matches_oracle_encoder_bit_for_bit(N, d, P):
    import torch
    c = rbe_synth.centres_numpy(32, d)
    x = rbe_synth.vectors_numpy(N, c, 0.3, seed=20 + N)
    x[0, 3] = 0.0                                               # rho(0) = -1
    planes, scales = oracle.encode(x, P)
    ix = rbe.rbe_encode_corpus(x, P)
    np.testing.assert_array_equal(rbe.rbe_debug_read_planes(ix, 0, N), planes)
    np.testing.assert_array_equal(rbe.rbe_debug_read_scales(ix, 0, N).view(np.uint32), scales.view(np.uint32))
    rbe.rbe_free(ix)
    # chunked, from device memory, then searched
    ix = rbe.rbe_index_create(N, d, P)
    cut = N // 3
    rbe.rbe_encode_chunk(ix, 0, torch.from_numpy(x[:cut]).cuda())
    rbe.rbe_encode_chunk(ix, cut, x[cut:])
    rbe.rbe_finalize(ix)
    np.testing.assert_array_equal(rbe.rbe_debug_read_planes(ix, 0, N), planes)
    q = rbe_synth.vectors_numpy(2, c, 0.3, seed=21)
    qp = np.stack([rbe.rbe_encode_query(q[i], P)[0] for i in range(2)])
    qs = np.stack([rbe.rbe_encode_query(q[i], P)[1] for i in range(2)])
    k = min(100, N)
    ids, sc = rbe.rbe_search(ix, qp, qs, k)
    check_batch(planes, scales, qp, qs, k, ids, sc)
    rbe.rbe_free(ix)


def test_encode_chunk_rejected_for_dyadic_index():
    ix = rbe.rbe_index_create(100, 64, 2, rbe.RBE_DYADIC)
    with pytest.raises(rbe.RbeError) as e:
        rbe.rbe_encode_chunk(ix, 0, np.zeros((100, 64), np.float32))
    assert e.value.code == rbe.RBE_EUNSUPPORTED
    rbe.rbe_free(ix)


# ------------------------------------------------------------------ hybrid scoring: fp32 query x binary items
def check_topk_float(planes, scales, q, k, ids, scores):
    """Same acceptance protocol as check_topk, against the oracle's hybrid score."""
    N = planes.shape[1]
    m = min(k, N)
    assert np.all(ids[m:] == -1) and np.all(np.isneginf(scores[m:]))
    got = ids[:m]
    assert got.min() >= 0 and got.max() < N and np.unique(got).size == m
    o_ids, o_sc = oracle.topk_fq(planes, scales, q, k)
    floor = 1e-6 * float(np.sum(np.abs(q))) * float(np.max(np.sum(scales.astype(np.float64), axis=0)))
    s_k = o_sc[m - 1]
    eps = max(1e-5 * abs(s_k), floor)
    true_sc = oracle.scores_at_fq(planes, scales, q, got)
    np.testing.assert_allclose(scores[:m], true_sc, rtol=1e-5, atol=floor)
    assert np.all(true_sc >= s_k - eps)
    assert set(o_ids[:m][o_sc[:m] > s_k + eps].tolist()) <= set(got.tolist())
    sc = scores[:m]
    assert np.all(sc[:-1] >= sc[1:])
    same = sc[:-1] == sc[1:]
    assert np.all(got[:-1][same] < got[1:][same])


@pytest.mark.parametrize("N,d,P,Q,k", [(1, 64, 1, 1, 1), (5000, 64, 3, 3, 100), (150_001, 64, 3, 2, 1000),
                                       (60_000, 128, 4, 2, 300), (20_000, 256, 2, 1, 50)])
def test_float_query_search(N, d, P, Q, k):
    c = rbe_synth.centres_numpy(32, d)
    x = rbe_synth.vectors_numpy(N, c, 0.3, seed=30 + N)
    q = rbe_synth.vectors_numpy(Q, c, 0.3, seed=31)
    planes, scales = oracle.encode(x, P)
    ix = rbe.rbe_load_corpus(planes, scales)
    dense = rbe.rbe_debug_scores_float(ix, q[0], 0, N).astype(np.float64)
    ref = oracle.scores_fq(planes, scales, q[0])
    tol = 1e-6 * float(np.sum(np.abs(q[0]))) * np.sum(scales.astype(np.float64), axis=0)
    assert np.all(np.abs(dense - ref) <= np.maximum(tol, 1e-5 * np.abs(ref)))
    ids, sc = rbe.rbe_search_float(ix, q, k)
    for i in range(Q):
        check_topk_float(planes, scales, q[i], k, ids[i], sc[i])
    # near-lossless selection of fp32 queries (selection by groups over the fp32-query scans)
    I = 4
    nids, nsc = rbe.rbe_search_float(ix, q, k, mode=rbe.RBE_SELECT_NEARLOSSLESS, group_size_I=I)
    for i in range(Q):
        check_nearlossless_float(planes, scales, q[i], k, I, nids[i], nsc[i])
    rbe.rbe_debug_set_nearlossless_path(ix, 1)          # the per-thread-queue scan takes binary queries only
    with pytest.raises(rbe.RbeError) as e:
        rbe.rbe_search_float(ix, q, k, mode=rbe.RBE_SELECT_NEARLOSSLESS)
    assert e.value.code == rbe.RBE_EUNSUPPORTED
    rbe.rbe_free(ix)


def check_nearlossless_float(planes, scales, q, k, I, ids, sc, Tb=256):
    """fp32-query result of the near-lossless selector against the oracle's hybrid scores and the group
    partition of Algorithm 1 (written here with numpy): at most one result per group, each within rounding of
    its group's best score; every group whose best beats the k-th forwarded score by more than rounding is
    present; scores match; sorted; padded past the number of groups."""
    N = planes.shape[1]
    ref = oracle.scores_fq(planes, scales, q)
    z = np.arange(N)
    group = (z // (Tb * I)) * Tb + (z % Tb)
    n_groups = (-(-N // (Tb * I))) * Tb
    best = np.full(n_groups, -np.inf)
    np.maximum.at(best, group, ref)
    live = np.isfinite(best)
    m = min(k, int(live.sum()))
    assert np.all(ids[m:] == -1) and np.all(np.isneginf(sc[m:]))
    got = ids[:m]
    if m == 0:
        return
    assert got.min() >= 0 and got.max() < N and np.unique(group[got]).size == m
    tol = 1e-6 * float(np.sum(np.abs(q))) * float(np.max(np.sum(scales.astype(np.float64), axis=0)))
    s_k = np.sort(best[live])[::-1][m - 1]
    eps = max(1e-5 * abs(s_k), tol)
    np.testing.assert_allclose(sc[:m], ref[got], rtol=1e-5, atol=tol)
    assert np.all(ref[got] >= best[group[got]] - eps), "not its group's best item"
    assert np.all(ref[got] >= s_k - eps)
    must = np.flatnonzero(best > s_k + eps)
    assert set(must.tolist()) <= set(group[got].tolist()), "a group above the k-th forwarded score is missing"
    assert np.all(sc[:m][:-1] >= sc[:m][1:])


def test_float_query_on_dyadic_index_and_hybrid_beats_binary_query():
    rng = np.random.default_rng(32)
    N, d = 80_000, 64
    c = rbe_synth.centres_numpy(16, d)
    x = rbe_synth.vectors_numpy(N, c, 0.3, seed=33)
    q = rbe_synth.vectors_numpy(4, c, 0.3, seed=34)
    planes, _ = oracle.encode(x, 2)
    w = dyadic_weights(2, N)
    folded = oracle.fold_cosine(planes, w)
    ix = rbe.rbe_load_corpus(planes, None, flags=rbe.RBE_DYADIC | rbe.RBE_COSINE)
    ids, sc = rbe.rbe_search_float(ix, q, 200)
    for i in range(4):
        check_topk_float(planes, folded, q[i], 200, ids[i], sc[i])
    rbe.rbe_free(ix)
    ix = rbe.rbe_load_corpus(planes, None, flags=rbe.RBE_DYADIC)
    ids, sc = rbe.rbe_search_float(ix, q, 200)
    for i in range(4):
        check_topk_float(planes, w, q[i], 200, ids[i], sc[i])
    rbe.rbe_free(ix)


# ------------------------------------------------------------------ near-lossless selector: group size sweep, id order
@pytest.mark.parametrize("I", [64, 256, 1024])
def test_nearlossless_recall_sweep_over_group_size(I):
    N, k, Q = 2_097_152, 1000, 16
    planes, scales, qp, qs = clustered(N, 64, 3, 256, 0.3, Q, 3, seed=12)
    ix = rbe.rbe_load_corpus(planes, scales)
    exact, _ = rbe.rbe_search(ix, qp, qs, k)
    near, _ = nl_search(ix, qp, qs, k, group_size_I=I)
    rec = np.mean([oracle.recall(near[q], exact[q]) for q in range(Q)])
    expect = oracle.expected_recall(k, N, I)
    print(f"  I={I}: recall {rec:.4f}, Appendix A {expect:.4f}")
    assert abs(rec - expect) < 4 * np.sqrt(expect * (1 - expect) / (k * Q)) + 3e-3, (I, rec, expect)
    rbe.rbe_free(ix)


def test_nearlossless_assumes_random_id_order():
    """Appendix A places the relevant items uniformly at random.  With ids sorted by cluster the
    true neighbours of a query are adjacent, share groups, and the selector loses most of them;
    the exact mode is unaffected."""
    N, k = 2_097_152, 1000
    planes, scales, qp, qs = clustered(N, 64, 3, 256, 0.3, 4, 3, seed=13, sort_by_cluster=True)
    ix = rbe.rbe_load_corpus(planes, scales)
    exact, esc = rbe.rbe_search(ix, qp, qs, k)
    check_batch(planes, scales, qp, qs, k, exact, esc)
    near, _ = nl_search(ix, qp, qs, k, group_size_I=256)
    rec = np.mean([oracle.recall(near[q], exact[q]) for q in range(4)])
    print(f"  cluster-sorted ids: recall {rec:.3f} (random order would give {oracle.expected_recall(k, N, 256):.3f})")
    assert rec < 0.6
    for q in range(4):
        check_nearlossless(planes, scales, qp[q], qs[q], k, 256, near[q], _[q])
    rbe.rbe_free(ix)


# ------------------------------------------------------------------ batched scan on the matrix cores
@pytest.mark.parametrize("d,P,Pq,Q,k", [(64, 3, 3, 16, 1000), (64, 3, 3, 1, 100), (64, 2, 3, 5, 64), (64, 4, 4, 33, 500),
                                        (64, 1, 1, 64, 10), (128, 4, 4, 17, 300), (128, 2, 1, 4, 50),
                                        (64, 3, 3, 40, 200),      # three 16-query tiles: launches of 2 + 1
                                        (128, 4, 4, 64, 100)])    # two launches of 32 queries
def test_matrix_core_batch_path_matches_oracle_and_popcount_path(d, P, Pq, Q, k):
    N = 120_011
    planes, scales, qp, qs = clustered(N, d, P, 64, 0.3, Q, Pq, seed=40 + Q)
    ix = rbe.rbe_load_corpus(planes, scales)
    rbe.rbe_debug_set_batch_path(ix, 2)
    ids_m, sc_m = rbe.rbe_search(ix, qp, qs, k)
    check_batch(planes, scales, qp, qs, k, ids_m, sc_m)
    rbe.rbe_debug_set_batch_path(ix, 1)
    ids_v, sc_v = rbe.rbe_search(ix, qp, qs, k)
    check_batch(planes, scales, qp, qs, k, ids_v, sc_v)
    # the contraction only filters; what passes is scored in the arithmetic of the XOR/popcount scan,
    # so a query's result does not depend on the kernel or on how many queries share the call
    np.testing.assert_array_equal(sc_m, sc_v)
    np.testing.assert_array_equal(ids_m, ids_v)
    rbe.rbe_debug_set_batch_path(ix, 3)          # half operands (path 2 takes eight-bit integers for these queries)
    ids_h, sc_h = rbe.rbe_search(ix, qp, qs, k)
    np.testing.assert_array_equal(sc_h, sc_v)
    np.testing.assert_array_equal(ids_h, ids_v)
    rbe.rbe_debug_set_batch_path(ix, 0)          # automatic: popcount scan on the coarse levels, matrix cores last
    ids_a, sc_a = rbe.rbe_search(ix, qp, qs, k)
    np.testing.assert_array_equal(sc_a, sc_v)
    np.testing.assert_array_equal(ids_a, ids_v)
    one_i, one_s = rbe.rbe_search(ix, qp[:1], qs[:1], k)
    np.testing.assert_array_equal(one_s[0], sc_v[0])
    np.testing.assert_array_equal(one_i[0], ids_v[0])
    rbe.rbe_free(ix)


@pytest.mark.parametrize("d,P,Pq,Q,k", [(64, 3, 3, 16, 100), (64, 2, 3, 7, 50), (64, 4, 2, 9, 100), (128, 3, 3, 12, 60),
                                        (128, 4, 4, 16, 40), (64, 3, 3, 20, 30)])
def test_matrix_core_scan_on_the_lean_stream(d, P, Pq, Q, k):
    """Integer operands, up to 16 queries per launch, an index with one-byte scale copies: the last levels stream all
    planes but the last and the copies only, and read the rest for the blocks of 32 items that the first look cannot
    rule out.  Same ids and scores as with whole rows streamed (switch 2), as the XOR/popcount scan's, and the
    oracle's; the extra reads are counted.  (20 queries: a launch of two query tiles, which streams whole rows.)"""
    N = 400_003
    planes, scales, qp, qs = clustered(N, d, P, 2048, 0.3, Q, Pq, seed=300 + d + P)
    ix = load_with_ratio(planes, scales, 8)
    rbe.rbe_debug_set_plan_split(ix, 1)
    rbe.rbe_debug_set_batch_path(ix, 2)
    res = {}
    for prog in (1, 2, 0):
        rbe.rbe_debug_set_progressive(ix, prog)
        res[prog] = rbe.rbe_search(ix, qp, qs, k)
        st = rbe.rbe_get_search_stats(ix)
        assert st["scan_kernel"][-1] == "scan_batch_mfma"
        assert (st["deep_units"] > 0) == (prog == 1 and Q <= 16), (prog, st["deep_units"])
        if prog == 1 and Q <= 16:
            # 32 items of (8W + 4P) bytes per block looked at again: no block more than once
            seen = sum(st["items_scanned"]) + 32 * len(st["items_scanned"])
            assert st["deep_units"] * 8 <= seen * (8 * (d // 64) + 4 * P), (st["deep_units"], seen)
    rbe.rbe_debug_set_progressive(ix, 1)
    rbe.rbe_debug_set_batch_path(ix, 1)
    res["xor"] = rbe.rbe_search(ix, qp, qs, k)
    for key in (2, 0, "xor"):
        np.testing.assert_array_equal(res[1][0], res[key][0])
        np.testing.assert_array_equal(res[1][1], res[key][1])
    check_batch(planes, scales, qp, qs, k, res[1][0], res[1][1])
    rbe.rbe_free(ix)


@pytest.mark.parametrize("d,P,Q", [(64, 3, 3), (64, 2, 8), (128, 4, 5), (64, 3, 12)])
def test_matrix_core_scan_on_the_lean_stream_with_fp32_queries(d, P, Q):
    """Up to eight fp32 queries per call take the lean stream too (the filter's second phase is the all-planes look
    they take anyway; larger batches stream whole rows): same ids and hybrid scores as with whole rows streamed, as
    the table scan's, and the oracle's."""
    N, k = 400_003, 40
    c = rbe_synth.centres_numpy(2048, d)
    x = rbe_synth.vectors_numpy(N, c, 0.3, seed=620 + d + P)
    q = rbe_synth.vectors_numpy(Q, c, 0.3, seed=621)
    q[1] *= 1e-3
    planes, scales = oracle.encode(x, P)
    ix = load_with_ratio(planes, scales, 8)
    rbe.rbe_debug_set_plan_split(ix, 1)
    rbe.rbe_debug_set_batch_path(ix, 2)
    res = {}
    for prog in (1, 2, 0):
        rbe.rbe_debug_set_progressive(ix, prog)
        res[prog] = rbe.rbe_search_float(ix, q, k)
        st = rbe.rbe_get_search_stats(ix)
        assert st["scan_kernel"][-1] == "scan_batch_mfma"
        assert (st["deep_units"] > 0) == (prog == 1 and Q <= 8), (prog, st["deep_units"])
    rbe.rbe_debug_set_progressive(ix, 1)
    rbe.rbe_debug_set_batch_path(ix, 1)
    res["table"] = rbe.rbe_search_float(ix, q, k)
    for key in (2, 0, "table"):
        np.testing.assert_array_equal(res[1][0], res[key][0])
        np.testing.assert_array_equal(res[1][1], res[key][1])
    for i in range(Q):
        check_topk_float(planes, scales, q[i], k, res[1][0][i], res[1][1][i])
    rbe.rbe_free(ix)


def test_matrix_core_scan_on_the_lean_stream_with_scales_outside_their_copies_range():
    """Scale arrays that span twelve binades (items below the smallest one-byte code of their array) and a corpus
    that cannot be pruned (random bits, scales that do not decay: waves go back to whole rows): ids and scores equal
    those of the scan that streams whole rows."""
    N, d, P, k, Q = 300_007, 64, 3, 12, 8
    planes, scales, qp, qs = clustered(N, d, P, 1024, 0.3, Q, 3, seed=375)
    rng = np.random.default_rng(376)
    factor = rng.choice(np.array([2.0 ** -9, 2.0 ** -3, 1.0, 1.0], dtype=np.float32), size=N)
    scales = (scales * factor[None, :]).astype(np.float32)
    scales[0, rng.choice(N, 3)] *= np.float32(1.9)
    N_r = 2_000_003                  # (at one workgroup per compute unit every wave has seven or eight rows of it)
    planes_r, scales_r = random_corpus(rng, N_r, d, P)
    qp_r, qs_r = random_queries(rng, Q, d, 3)
    for pl, sc, q1, q2, hard in ((planes, scales, qp, qs, False), (planes_r, scales_r, qp_r, qs_r, True)):
        ix = load_with_ratio(pl, sc, 8)
        rbe.rbe_debug_set_plan_split(ix, 1)
        rbe.rbe_debug_set_batch_path(ix, 2)
        if hard:
            rbe.rbe_set_tuning(ix, 0, 1)
        res = {}
        for prog in (1, 2):
            rbe.rbe_debug_set_progressive(ix, prog)
            res[prog] = rbe.rbe_search(ix, q1, q2, k)
            if hard and prog == 1:
                # nearly every block is looked at again, so the waves give the lean stream up after their first rows
                st = rbe.rbe_get_search_stats(ix)
                share = st["deep_units"] * 8 / (sum(st["items_scanned"]) * (8 + 4 * P))
                assert 0.05 < share < 0.75, share
        np.testing.assert_array_equal(res[1][0], res[2][0])
        np.testing.assert_array_equal(res[1][1], res[2][1])
        check_batch(pl, sc, q1, q2, k, res[1][0], res[1][1])
        rbe.rbe_free(ix)


def test_matrix_core_batch_path_random_corpus_multi_level_and_dyadic():
    rng = np.random.default_rng(41)
    planes, scales = random_corpus(rng, 300_000, 64, 3)
    qp, qs = random_queries(rng, 12, 64, 3)
    ix = load_with_ratio(planes, scales, 8)
    rbe.rbe_set_tuning(ix, cand_capacity=6144)
    rbe.rbe_debug_set_batch_path(ix, 2)
    ids, sc = rbe.rbe_search(ix, qp, qs, 100)
    assert rbe.rbe_get_search_stats(ix)["n_levels"] >= 3
    check_batch(planes, scales, qp, qs, 100, ids, sc)
    rbe.rbe_free(ix)
    # dyadic weights: exact integers times powers of two survive the half split exactly
    planes = rng.integers(0, 2**64, size=(2, 90_000, 1), dtype=np.uint64)
    qp = rng.integers(0, 2**64, size=(20, 3, 1), dtype=np.uint64)
    qs = np.tile(np.array([1.0, 0.5, 0.25], dtype=np.float32), (20, 1))
    for flags, oscales in ((rbe.RBE_DYADIC, dyadic_weights(2, 90_000)),
                           (rbe.RBE_DYADIC | rbe.RBE_COSINE, oracle.fold_cosine(planes, dyadic_weights(2, 90_000)))):
        ix = rbe.rbe_load_corpus(planes, None, flags=flags)
        ids, sc = rbe.rbe_search(ix, qp, None, 400)          # 20 queries: matrix cores by default
        check_batch(planes, oscales, qp, qs, 400, ids, sc)
        rbe.rbe_free(ix)


@pytest.mark.parametrize("d,P,Pq,Q,cosine", [(64, 2, 3, 16, False), (64, 4, 4, 37, True), (128, 3, 4, 24, False),
                                             (128, 4, 2, 20, True), (128, 2, 2, 33, False), (64, 3, 3, 16, True),
                                             (64, 4, 3, 9, False), (64, 2, 1, 7, True), (128, 4, 3, 40, False)])
def test_matrix_core_batch_path_dyadic_is_bit_equal_to_popcount_path(d, P, Pq, Q, cosine):
    """Dyadic weights: every term of the contraction is a short dyadic fraction, so the matrix-core
    path (plane weights folded into the query operand, one accumulator chain; 16 queries per launch
    at d=128 with 3 or 4 planes, else 32) must reproduce the integer shift-add path bit for bit, ids
    included -- with eight-bit integer operands (while 2 (2^Pq - 1) 2^(P-1) <= 127: every shape here
    but 4 + 4 planes) and with one query half per component (path 3)."""
    rng = np.random.default_rng(1000 + d + P + Q)
    N, k = 70_003, 300
    planes = rng.integers(0, 2**64, size=(P, N, d // 64), dtype=np.uint64)
    qp = rng.integers(0, 2**64, size=(Q, Pq, d // 64), dtype=np.uint64)
    ix = rbe.rbe_load_corpus(planes, None, flags=rbe.RBE_DYADIC | (rbe.RBE_COSINE if cosine else 0))
    rbe.rbe_debug_set_batch_path(ix, 2)
    ids_m, sc_m = rbe.rbe_search(ix, qp, None, k)
    rbe.rbe_debug_set_batch_path(ix, 1)
    ids_v, sc_v = rbe.rbe_search(ix, qp, None, k)
    np.testing.assert_array_equal(sc_m, sc_v)
    np.testing.assert_array_equal(ids_m, ids_v)
    rbe.rbe_debug_set_batch_path(ix, 3)
    ids_h, sc_h = rbe.rbe_search(ix, qp, None, k)
    np.testing.assert_array_equal(sc_h, sc_v)
    np.testing.assert_array_equal(ids_h, ids_v)
    oscales = dyadic_weights(P, N)
    if cosine:
        oscales = oracle.fold_cosine(planes, oscales)
    qs = np.tile(np.array([2.0 ** -i for i in range(Pq)], dtype=np.float32), (Q, 1))
    check_batch(planes, oscales, qp, qs, k, ids_m, sc_m)
    rbe.rbe_free(ix)


@pytest.mark.parametrize("d,P,Pq,cosine", [(64, 2, 3, True), (64, 3, 3, False), (128, 3, 2, True), (64, 4, 4, False)])
def test_matrix_core_dyadic_on_a_clustered_corpus_with_tight_thresholds(d, P, Pq, cosine):
    """Several levels on a clustered corpus, dyadic weights: the last levels start from tight thresholds, so the
    first look (last plane left out) rules most blocks out and the second look scores the rest exactly.  Integer
    operands, half operands and the shift-add scan give the same ids and scores."""
    N, k, Q = 400_003, 50, 12
    c = rbe_synth.centres_numpy(2048, d)
    x = rbe_synth.vectors_numpy(N, c, 0.3, seed=500 + d + P)
    planes, _ = oracle.encode(x, P)
    qpl, _ = oracle.encode(rbe_synth.vectors_numpy(Q, c, 0.3, seed=501), Pq)
    qp = np.ascontiguousarray(qpl.transpose(1, 0, 2))
    oscales = dyadic_weights(P, N)
    if cosine:
        oscales = oracle.fold_cosine(planes, oscales)
    ix = load_with_ratio(planes, None, 8, flags=rbe.RBE_DYADIC | (rbe.RBE_COSINE if cosine else 0))
    res = {}
    for path in (2, 3, 1):
        rbe.rbe_debug_set_batch_path(ix, path)
        res[path] = rbe.rbe_search(ix, qp, None, k)
        st = rbe.rbe_get_search_stats(ix)
        assert st["n_levels"] >= 3
        assert (st["scan_kernel"][-1] == "scan_batch_mfma") == (path != 1)
    for path in (3, 1):
        np.testing.assert_array_equal(res[2][0], res[path][0])
        np.testing.assert_array_equal(res[2][1], res[path][1])
    qs = np.tile(np.array([2.0 ** -i for i in range(Pq)], dtype=np.float32), (Q, 1))
    check_batch(planes, oscales, qp, qs, k, res[2][0], res[2][1])
    # integer operands take the lean stream (the last plane is read only for the blocks the first look cannot rule
    # out); with the pruning switched down or off the same scan streams whole rows: same results
    rbe.rbe_debug_set_batch_path(ix, 2)
    fits = 2 * (2 ** Pq - 1) * 2 ** (P - 1) <= 127
    for prog in (1, 2, 0):
        rbe.rbe_debug_set_progressive(ix, prog)
        got = rbe.rbe_search(ix, qp, None, k)
        assert (rbe.rbe_get_search_stats(ix)["deep_units"] > 0) == (prog == 1 and fits)
        np.testing.assert_array_equal(got[0], res[2][0])
        np.testing.assert_array_equal(got[1], res[2][1])
    rbe.rbe_free(ix)


# ------------------------------------------------------------------ near-lossless selection, priority queues of length 2
@pytest.mark.parametrize("N,I,Q,k,d,P", [(1000, 3, 2, 50, 64, 3), (65536, 256, 1, 100, 64, 3), (70001, 16, 5, 1000, 64, 2),
                                         (300_000, 4, 3, 1000, 64, 3), (5000, 256, 2, 300, 64, 3), (200_003, 256, 4, 200, 128, 4),
                                         (90_000, 64, 2, 150, 256, 2), (6_000_123, 2, 1, 4000, 64, 1)])
def test_nearlossless_queue_length_two_matches_oracle(N, I, Q, k, d, P):
    rng = np.random.default_rng(2 * N + I + Q + k)
    planes, scales = random_corpus(rng, N, d, P)
    qp, qs = random_queries(rng, Q, d, P)
    ix = rbe.rbe_load_corpus(planes, scales)
    ids, sc = nl_search(ix, qp, qs, k, mode=rbe.RBE_SELECT_NEARLOSSLESS_Q2, group_size_I=I)
    for q in range(Q):
        check_nearlossless(planes, scales, qp[q], qs[q], k, I, ids[q], sc[q], queue_len=2)
    rbe.rbe_free(ix)


def test_nearlossless_queue_length_two_exact_ties_and_dyadic():
    """All scores equal: each group forwards its two lowest ids; dyadic weights: bit-equal to the oracle."""
    N = 100_000
    one = np.array([0x0F0F0F0F0F0F0F0F], dtype=np.uint64)
    planes = np.broadcast_to(one, (2, N, 1)).copy()
    scales = np.full((2, N), 0.5, dtype=np.float32)
    qp = planes[:, :1].transpose(1, 0, 2).copy()
    qs = np.ones((1, 2), dtype=np.float32)
    ix = rbe.rbe_load_corpus(planes, scales)
    ids, sc = nl_search(ix, qp, qs, 700, mode=rbe.RBE_SELECT_NEARLOSSLESS_Q2, group_size_I=256)
    o_ids, _ = oracle.nearlossless(planes, scales, qp[0], qs[0], 700, I=256, queue_len=2)
    np.testing.assert_array_equal(ids[0], o_ids)
    rbe.rbe_free(ix)
    rng = np.random.default_rng(77)
    planes = rng.integers(0, 2**64, size=(2, 150_000, 1), dtype=np.uint64)
    qp = rng.integers(0, 2**64, size=(3, 3, 1), dtype=np.uint64)
    qs = np.tile(np.array([1.0, 0.5, 0.25], dtype=np.float32), (3, 1))
    ix = rbe.rbe_load_corpus(planes, None, flags=rbe.RBE_DYADIC)
    ids, sc = nl_search(ix, qp, None, 300, mode=rbe.RBE_SELECT_NEARLOSSLESS_Q2, group_size_I=32)
    for q in range(3):
        o_ids, o_sc = oracle.nearlossless(planes, dyadic_weights(2, 150_000), qp[q], qs[q], 300, I=32, queue_len=2)
        np.testing.assert_array_equal(ids[q], o_ids)
        np.testing.assert_array_equal(sc[q], o_sc.astype(np.float32))
    rbe.rbe_free(ix)


def test_nearlossless_queue_length_two_recall():
    """Same corpus and queries as the Appendix A check above: the second queue entry removes nearly all
    of the loss, as the hypergeometric model of the oracle predicts; a multi-level plan is exercised too."""
    N, I, k, Q = 2_097_152, 256, 1000, 32
    planes, scales, qp, qs = clustered(N, 64, 3, 256, 0.3, Q, 3, seed=11)
    ix = rbe.rbe_load_corpus(planes, scales)
    exact, _ = rbe.rbe_search(ix, qp, qs, k)
    near1, _ = nl_search(ix, qp, qs, k, group_size_I=I)
    near2, _ = nl_search(ix, qp, qs, k, mode=rbe.RBE_SELECT_NEARLOSSLESS_Q2, group_size_I=I)
    r1 = np.mean([oracle.recall(near1[q], exact[q]) for q in range(Q)])
    r2 = np.mean([oracle.recall(near2[q], exact[q]) for q in range(Q)])
    e2 = oracle.expected_recall(k, N, I, queue_len=2)
    assert r2 > r1 and e2 > 0.99
    assert abs(r2 - e2) < 4 * np.sqrt(e2 * (1 - e2) / (k * Q)) + 2e-3, (r2, e2)
    rbe.rbe_free(ix)


# ------------------------------------------------------------------ measurement yardsticks
@pytest.mark.parametrize("n_vec", [1, 255, 2048, 2049, 1_000_003])
def test_read_yardstick_touches_every_vector(n_vec):
    """calib_read folds every 16-byte vector of the source exactly once (XOR), ragged tail included."""
    import torch
    rng = np.random.default_rng(n_vec)
    host = rng.integers(0, 2**32, size=(n_vec, 4), dtype=np.uint32)
    src = torch.from_numpy(host.view(np.int32)).cuda()
    sink = torch.zeros(8 << 20, dtype=torch.uint8, device="cuda:0")
    rbe.rbe_debug_read(src, sink)
    torch.cuda.synchronize()
    folded = sink.cpu().numpy().view(np.uint32).reshape(-1, 4)
    np.testing.assert_array_equal(np.bitwise_xor.reduce(folded, axis=0), np.bitwise_xor.reduce(host, axis=0))
    dst = torch.empty_like(src)
    rbe.rbe_debug_copy(dst, src)
    torch.cuda.synchronize()
    assert torch.equal(dst, src)


# ------------------------------------------------------------------ hybrid scoring, batches on the matrix cores
@pytest.mark.parametrize("N,d,P,Q,k", [(150_001, 64, 3, 16, 500), (60_000, 128, 4, 5, 300), (80_000, 64, 2, 40, 100),
                                       (1, 64, 1, 4, 1)])
def test_float_query_batches_use_the_matrix_cores_and_match_the_table_path(N, d, P, Q, k):
    """Three or more fp32 queries per call are filtered by one dense contraction (the query itself is the
    left operand) instead of one table pass per query; both must pass the oracle's hybrid score."""
    c = rbe_synth.centres_numpy(32, d)
    x = rbe_synth.vectors_numpy(N, c, 0.3, seed=60 + N % 97)
    q = rbe_synth.vectors_numpy(Q, c, 0.3, seed=61)
    q[0] *= 37.5                       # scores scale with the query; the power-of-two scaling must follow
    planes, scales = oracle.encode(x, P)
    ix = rbe.rbe_load_corpus(planes, scales)
    ids_m, sc_m = rbe.rbe_search_float(ix, q, k)
    rbe.rbe_debug_set_batch_path(ix, 1)
    ids_t, sc_t = rbe.rbe_search_float(ix, q, k)
    for i in range(Q):
        check_topk_float(planes, scales, q[i], k, ids_m[i], sc_m[i])
        check_topk_float(planes, scales, q[i], k, ids_t[i], sc_t[i])
    # the contraction only filters; what passes is scored from the byte tables, so both paths agree bit for bit
    np.testing.assert_array_equal(sc_m, sc_t)
    np.testing.assert_array_equal(ids_m, ids_t)
    rbe.rbe_debug_set_batch_path(ix, 3)            # half operands (the default contracts eight-bit integers)
    ids_h, sc_h = rbe.rbe_search_float(ix, q, k)
    np.testing.assert_array_equal(sc_h, sc_t)
    np.testing.assert_array_equal(ids_h, ids_t)
    rbe.rbe_debug_set_batch_path(ix, 0)
    # components 2^-30 of the largest one (their operand halves would be subnormal) and a zero query
    q2 = q.copy()
    q2[1, ::3] *= 2.0 ** -30
    q2[2] = 0.0
    rbe.rbe_debug_set_batch_path(ix, 0)
    ids_m, sc_m = rbe.rbe_search_float(ix, q2, k)
    rbe.rbe_debug_set_batch_path(ix, 1)
    ids_t, sc_t = rbe.rbe_search_float(ix, q2, k)
    np.testing.assert_array_equal(sc_m, sc_t)
    np.testing.assert_array_equal(ids_m, ids_t)
    for i in range(min(Q, 3)):
        check_topk_float(planes, scales, q2[i], k, ids_m[i], sc_m[i])
    rbe.rbe_free(ix)
    # dyadic index: the one-half kernels cannot carry a full-precision query; the table path serves any batch
    rng = np.random.default_rng(62)
    dplanes = rng.integers(0, 2**64, size=(2, 50_000, d // 64), dtype=np.uint64) if d <= 128 else None
    if dplanes is not None:
        ixd = rbe.rbe_load_corpus(dplanes, None, flags=rbe.RBE_DYADIC)
        ids, sc = rbe.rbe_search_float(ixd, q[:6], 50)
        for i in range(min(6, Q)):
            check_topk_float(dplanes, dyadic_weights(2, 50_000), q[i], 50, ids[i], sc[i])
        rbe.rbe_free(ixd)


# ------------------------------------------------------------------ a query's result does not depend on its batch
@pytest.mark.parametrize("d,P,Pq,flags", [(64, 3, 3, 0), (128, 4, 3, 0), (64, 2, 3, "dyadic"), (128, 3, 2, "dyadic_cosine")])
def test_results_are_identical_for_every_batch_size(d, P, Pq, flags):
    """Exact mode: ids and scores of a query are the same bit for bit whether it is searched alone (one-query
    scan), in a small batch (XOR/popcount batch scan) or in a large one (matrix-core filter + exact rescoring,
    one or several launches per level)."""
    N, k = 180_017, 400
    rng = np.random.default_rng(4242 + d + P)
    if flags == 0:
        planes, scales, qp, qs = clustered(N, d, P, 48, 0.3, 40, Pq, seed=70 + d)
        ix = rbe.rbe_load_corpus(planes, scales)
    else:
        planes = rng.integers(0, 2**64, size=(P, N, d // 64), dtype=np.uint64)
        qp = rng.integers(0, 2**64, size=(40, Pq, d // 64), dtype=np.uint64)
        qs = None
        ix = rbe.rbe_load_corpus(planes, None, flags=rbe.RBE_DYADIC | (rbe.RBE_COSINE if flags == "dyadic_cosine" else 0))
    ref_ids, ref_sc = [], []
    for q in range(40):
        i, s = rbe.rbe_search(ix, qp[q:q + 1], None if qs is None else qs[q:q + 1], k)
        ref_ids.append(i[0]); ref_sc.append(s[0])
    ref_ids = np.stack(ref_ids); ref_sc = np.stack(ref_sc)
    for Q in (2, 3, 7, 8, 9, 16, 17, 33, 40):
        ids, sc = rbe.rbe_search(ix, qp[:Q], None if qs is None else qs[:Q], k)
        np.testing.assert_array_equal(sc, ref_sc[:Q], err_msg=f"scores differ at batch size {Q}")
        np.testing.assert_array_equal(ids, ref_ids[:Q], err_msg=f"ids differ at batch size {Q}")
    rbe.rbe_free(ix)


# ------------------------------------------------------------------ seeded sweep over shapes and modes
@pytest.mark.parametrize("seed", list(range(24)))
def test_random_shapes_and_modes(seed):
    """Seeded draw of corpus size (ragged tails, below and above one tile), dimension, plane counts,
    batch size, k, selection mode and group size; every case against the oracle."""
    rng = np.random.default_rng(9000 + seed)
    d = int(rng.choice([64, 64, 128, 256]))
    P = int(rng.integers(1, 5)); Pq = int(rng.integers(1, 5))
    N = int(rng.choice([1, 63, 1024, 1025, 4097, 30_011, 131_072, 250_003]))
    Q = int(rng.choice([1, 2, 5, 8, 13, 16, 31, 64]))
    k = int(rng.choice([1, 10, 100, 1000, 4096]))
    mode = int(rng.choice([rbe.RBE_SELECT_EXACT, rbe.RBE_SELECT_EXACT, rbe.RBE_SELECT_NEARLOSSLESS, rbe.RBE_SELECT_NEARLOSSLESS_Q2]))
    I = int(rng.choice([1, 2, 7, 64, 256]))
    dyadic = bool(rng.integers(0, 3) == 0) and d <= 128
    planes = rng.integers(0, 2**64, size=(P, N, d // 64), dtype=np.uint64)
    qp = rng.integers(0, 2**64, size=(Q, Pq, d // 64), dtype=np.uint64)
    if dyadic:
        scales, flags = dyadic_weights(P, N), rbe.RBE_DYADIC
        qs = np.tile(np.array([2.0 ** -i for i in range(Pq)], dtype=np.float32), (Q, 1))
        ix = rbe.rbe_load_corpus(planes, None, flags=flags)
    else:
        scales = rng.uniform(0.01, 1.0, size=(P, N)).astype(np.float32)
        qs = rng.uniform(0.01, 1.0, size=(Q, Pq)).astype(np.float32)
        ix = rbe.rbe_load_corpus(planes, scales)
    label = f"d={d} P={P} Pq={Pq} N={N} Q={Q} k={k} mode={mode} I={I} dyadic={dyadic}"
    print(label, flush=True)
    ids, sc = rbe.rbe_search(ix, qp, None if dyadic else qs, k, mode=mode, group_size_I=I)
    if mode == rbe.RBE_SELECT_EXACT:
        check_batch(planes, scales, qp, qs, k, ids, sc)
    else:
        for q in range(min(Q, 6)):
            check_nearlossless(planes, scales, qp[q], qs[q], k, I, ids[q], sc[q],
                               queue_len=2 if mode == rbe.RBE_SELECT_NEARLOSSLESS_Q2 else 1)
    rbe.rbe_free(ix)


@pytest.mark.parametrize("seed", list(range(10)))
def test_random_shapes_every_scan_gives_the_same_lists(seed):
    """Seeded draw of shape, corpus kind (clustered; clustered with scales over twelve binades; random bits;
    dyadic weights), batch size and sample ratio: the search under every combination of the switches -- last level
    whole or in two parts, XOR/popcount or matrix cores (integer or half operands), pruning scans on, without scale
    copies, without the first stage, off -- returns the same ids and scores bit for bit, which are the oracle's."""
    rng = np.random.default_rng(7700 + seed)
    d = int(rng.choice([64, 64, 128])); P = int(rng.choice([2, 3, 3, 4])); Pq = int(rng.integers(1, 5))
    N = int(rng.integers(60_000, 300_000)); k = int(rng.choice([1, 10, 100, 300])); Q = int(rng.choice([1, 2, 3, 4, 5, 9, 16, 20, 33]))
    ratio = int(rng.choice([4, 8, 16])); ncl = int(rng.choice([64, 1024])); sigma = float(rng.choice([0.05, 0.3, 1.0]))
    kind = seed % 4
    c = rbe_synth.centres_numpy(ncl, d)
    if kind == 2:
        planes, scales = random_corpus(rng, N, d, P); qp, qs = random_queries(rng, Q, d, Pq)
    else:
        planes, scales, qp, qs = clustered(N, d, P, ncl, sigma, Q, Pq, seed=7800 + seed)
        if kind == 1:
            f = rng.choice(np.array([2.0 ** -9, 2.0 ** -3, 1.0, 1.0], dtype=np.float32), size=N)
            scales = (scales * f[None, :]).astype(np.float32)
    flags = 0
    if kind == 3:
        flags = rbe.RBE_DYADIC | (rbe.RBE_COSINE if seed % 8 == 3 else 0)
        scales = dyadic_weights(P, N)
        if flags & rbe.RBE_COSINE:
            scales = oracle.fold_cosine(planes, scales)
        qs = np.tile(np.array([2.0 ** -i for i in range(Pq)], dtype=np.float32), (Q, 1))
    print(f"d={d} P={P} Pq={Pq} N={N} k={k} Q={Q} ratio={ratio} clusters={ncl} sigma={sigma} kind={kind}", flush=True)
    ix = load_with_ratio(planes, None if kind == 3 else scales, ratio, flags=flags)
    ref = None
    for split in (0, 1):
        rbe.rbe_debug_set_plan_split(ix, split)
        for path in (0, 1, 2, 3):
            rbe.rbe_debug_set_batch_path(ix, path)
            for prog in (1, 2, 3, 0):
                rbe.rbe_debug_set_progressive(ix, prog)
                got = rbe.rbe_search(ix, qp, None if kind == 3 else qs, k)
                if ref is None:
                    ref = got
                else:
                    np.testing.assert_array_equal(got[0], ref[0], err_msg=f"split {split} path {path} prog {prog}")
                    np.testing.assert_array_equal(got[1], ref[1], err_msg=f"split {split} path {path} prog {prog}")
    check_batch(planes, scales, qp, qs, k, ref[0], ref[1])
    if kind != 3:
        # fp32 queries: table scan and matrix cores, every pruning switch
        x = rbe_synth.vectors_numpy(min(Q, 9), c, sigma, seed=7900 + seed)
        fref = None
        for path in (1, 2):
            rbe.rbe_debug_set_batch_path(ix, path)
            for prog in (1, 2, 3, 0):
                rbe.rbe_debug_set_progressive(ix, prog)
                got = rbe.rbe_search_float(ix, x, k)
                if fref is None:
                    fref = got
                else:
                    np.testing.assert_array_equal(got[0], fref[0], err_msg=f"float path {path} prog {prog}")
                    np.testing.assert_array_equal(got[1], fref[1], err_msg=f"float path {path} prog {prog}")
        for i in range(x.shape[0]):
            check_topk_float(planes, scales, x[i], k, fref[0][i], fref[1][i])
    rbe.rbe_free(ix)


@pytest.mark.parametrize("d", [64, 128])
def test_cancelling_query_planes_in_a_batch(d):
    """Queries whose second plane is the complement of the first, with nearly equal coefficients: the
    reconstructed query is tiny next to d * sum|c_i|, the case where the XOR/popcount arithmetic rounds at a
    magnitude far above the query's own. Batch results (matrix-core filter) still equal the one-query results
    bit for bit and pass the oracle check."""
    N, P, Q, k = 70_001, 3, 16, 300
    rng = np.random.default_rng(515 + d)
    planes = rng.integers(0, 2**64, size=(P, N, d // 64), dtype=np.uint64)
    scales = rng.uniform(0.05, 1.0, size=(P, N)).astype(np.float32)
    qp = rng.integers(0, 2**64, size=(Q, 2, d // 64), dtype=np.uint64)
    qp[:, 1] = ~qp[:, 0]
    qs = np.stack([np.full(Q, 0.7, dtype=np.float32),
                   (0.7 * (1.0 - 2.0 ** -rng.integers(3, 14, size=Q))).astype(np.float32)], axis=1)
    ix = rbe.rbe_load_corpus(planes, scales)
    ids, sc = rbe.rbe_search(ix, qp, qs, k)
    for q in range(Q):
        i1, s1 = rbe.rbe_search(ix, qp[q:q + 1], qs[q:q + 1], k)
        np.testing.assert_array_equal(sc[q], s1[0]); np.testing.assert_array_equal(ids[q], i1[0])
    check_batch(planes, scales, qp, qs, k, ids, sc)
    rbe.rbe_free(ix)


# ------------------------------------------------------------------ several indexes, streams and host threads
def test_two_indexes_searched_from_two_threads_on_their_own_streams():
    """An index is used by one thread at a time, but different indexes are independent: two host threads,
    each with its own index (different shapes) and its own stream (default priority), run searches of
    varying batch size, k and selection mode at the same time; every result against the oracle."""
    import threading
    import torch
    rng = np.random.default_rng(77)
    cases = [(90_001, 64, 3), (40_003, 128, 4)]
    data, errors = [], []
    for N, d, P in cases:
        planes, scales = random_corpus(rng, N, d, P)
        data.append((planes, scales, rbe.rbe_load_corpus(planes, scales), torch.cuda.Stream()))
    schedule = [(1, 100, rbe.RBE_SELECT_EXACT), (16, 1000, rbe.RBE_SELECT_EXACT), (3, 10, rbe.RBE_SELECT_NEARLOSSLESS),
                (40, 50, rbe.RBE_SELECT_EXACT), (2, 4096, rbe.RBE_SELECT_EXACT), (9, 300, rbe.RBE_SELECT_EXACT),
                (1, 1000, rbe.RBE_SELECT_NEARLOSSLESS_Q2), (5, 7, rbe.RBE_SELECT_EXACT)]
    results = [[], []]

    def worker(t):
        try:
            planes, scales, ix, stream = data[t]
            r = np.random.default_rng(100 + t)
            for Q, k, mode in schedule:
                qp, qs = random_queries(r, Q, 64 * planes.shape[2], 3)
                ids, sc = rbe.rbe_search(ix, qp, qs, k, mode=mode, group_size_I=4, stream=stream)
                results[t].append((qp, qs, k, mode, ids, sc))
        except Exception as e:      # noqa: BLE001 - reported by the main thread
            errors.append((t, repr(e)))

    threads = [threading.Thread(target=worker, args=(t,)) for t in range(2)]
    for th in threads:
        th.start()
    for th in threads:
        th.join()
    assert not errors, errors
    for t in range(2):
        planes, scales, ix, _ = data[t]
        assert len(results[t]) == len(schedule)
        for qp, qs, k, mode, ids, sc in results[t]:
            if mode == rbe.RBE_SELECT_EXACT:
                check_batch(planes, scales, qp, qs, k, ids, sc)
            else:
                for q in range(qp.shape[0]):
                    check_nearlossless(planes, scales, qp[q], qs[q], k, 4, ids[q], sc[q],
                                       queue_len=2 if mode == rbe.RBE_SELECT_NEARLOSSLESS_Q2 else 1)
        rbe.rbe_free(ix)


# ------------------------------------------------------------------ progressive scan (one query, last level)
def _search_both_ways(ix, qp, qs, k):
    """Every query alone, with the progressive scan on and off; returns the two result lists and the share of
    rows whose last plane was read."""
    rbe.rbe_debug_set_plan_split(ix, 1)      # no automatic choices: the switch alone decides which scan runs
    out, shares = {}, []
    for prog in (1, 2, 3, 0):        # on; on without the one-byte scale copies; on without the first stage on plane 0; off
        rbe.rbe_debug_set_progressive(ix, prog)
        res = []
        for q in range(qp.shape[0]):
            res.append(rbe.rbe_search(ix, qp[q:q + 1], None if qs is None else qs[q:q + 1], k))
            st = rbe.rbe_get_search_stats(ix)
            rows = -(-st["items_scanned"][st["n_levels"] - 1] // 256)
            if prog == 1:
                shares.append(st["deep_rows"] / rows)
            elif prog == 0:
                assert st["deep_rows"] == 0
        # the same queries two, three and four to a call (the small-batch forms of the same scans): same lists
        nq = qp.shape[0]
        for Q in (2, 3, 4):
            if Q > nq:
                break
            for b in range(0, nq - Q + 1, Q):
                ib, sb = rbe.rbe_search(ix, qp[b:b + Q], None if qs is None else qs[b:b + Q], k)
                for j in range(Q):
                    np.testing.assert_array_equal(ib[j], res[b + j][0][0], err_msg=f"prog {prog} Q {Q} query {b + j}")
                    np.testing.assert_array_equal(sb[j], res[b + j][1][0], err_msg=f"prog {prog} Q {Q} query {b + j}")
        out[prog] = res
    rbe.rbe_debug_set_progressive(ix, True)
    for (i1, s1), (i2, s2), (i3, s3) in zip(out[1], out[2], out[3]):
        np.testing.assert_array_equal(i1, i2); np.testing.assert_array_equal(s1, s2)
        np.testing.assert_array_equal(i1, i3); np.testing.assert_array_equal(s1, s3)
    return out[1], out[0], shares


@pytest.mark.parametrize("d,P,Pq,flags", [(64, 3, 3, 0), (64, 2, 3, 0), (128, 4, 4, 0), (256, 2, 2, 0), (64, 2, 3, "dyadic"),
                                          (128, 3, 2, "dyadic_cosine"), (64, 4, 1, "dyadic"), (256, 3, 2, 0), (128, 3, 1, 0), (64, 4, 2, 0)])
def test_progressive_scan_changes_nothing_but_the_bytes_read(d, P, Pq, flags):
    """One query, several levels: the last level reads the last plane only of rows that the other planes and the
    scales cannot rule out.  Ids and scores are those of the plain scan bit for bit (and pass the oracle); on a
    clustered corpus most rows are ruled out."""
    N, k, Q = 400_003, 20, 6        # 2048 clusters of about 195 items: one row in nine holds an item of the query's
    if flags == 0:
        planes, scales, qp, qs = clustered(N, d, P, 2048, 0.3, Q, Pq, seed=90 + d + P)
        ix = load_with_ratio(planes, scales, 8)
    else:
        c = rbe_synth.centres_numpy(2048, d)
        x = rbe_synth.vectors_numpy(N, c, 0.3, seed=95 + d)
        planes, _ = oracle.encode(x, P)
        qpl, _ = oracle.encode(rbe_synth.vectors_numpy(Q, c, 0.3, seed=96), Pq)
        qp, qs = np.ascontiguousarray(qpl.transpose(1, 0, 2)), None
        scales = dyadic_weights(P, N)
        fl = rbe.RBE_DYADIC | (rbe.RBE_COSINE if flags == "dyadic_cosine" else 0)
        if flags == "dyadic_cosine":
            scales = oracle.fold_cosine(planes, dyadic_weights(P, N))
        ix = load_with_ratio(planes, None, 8, flags=fl)
    on, off, shares = _search_both_ways(ix, qp, qs, k)
    for (i1, s1), (i0, s0) in zip(on, off):
        np.testing.assert_array_equal(i1, i0); np.testing.assert_array_equal(s1, s0)
    qs_o = qs if qs is not None else np.tile(np.array([2.0 ** -i for i in range(Pq)], dtype=np.float32), (Q, 1))
    for q in range(Q):
        check_topk(planes, scales, qp[q], qs_o[q], k, on[q][0][0], on[q][1][0])
    # rows of the query's own cluster are read in full, most others not (with two planes and general scales the
    # left-out plane weighs about 0.6 of the first one: the bound is correct but prunes little)
    assert 0 < np.mean(shares) < (0.5 if (P >= 3 or flags != 0) else 1.0), shares
    rbe.rbe_free(ix)


def test_progressive_scan_on_corpora_where_the_bound_cannot_help():
    """Random bits with random (non-decaying) scales, a zero query, a query whose planes cancel: the bound lets
    most rows through, waves fall back to whole rows, and the results still equal the plain scan's."""
    N, d, P, k = 300_007, 64, 3, 50
    rng = np.random.default_rng(808)
    planes, scales = random_corpus(rng, N, d, P)
    qp, qs = random_queries(rng, 5, d, 3)
    qs[1] = 0.0
    qp[2, 1] = ~qp[2, 0]; qs[2, 1] = qs[2, 0] * np.float32(1 - 2.0 ** -12); qs[2, 2] = 0.0
    qs[3] *= -1.0                                              # negative query scales: M uses |qhat|
    ix = load_with_ratio(planes, scales, 8)
    on, off, shares = _search_both_ways(ix, qp, qs, k)
    for (i1, s1), (i0, s0) in zip(on, off):
        np.testing.assert_array_equal(i1, i0); np.testing.assert_array_equal(s1, s0)
    for q in range(5):
        check_topk(planes, scales, qp[q], qs[q], k, on[q][0][0], on[q][1][0])
    rbe.rbe_free(ix)


@pytest.mark.parametrize("d,P,flags", [(64, 3, 0), (128, 4, 0), (64, 2, "dyadic"), (128, 3, "dyadic_cosine"), (64, 4, 0), (128, 3, 0)])
def test_progressive_scan_with_fp32_queries(d, P, flags):
    """Hybrid scoring, one table pass per query: the last level is progressive too, with the table sums in place of
    the popcounts; same ids and scores as with every plane read, and the oracle's hybrid score."""
    N, k, Q = 300_011, 20, 4
    c = rbe_synth.centres_numpy(2048, d)
    x = rbe_synth.vectors_numpy(N, c, 0.3, seed=120 + d)
    q = rbe_synth.vectors_numpy(Q, c, 0.3, seed=121)
    q[1] *= 1e-3
    q[2, ::2] = 0.0
    planes, scales = oracle.encode(x, P)
    if flags == 0:
        ix = load_with_ratio(planes, scales, 8)
    else:
        scales = dyadic_weights(P, N)
        if flags == "dyadic_cosine":
            scales = oracle.fold_cosine(planes, scales)
        ix = load_with_ratio(planes, None, 8, flags=rbe.RBE_DYADIC | (rbe.RBE_COSINE if flags == "dyadic_cosine" else 0))
    rbe.rbe_debug_set_batch_path(ix, 1)         # the table path for every batch size
    rbe.rbe_debug_set_plan_split(ix, 1)         # no automatic choices
    res = {}
    for prog in (1, 2, 3, 0):        # on; on without the one-byte scale copies; on without the first stage on plane 0; off
        rbe.rbe_debug_set_progressive(ix, prog)
        res[prog] = [rbe.rbe_search_float(ix, q[i:i + 1], k) for i in range(Q)] + [rbe.rbe_search_float(ix, q, k)]
        st = rbe.rbe_get_search_stats(ix)
        assert (st["deep_rows"] > 0) == (prog != 0)
    rbe.rbe_debug_set_progressive(ix, 1)
    res[True], res[False] = res[1], res[0]
    for (i1, s1), (i2, s2), (i3, s3), (i0, s0) in zip(res[1], res[2], res[3], res[0]):
        np.testing.assert_array_equal(i1, i0); np.testing.assert_array_equal(s1, s0)
        np.testing.assert_array_equal(i2, i0); np.testing.assert_array_equal(s2, s0)
        np.testing.assert_array_equal(i3, i0); np.testing.assert_array_equal(s3, s0)
    for i in range(Q):
        check_topk_float(planes, scales, q[i], k, res[True][i][0][0], res[True][i][1][0])
        np.testing.assert_array_equal(res[True][Q][0][i], res[True][i][0][0])
    rbe.rbe_free(ix)


@pytest.mark.parametrize("d,P,Pq,flags", [(64, 3, 3, 0), (128, 4, 2, 0), (64, 2, 3, "dyadic"), (128, 3, 3, "dyadic_cosine"),
                                          (64, 4, 4, 0), (128, 3, 1, 0), (256, 3, 2, 0)])
def test_progressive_scan_for_small_batches(d, P, Pq, flags):
    """A few queries per call (and any batch on the XOR/popcount kernel): the last level forms partial scores from all
    planes but the last for every query and reads a row's last plane once, for the first query that needs it.
    Same ids and scores with the switch on and off, and against the oracle."""
    N, k = 350_003, 30
    c = rbe_synth.centres_numpy(2048, d)
    x = rbe_synth.vectors_numpy(N, c, 0.3, seed=140 + d)
    planes, scales = oracle.encode(x, P)
    qpl, qsl = oracle.encode(rbe_synth.vectors_numpy(16, c, 0.3, seed=141), Pq)
    qp, qs = np.ascontiguousarray(qpl.transpose(1, 0, 2)), np.ascontiguousarray(qsl.T)
    if flags == 0:
        ix = load_with_ratio(planes, scales, 8)
    else:
        scales = dyadic_weights(P, N)
        if flags == "dyadic_cosine":
            scales = oracle.fold_cosine(planes, scales)
        ix = load_with_ratio(planes, None, 8, flags=rbe.RBE_DYADIC | (rbe.RBE_COSINE if flags == "dyadic_cosine" else 0))
        qs = None
    qs_o = qs if qs is not None else np.tile(np.array([2.0 ** -i for i in range(Pq)], dtype=np.float32), (16, 1))
    rbe.rbe_debug_set_batch_path(ix, 1)
    rbe.rbe_debug_set_plan_split(ix, 1)         # no automatic choices
    for Q in (2, 4, 5, 7, 16):       # up to 4: the scan that streams the one-byte scale copies; above: the fp32 scales
        res = {}
        for prog in (1, 3, 0):       # on (up to 4 queries and from three planes on: first stage on plane 0); on without that stage; off
            rbe.rbe_debug_set_progressive(ix, prog)
            res[prog] = rbe.rbe_search(ix, qp[:Q], None if qs is None else qs[:Q], k)
            st = rbe.rbe_get_search_stats(ix)
            assert (st["deep_rows"] > 0) == (prog != 0)
            if prog == 1 and flags == 0 and P >= 3 and Q <= 4:
                assert st["scan_kernel"][st["n_levels"] - 1] == "scan_exact_prog2_hint"
        for prog in (1, 3):
            np.testing.assert_array_equal(res[prog][0], res[0][0])
            np.testing.assert_array_equal(res[prog][1], res[0][1])
        check_batch(planes, scales, qp[:Q], qs_o[:Q], k, res[1][0], res[1][1])
    rbe.rbe_debug_set_progressive(ix, 1)
    rbe.rbe_free(ix)


def test_progressive_scan_honours_large_last_scales():
    """The one-query progressive scans do not read the last scale array; the row's largest value stands in for
    it.  A few items whose last scale is 50x the usual one (and which owe their rank to it) must still be found,
    with binary and with fp32 queries."""
    N, d, P, k = 300_007, 64, 3, 40
    c = rbe_synth.centres_numpy(2048, d)
    x = rbe_synth.vectors_numpy(N, c, 0.3, seed=160)
    planes, scales = oracle.encode(x, P)
    rng = np.random.default_rng(161)
    big = rng.choice(N, size=300, replace=False)
    scales[P - 1, big] *= 50.0
    qx = rbe_synth.vectors_numpy(4, c, 0.3, seed=162)
    qpl, qsl = oracle.encode(qx, P)
    qp, qs = np.ascontiguousarray(qpl.transpose(1, 0, 2)), np.ascontiguousarray(qsl.T)
    ix = load_with_ratio(planes, scales, 8)
    on, off, shares = _search_both_ways(ix, qp, qs, k)
    hits = 0
    for q in range(4):
        np.testing.assert_array_equal(on[q][0], off[q][0]); np.testing.assert_array_equal(on[q][1], off[q][1])
        check_topk(planes, scales, qp[q], qs[q], k, on[q][0][0], on[q][1][0])
        hits += len(set(on[q][0][0].tolist()) & set(big.tolist()))
        rbe.rbe_debug_set_batch_path(ix, 1)
        i1, s1 = rbe.rbe_search_float(ix, qx[q:q + 1], k)
        rbe.rbe_debug_set_progressive(ix, False)
        i0, s0 = rbe.rbe_search_float(ix, qx[q:q + 1], k)
        rbe.rbe_debug_set_progressive(ix, True)
        rbe.rbe_debug_set_batch_path(ix, 0)
        np.testing.assert_array_equal(i1, i0); np.testing.assert_array_equal(s1, s0)
        check_topk_float(planes, scales, qx[q], k, i1[0], s1[0])
    assert hits > 0          # the boosted items do reach the top k
    rbe.rbe_free(ix)


def test_progressive_scan_with_extreme_scales():
    """Scales across the fp32 range (1e-37 .. 1e30, zeros, subnormals): the one-byte copies (most of them the
    smallest code of their array here) still give valid bounds; ids and scores equal the plain scan's."""
    N, d, P, k = 200_003, 64, 3, 25
    rng = np.random.default_rng(171)
    planes = rng.integers(0, 2**64, size=(P, N, 1), dtype=np.uint64)
    expo = rng.integers(-37, 8, size=(P, N))
    scales = (rng.uniform(1.0, 9.99, size=(P, N)) * 10.0 ** expo).astype(np.float32)
    scales[:, rng.choice(N, 5000, replace=False)] = 0.0
    scales[1, rng.choice(N, 5000, replace=False)] = np.float32(1e-41)          # subnormal
    scales[0, :100] = np.float32(3e30)
    qp, qs = random_queries(rng, 4, d, 3)
    ix = load_with_ratio(planes, scales, 8)
    on, off, _ = _search_both_ways(ix, qp, qs, k)
    for (i1, s1), (i0, s0) in zip(on, off):
        np.testing.assert_array_equal(i1, i0); np.testing.assert_array_equal(s1, s0)
        assert np.isfinite(s1).all()
    for q in range(4):
        check_topk(planes, scales, qp[q], qs[q], k, on[q][0][0], on[q][1][0])
    rbe.rbe_free(ix)


def test_progressive_scan_with_scales_below_the_range_of_their_copies():
    """Clustered corpus whose scale arrays span twelve binades (half of the items scaled by 2^-9, below the smallest
    one-byte code of their array, a quarter by 2^-3): ids and scores equal the plain scan's, and the bound still
    prunes.  With a negative scale in the corpus the index stands every pruning scan down (their bounds assume
    scales >= 0) and the plain scan serves."""
    N, d, P, k = 300_007, 64, 3, 12      # about 145 full-scale items per cluster: the sample's threshold (8 k) lies inside
    planes, scales, qp, qs = clustered(N, d, P, 1024, 0.3, 4, 3, seed=175)
    rng = np.random.default_rng(176)
    factor = rng.choice(np.array([2.0 ** -9, 2.0 ** -3, 1.0, 1.0], dtype=np.float32), size=N)
    scales = (scales * factor[None, :]).astype(np.float32)
    scales[0, rng.choice(N, 3)] *= np.float32(1.9)           # and the largest value sits alone at the top
    for negative in (False, True):
        if negative:
            scales[0, rng.choice(N, 2000, replace=False)] *= np.float32(-1.0)
        ix = load_with_ratio(planes, scales, 8)
        info = rbe.rbe_debug_index_info(ix)
        assert info["can_prune"] == (not negative) and info["scale_copies"] == (not negative)
        on, off, shares = _search_both_ways(ix, qp, qs, k)
        for (i1, s1), (i0, s0) in zip(on, off):
            np.testing.assert_array_equal(i1, i0); np.testing.assert_array_equal(s1, s0)
        for q in range(4):
            check_topk(planes, scales, qp[q], qs[q], k, on[q][0][0], on[q][1][0])
        if negative:
            assert np.all(np.array(shares) == 0), shares
        else:
            assert 0 < np.mean(shares) < 0.5, shares
        rbe.rbe_free(ix)


def test_last_level_in_two_parts_gives_the_same_results():
    """The last level taken whole or in two parts (an eighth first): same ids and scores, one query and a batch."""
    N, d, P, k = 600_011, 64, 3, 20
    planes, scales, qp, qs = clustered(N, d, P, 6000, 0.3, 6, 3, seed=181)
    ix = load_with_ratio(planes, scales, 64)
    res = {}
    for mode in (1, 2):                       # never / always
        rbe.rbe_debug_set_plan_split(ix, mode)
        res[mode] = []
        for q in range(6):
            res[mode].append(rbe.rbe_search(ix, qp[q:q + 1], qs[q:q + 1], k))
            st = rbe.rbe_get_search_stats(ix)
            assert st["n_levels"] == (2 if mode == 1 else 3)
        b16 = rbe.rbe_search(ix, qp, qs, k)
        for q in range(6):
            np.testing.assert_array_equal(b16[0][q], res[mode][q][0][0])
    for (i1, s1), (i2, s2) in zip(res[1], res[2]):
        np.testing.assert_array_equal(i1, i2); np.testing.assert_array_equal(s1, s2)
    for q in range(6):
        check_topk(planes, scales, qp[q], qs[q], k, res[2][q][0][0], res[2][q][1][0])
    rbe.rbe_free(ix)


def test_last_level_in_two_parts_prunes_where_its_own_threshold_is_loose():
    """5 M items in clusters of about 800: ratio * k = 64 * 30 lies outside the cluster, so with the last level whole
    most rows are read in full; taken in two parts (the default for a level of this size) the scan prunes.  Same
    results either way."""
    import torch
    N, d, P, k = 5_000_000, 64, 3, 30
    centres = rbe_synth.centres_torch(6000, d, torch.device("cuda:0"))
    ix = rbe.rbe_index_create(N, d, P, 0)
    for c_, z0 in enumerate(range(0, N, 1_000_000)):
        v = rbe_synth.vectors_torch(1_000_000, centres, 0.3, rbe_synth.SEED_ITEMS, c_)
        pl, sc = rbe_synth.pack_planes_torch(v, P)
        rbe.rbe_load_chunk(ix, z0, pl, sc)
    rbe.rbe_finalize(ix)
    x = rbe_synth.vectors_torch(3, centres, 0.3, rbe_synth.SEED_QUERIES, 0).cpu().numpy()
    enc = [rbe.rbe_encode_query(x[i], P) for i in range(3)]
    qp = np.stack([e[0] for e in enc]); qs = np.stack([e[1] for e in enc])
    r1 = rbe.rbe_search(ix, qp[:1], qs[:1], k)
    st1 = rbe.rbe_get_search_stats(ix)
    rbe.rbe_debug_set_plan_split(ix, 1)
    r0 = rbe.rbe_search(ix, qp[:1], qs[:1], k)
    st0 = rbe.rbe_get_search_stats(ix)
    assert st0["last_level_parts"] == 1 and st1["last_level_parts"] == 2
    assert st1["n_levels"] == st0["n_levels"] + 1, (st0["n_levels"], st1["n_levels"])
    assert st1["deep_rows"] < st0["deep_rows"] // 2, (st0["deep_rows"], st1["deep_rows"])
    assert sum(st1["deep_rows_level"]) == st1["deep_rows"]
    np.testing.assert_array_equal(r0[0], r1[0]); np.testing.assert_array_equal(r0[1], r1[1])
    # it helped, so it stays: one-query searches drop the split only after several in a row that it did not help
    rbe.rbe_debug_set_plan_split(ix, 0)
    for i in range(8):
        rbe.rbe_search(ix, qp[i % 3:i % 3 + 1], qs[i % 3:i % 3 + 1], k)
        assert rbe.rbe_get_search_stats(ix)["last_level_parts"] == 2
    rbe.rbe_free(ix)


@pytest.mark.parametrize("P", [2, 3])
def test_a_corpus_that_cannot_be_pruned_keeps_its_pruning_scans_and_drops_the_split_for_one_query_only(P):
    """Unclustered corpus: every row has to be read in full, split or not.  With two planes, one-query searches take
    the last level in two parts four times, find the second part no better than the first each time, and then take
    it whole (for the next 64 searches); with three planes their scan has a first stage on plane 0 alone, which
    gains from any tighter threshold, and the split stays.  Batches and fp32 queries keep the split, whatever came
    before them.  The pruning scans stay on throughout (their waves read like the plain scan once their bound has
    failed them; rows are still counted), and every search returns what the plain scan returns."""
    N, d, k = 5_000_000, 64, 30
    import torch
    centres = rbe_synth.centres_torch(64, d, torch.device("cuda:0"))
    ix = rbe.rbe_index_create(N, d, P, 0)
    for c_, z0 in enumerate(range(0, N, 1_000_000)):
        v = rbe_synth.vectors_torch(1_000_000, centres, 10.0, rbe_synth.SEED_ITEMS, c_)      # sigma 10: no clusters left
        pl, sc = rbe_synth.pack_planes_torch(v, P)
        rbe.rbe_load_chunk(ix, z0, pl, sc)
    rbe.rbe_finalize(ix)
    x = rbe_synth.vectors_torch(4, centres, 10.0, rbe_synth.SEED_QUERIES, 0).cpu().numpy()
    enc = [rbe.rbe_encode_query(x[i], P) for i in range(4)]
    qp = np.stack([e[0] for e in enc]); qs = np.stack([e[1] for e in enc])
    seen = []
    for _ in range(7):
        r = rbe.rbe_search(ix, qp[:1], qs[:1], k)
        st = rbe.rbe_get_search_stats(ix)
        seen.append((st["last_level_parts"], st["deep_rows"] > 0, st["scan_kernel"][st["n_levels"] - 1], r))
    want = [(2, True)] * 7 if P == 3 else [(2, True)] * 4 + [(1, True)] * 3
    assert [s[:2] for s in seen] == want, [s[:2] for s in seen]
    assert all(s[2] == ("scan_exact_prog2_hint" if P == 3 else "scan_exact_prog_hint") for s in seen), [s[2] for s in seen]
    r3 = rbe.rbe_search(ix, qp[1:4], qs[1:4], k)                 # a small batch: split, as always
    assert rbe.rbe_get_search_stats(ix)["last_level_parts"] == 2
    rf = rbe.rbe_search_float(ix, x[:1], k)                      # an fp32 query: split, as always
    assert rbe.rbe_get_search_stats(ix)["last_level_parts"] == 2
    r_again = rbe.rbe_search(ix, qp[:1], qs[:1], k)              # and the one-query searches are where they were
    assert rbe.rbe_get_search_stats(ix)["last_level_parts"] == (2 if P == 3 else 1)
    rbe.rbe_debug_set_progressive(ix, False)
    plain = rbe.rbe_search(ix, qp[:1], qs[:1], k)
    st = rbe.rbe_get_search_stats(ix)
    assert st["scan_kernel"][st["n_levels"] - 1] == "scan_exact" and st["last_level_parts"] == 1
    for s_ in seen:
        np.testing.assert_array_equal(s_[3][0], plain[0]); np.testing.assert_array_equal(s_[3][1], plain[1])
    np.testing.assert_array_equal(r_again[0], plain[0])
    plain3 = rbe.rbe_search(ix, qp[1:4], qs[1:4], k)
    np.testing.assert_array_equal(r3[0], plain3[0]); np.testing.assert_array_equal(r3[1], plain3[1])
    plainf = rbe.rbe_search_float(ix, x[:1], k)
    np.testing.assert_array_equal(rf[0], plainf[0]); np.testing.assert_array_equal(rf[1], plainf[1])
    rbe.rbe_free(ix)


# ------------------------------------------------------------------ negative scales: no pruning path may run
@pytest.mark.parametrize("d,P", [(64, 3), (128, 4), (64, 1)])
def test_negative_scales_in_the_last_array_are_searched_exactly(d, P):
    """The pruning scans bound the last plane's contribution by (largest last scale) x (query mass), and the
    matrix-core filter's slack is margin x (sum of scales): both under-estimate when a scale is negative.  Items
    whose LAST scale is negative and large in magnitude, planted next to the queries, must still be found: one
    query, a small batch, a batch that would go to the matrix cores, and fp32 queries."""
    N, k = 200_003, 25
    planes, scales, qp, qs = clustered(N, d, P, 512, 0.3, 16, P, seed=300 + d + P)
    rng = np.random.default_rng(301 + P)
    # planted items: every plane the complement of query q's base plane, last scale strongly negative, so the last
    # plane's true contribution is large and positive while any bound that takes max(a, 0) sees none of it
    for q in range(16):
        for z in rng.choice(N, 3, replace=False):
            for j in range(P):
                planes[j, z] = ~qp[q, 0]
            scales[:, z] = 0.0
            scales[P - 1, z] = -3.0
    scales[P - 1, rng.choice(N, N // 50, replace=False)] *= np.float32(-1.0)
    ix = load_with_ratio(planes, scales, 8)
    info = rbe.rbe_debug_index_info(ix)
    assert not info["can_prune"] and not info["scale_copies"]
    ids1, sc1 = rbe.rbe_search(ix, qp[:1], qs[:1], k)
    assert rbe.rbe_get_search_stats(ix)["n_levels"] >= 2 and rbe.rbe_get_search_stats(ix)["deep_rows"] == 0
    ids3, sc3 = rbe.rbe_search(ix, qp[1:4], qs[1:4], k)
    ids12, sc12 = rbe.rbe_search(ix, qp[4:], qs[4:], k)
    ids = np.concatenate([ids1, ids3, ids12]); sc = np.concatenate([sc1, sc3, sc12])
    check_batch(planes, scales, qp, qs, k, ids, sc)
    for q in range(16):                      # the planted items lead every list
        assert sc[q][0] > 0 and scales[P - 1, ids[q][0]] == np.float32(-3.0)
    # forcing the matrix-core path cannot bring its filter back either
    rbe.rbe_debug_set_batch_path(ix, 2)
    ids12b, sc12b = rbe.rbe_search(ix, qp[4:], qs[4:], k)
    np.testing.assert_array_equal(ids12b, ids12); np.testing.assert_array_equal(sc12b, sc12)
    rbe.rbe_debug_set_batch_path(ix, 0)
    # fp32 queries (one scan per query, and the would-be matrix-core batch)
    qf = rbe_synth.vectors_numpy(5, rbe_synth.centres_numpy(512, d), 0.3, seed=rbe_synth.SEED_QUERIES + 300 + d + P)
    for lo, hi in ((0, 1), (1, 5)):
        fi, fs = rbe.rbe_search_float(ix, qf[lo:hi], k)
        for q in range(lo, hi):
            o_ids, o_sc = oracle.topk_fq(planes, scales, qf[q], k)
            eps = 1e-5 * abs(o_sc[-1]) + 1e-6
            got = oracle.scores_at_fq(planes, scales, qf[q], fi[q - lo])
            np.testing.assert_allclose(fs[q - lo], got, rtol=1e-5, atol=1e-6)
            assert np.all(got >= o_sc[-1] - eps)
            assert set(o_ids[o_sc > o_sc[-1] + eps].tolist()) <= set(fi[q - lo].tolist())
    rbe.rbe_free(ix)


def test_non_finite_scale_is_rejected_at_finalize_and_can_be_repaired():
    rng = np.random.default_rng(311)
    planes, scales = random_corpus(rng, 5000, 64, 3)
    bad = scales.copy()
    bad[1, 4321] = np.inf
    ix = rbe.rbe_index_create(5000, 64, 3)
    rbe.rbe_load_chunk(ix, 0, planes, bad)
    with pytest.raises(rbe.RbeError) as e:
        rbe.rbe_finalize(ix)
    assert e.value.code == rbe.RBE_EINVAL and "not finite" in str(e.value)
    bad[2, 17] = np.nan; bad[1, 4321] = 1.0
    rbe.rbe_load_chunk(ix, 0, planes, bad)
    with pytest.raises(rbe.RbeError):
        rbe.rbe_finalize(ix)
    rbe.rbe_load_chunk(ix, 0, planes, scales)          # still loading: the chunk can be replaced
    rbe.rbe_finalize(ix)
    qp, qs = random_queries(rng, 1, 64, 3)
    ids, sc = rbe.rbe_search(ix, qp, qs, 10)
    check_topk(planes, scales, qp[0], qs[0], 10, ids[0], sc[0])
    rbe.rbe_free(ix)


# ------------------------------------------------------------------ caller-owned memory
def test_search_with_caller_supplied_workspace_matches_the_oracle():
    """All device scratch of a search in a torch tensor (rbe_workspace_bytes / rbe_set_workspace): one query, a
    batch on the matrix cores, fp32 queries and the near-lossless mode give the results of library-owned scratch and
    pass the oracle; a workspace that is too small is refused with the required size, and nothing is overwritten
    outside the tensor."""
    import torch
    N, d, P, k = 150_001, 64, 3, 100
    planes, scales, qp, qs = clustered(N, d, P, 256, 0.3, 9, P, seed=320)
    ix = load_with_ratio(planes, scales, 8)
    ref1 = rbe.rbe_search(ix, qp[:1], qs[:1], k)
    ref9 = rbe.rbe_search(ix, qp, qs, k)
    refn = nl_search(ix, qp[:2], qs[:2], k, group_size_I=16)
    qf = rbe_synth.vectors_numpy(3, rbe_synth.centres_numpy(256, d), 0.3, seed=rbe_synth.SEED_QUERIES + 321)
    reff = rbe.rbe_search_float(ix, qf, k)
    need1 = rbe.rbe_workspace_bytes(ix, 1, k)
    need9 = rbe.rbe_workspace_bytes(ix, 9, k)
    assert 0 < need1 < need9 and need9 % 256 == 0
    need_nl = rbe.rbe_workspace_bytes(ix, 2, k, rbe.RBE_SELECT_NEARLOSSLESS)          # group tables on top
    assert need_nl > rbe.rbe_workspace_bytes(ix, 2, k) and need_nl == rbe.rbe_workspace_bytes(ix, 2, k, rbe.RBE_SELECT_NEARLOSSLESS_Q2)
    need9_exact, need9 = need9, max(need9, need_nl)
    assert rbe.rbe_workspace_bytes(ix, 0, k) == 0 and rbe.rbe_workspace_bytes(ix, 65, k) == 0 and rbe.rbe_workspace_bytes(ix, 1, 4097) == 0
    guard = 4096
    buf = torch.full((guard + need9 + guard,), 0xA5, dtype=torch.uint8, device="cuda:0")
    assert buf.data_ptr() % 256 == 0
    ws = buf[guard:guard + need9]
    rbe.rbe_set_workspace(ix, ws)
    assert rbe.rbe_debug_index_info(ix)["caller_workspace"]
    for _ in range(2):                                   # a second round reuses the same block
        got1 = rbe.rbe_search(ix, qp[:1], qs[:1], k)
        got9 = rbe.rbe_search(ix, qp, qs, k)
        gotn = nl_search(ix, qp[:2], qs[:2], k, group_size_I=16)
        gotf = rbe.rbe_search_float(ix, qf, k)
        for got, ref in ((got1, ref1), (got9, ref9), (gotn, refn), (gotf, reff)):
            np.testing.assert_array_equal(got[0], ref[0]); np.testing.assert_array_equal(got[1], ref[1])
    check_batch(planes, scales, qp, qs, k, got9[0], got9[1])
    for q in range(2):
        check_nearlossless(planes, scales, qp[q], qs[q], k, 16, gotn[0][q], gotn[1][q])
    torch.cuda.synchronize()
    assert bool((buf[:guard] == 0xA5).all()) and bool((buf[guard + need9:] == 0xA5).all()), "wrote outside the workspace"
    # too small for nine queries, large enough for one
    rbe.rbe_set_workspace(ix, buf[guard:guard + need1])
    with pytest.raises(rbe.RbeError) as e:
        rbe.rbe_search(ix, qp, qs, k)
    assert e.value.code == rbe.RBE_EINVAL and str(need9_exact) in str(e.value)
    got1 = rbe.rbe_search(ix, qp[:1], qs[:1], k)
    np.testing.assert_array_equal(got1[0], ref1[0])
    with pytest.raises(rbe.RbeError):
        rbe.rbe_set_workspace(ix, buf[guard + 8:guard + need1])      # not 256-byte aligned
    rbe.rbe_set_workspace(ix, None)                      # back to library-owned scratch
    assert not rbe.rbe_debug_index_info(ix)["caller_workspace"]
    got9 = rbe.rbe_search(ix, qp, qs, k)
    np.testing.assert_array_equal(got9[0], ref9[0])
    rbe.rbe_free(ix)


@pytest.mark.parametrize("flags", [0, "dyadic_cosine"])
def test_index_in_caller_owned_storage(flags):
    """RBE_BORROW: tiles and side arrays inside a torch tensor of rbe_index_bytes() bytes; same results as an index
    the library allocates, pruning scans included; nothing written outside the tensor; the tensor survives rbe_free."""
    import torch
    N, d, P, k = 120_007, 64, 3, 20       # k * 500 below the items read before the last level: it runs the pruning scan
    planes, scales, qp, qs = clustered(N, d, P, 256, 0.3, 8, P, seed=330)
    fl = (rbe.RBE_DYADIC | rbe.RBE_COSINE) if flags else 0
    if fl:
        scales_in, qs_in = None, None
    else:
        scales_in, qs_in = scales, qs
    own = rbe.rbe_index_create_ex(N, d, P, fl, 8)
    rbe.rbe_load_chunk(own, 0, planes, scales_in)
    rbe.rbe_finalize(own)
    ref1 = rbe.rbe_search(own, qp[:1], qs_in[:1] if qs_in is not None else None, k)
    ref8 = rbe.rbe_search(own, qp, qs_in, k)
    assert rbe.rbe_get_search_stats(own)["n_levels"] >= 2
    rbe.rbe_free(own)
    need = rbe.rbe_index_bytes(N, d, P, fl | rbe.RBE_BORROW, 8)
    guard = 4096
    buf = torch.full((guard + need + guard,), 0x5A, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(rbe.RbeError):
        rbe.rbe_index_create_in(N, d, P, fl | rbe.RBE_BORROW, 8, buf[guard:guard + need - 256])     # too small
    ix = rbe.rbe_index_create_in(N, d, P, fl | rbe.RBE_BORROW, 8, buf[guard:guard + need])
    dev_planes = torch.from_numpy(planes.view(np.int64)).cuda()
    dev_scales = None if scales_in is None else torch.from_numpy(scales).cuda()
    rbe.rbe_load_chunk(ix, 0, dev_planes, dev_scales)
    rbe.rbe_finalize(ix)
    info = rbe.rbe_debug_index_info(ix)
    assert info["borrowed"] and info["can_prune"] and info["scale_copies"] == (fl == 0)
    got1 = rbe.rbe_search(ix, qp[:1], qs_in[:1] if qs_in is not None else None, k)
    assert rbe.rbe_get_search_stats(ix)["deep_rows"] > 0          # the progressive last level ran on the lent side arrays
    got8 = rbe.rbe_search(ix, qp, qs_in, k)
    for got, ref in ((got1, ref1), (got8, ref8)):
        np.testing.assert_array_equal(got[0], ref[0]); np.testing.assert_array_equal(got[1], ref[1])
    if not fl:
        check_batch(planes, scales, qp, qs, k, got8[0], got8[1])
    rbe.rbe_free(ix)
    torch.cuda.synchronize()
    assert bool((buf[:guard] == 0x5A).all()) and bool((buf[guard + need:] == 0x5A).all()), "wrote outside the storage"
    assert int(buf[guard:guard + need].to(torch.int64).sum()) != 0x5A * need       # still readable, and was written


def test_issue_rate_yardstick_runs_and_leaves_searches_untouched():
    """rbe_debug_issue_rate launches the batch scans with unreachable thresholds over tiles they go over again and
    again: it reports a time and the pairs scored, queues nothing, and later searches are unaffected."""
    N, d, P, k = 300_000, 64, 3, 50
    planes, scales, qp, qs = clustered(N, d, P, 256, 0.3, 16, P, seed=350)
    ix = load_with_ratio(planes, scales, 8)
    ref = rbe.rbe_search(ix, qp, qs, k)
    n_tiles = -(-N // 1024)
    for kernel in (0, 1):
        ms, pairs = rbe.rbe_debug_issue_rate(ix, qp, qs, kernel, 7)
        assert ms > 0 and pairs == min(n_tiles, 1024) * 1024 * 8 * 16
        ms2, pairs2 = rbe.rbe_debug_issue_rate(ix, qp, qs, kernel, 15)
        assert pairs2 == 2 * pairs and ms2 > 0
    with pytest.raises(rbe.RbeError):
        rbe.rbe_debug_issue_rate(ix, qp[:2], qs[:2], 0, 7)
    got = rbe.rbe_search(ix, qp, qs, k)
    np.testing.assert_array_equal(got[0], ref[0]); np.testing.assert_array_equal(got[1], ref[1])
    got1 = rbe.rbe_search(ix, qp[:1], qs[:1], k)
    np.testing.assert_array_equal(got1[0][0], ref[0][0])
    rbe.rbe_free(ix)
