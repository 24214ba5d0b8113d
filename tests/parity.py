"""Acceptance protocol shared by the GPU parity tests.

The GPU combines scores in fp32, the oracle in float64, so ids can legitimately
differ where scores tie to within rounding at the k-th place.  Tolerance: 1e-5
relative to the score, but never tighter than the fp32 rounding floor of the
sum itself -- the GPU performs Pq+1 roundings per plane and P per item on
partial sums bounded by M = d * sum_i |c_i| * max_z sum_j a_j[z], i.e. an
absolute error up to about (Pq+2) * P * 2^-24 * M <= 1e-6 * M, which matters only
when a score is a near-cancellation (random, unclustered corpora).  With s_k the
oracle's k-th best score and eps = max(1e-5 * |s_k|, 1e-6 * M) a result is
accepted iff
  * ids are unique, in range, and padded with -1 / -inf only past the number
    of existing results;
  * every returned score is within 1e-5 relative (or 1e-6 * M absolute) of the
    oracle's score of that id;
  * every item the oracle scores above s_k + eps is returned;
  * no returned item scores below s_k - eps in the oracle;
  * the list is sorted by (score desc, id asc) in the GPU's own fp32 scores.
"""
import numpy as np

import oracle

REL = 1e-5


def check_topk(planes, scales, q_planes, q_scales, k, ids, scores, n_valid=None, exact=None):
    """Check one query's result (ids int64[k], scores f32[k]).  `exact` may carry a
    precomputed oracle.topk result; n_valid is the number of results that exist."""
    N = planes.shape[1]
    m = min(k, N) if n_valid is None else n_valid
    ids = np.asarray(ids)
    scores = np.asarray(scores)
    assert ids.shape == (k,) and scores.shape == (k,)
    assert np.all(ids[m:] == -1), "tail must be padded with id -1"
    assert np.all(np.isneginf(scores[m:])), "tail must be padded with -inf"
    got = ids[:m]
    assert got.min(initial=0) >= 0 and got.max(initial=0) < N, "id out of range"
    assert np.unique(got).size == m, "duplicate ids in the result"

    o_ids, o_sc = exact if exact is not None else oracle.topk(planes, scales, q_planes, q_scales, k)
    if m == 0:
        return
    s_k = o_sc[m - 1]
    floor = rounding_floor(planes, scales, q_scales)
    eps = max(REL * abs(s_k), floor)
    true_sc = oracle.scores_at(planes, scales, q_planes, q_scales, got)
    np.testing.assert_allclose(scores[:m], true_sc, rtol=REL, atol=floor,
                               err_msg="returned score differs from the oracle's score of that id")
    assert np.all(true_sc >= s_k - eps), "returned an item below the k-th best"
    must = set(o_ids[:m][o_sc[:m] > s_k + eps].tolist())
    missing = must - set(got.tolist())
    assert not missing, f"missed {len(missing)} items above the k-th best, e.g. {sorted(missing)[:5]}"
    # order: score descending, equal scores by ascending id
    sc = scores[:m]
    assert np.all(sc[:-1] >= sc[1:]), "scores not sorted"
    same = sc[:-1] == sc[1:]
    assert np.all(got[:-1][same] < got[1:][same]), "equal scores must be ordered by id"


def rounding_floor(planes, scales, q_scales):
    d = 64 * planes.shape[2]
    return 1e-6 * d * float(np.sum(np.abs(q_scales))) * float(np.max(np.sum(scales.astype(np.float64), axis=0)))


def check_batch(planes, scales, q_planes, q_scales, k, ids, scores):
    for q in range(q_planes.shape[0]):
        check_topk(planes, scales, q_planes[q], q_scales[q], k, ids[q], scores[q])


def score_tolerance(scales, q_scales, d):
    """Absolute tolerance for dense fp32 scores: 1e-5 of the largest magnitude the
    sum can reach, d * (sum_i |c_i|) * (sum_j a_j[z])."""
    return REL * d * float(np.sum(np.abs(q_scales))) * np.sum(scales.astype(np.float64), axis=0)


def check_nearlossless(planes, scales, q_planes, q_scales, k, I, ids, scores, Tb=256, queue_len=1):
    """Check one query's near-lossless result against the oracle's Algorithm 1 (priority
    queues of `queue_len` entries).

    What a group forwards is decided in fp32 on the GPU and in float64 in the oracle, so a
    group may legitimately forward a different item when two of its items score within
    rounding of each other.  Accepted iff
      * every returned id is in range, ids are unique and at most queue_len share a group;
      * every returned item belongs in its group's queue: its oracle score is within eps of
        the oracle queue's last (worst) entry or better;
      * for every group, at least as many items are returned as its oracle queue holds above
        s_k + eps, and no returned item scores below s_k - eps (s_k = the oracle result's
        k-th score);
      * scores match the oracle's score of the returned id; sorted (score desc, id asc);
        the tail past the number of forwarded items is (-1, -inf).
    """
    N = planes.shape[1]
    o_ids, o_sc, w_ids, w_sc = oracle.nearlossless(planes, scales, q_planes, q_scales, k, I=I, Tb=Tb,
                                                   return_winners=True, queue_len=queue_len)
    w_ids = w_ids.reshape(-1, queue_len); w_sc = w_sc.reshape(-1, queue_len)
    n_live = int(np.sum(w_ids >= 0))
    m = min(k, n_live)
    ids = np.asarray(ids); scores = np.asarray(scores)
    assert np.all(ids[m:] == -1) and np.all(np.isneginf(scores[m:]))
    got = ids[:m]
    if m == 0:
        return
    assert got.min() >= 0 and got.max() < N and np.unique(got).size == m
    group = (got // (Tb * I)) * Tb + (got % Tb)
    per_group = np.bincount(group, minlength=w_ids.shape[0])
    assert per_group.max() <= queue_len, "more results from one group than its queue holds"
    floor = rounding_floor(planes, scales, q_scales)
    s_k = o_sc[m - 1]
    eps = max(REL * abs(s_k), floor)
    true_sc = oracle.scores_at(planes, scales, q_planes, q_scales, got)
    np.testing.assert_allclose(scores[:m], true_sc, rtol=REL, atol=floor)
    # worst entry of each oracle queue (a queue that is not full accepts anything)
    worst = np.where(w_ids[:, -1] >= 0, w_sc[:, -1], -np.inf)
    lim = worst[group]
    assert np.all(true_sc >= lim - np.maximum(REL * np.abs(np.where(np.isfinite(lim), lim, 0.0)), floor)), \
        "an item that does not belong in its group's queue"
    assert np.all(true_sc >= s_k - eps)
    need = np.sum((w_ids >= 0) & (w_sc > s_k + eps), axis=1)
    assert np.all(per_group >= need), "a queue entry above the k-th best forwarded item is missing"
    sc = scores[:m]
    assert np.all(sc[:-1] >= sc[1:])
    same = sc[:-1] == sc[1:]
    assert np.all(got[:-1][same] < got[1:][same])
