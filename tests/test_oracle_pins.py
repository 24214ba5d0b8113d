"""Pins for the CPU oracle: each oracle function is checked against something
other than itself -- naive +-1 arithmetic on unpacked vectors, closed forms,
invariants, textbook special cases and the figures the paper prints."""
import itertools
import math
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
import rbe_synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ---------------------------------------------------------------- helpers
def unpack_pm1(words, d):
    """Packed words -> +-1 vector, written independently of the oracle:
    dimension i is bit i%64 of word i//64, 1 -> +1, 0 -> -1."""
    words = np.asarray(words, dtype=np.uint64).ravel()
    out = np.empty(d, dtype=np.float64)
    for i in range(d):
        out[i] = 1.0 if (int(words[i // 64]) >> (i % 64)) & 1 else -1.0
    return out


def reconstruct(planes, scales, z, d):
    """khat_z = sum_j a_j[z] * b_z^j as a float64 vector."""
    v = np.zeros(d)
    for j in range(planes.shape[0]):
        v += float(scales[j, z]) * unpack_pm1(planes[j, z], d)
    return v


def reconstruct_query(q_planes, q_scales, d):
    v = np.zeros(d)
    for i in range(q_planes.shape[0]):
        v += float(q_scales[i]) * unpack_pm1(q_planes[i], d)
    return v


def random_corpus(rng, N, d, P):
    W = d // 64
    planes = rng.integers(0, 2**64, size=(P, N, W), dtype=np.uint64)
    scales = rng.uniform(0.01, 1.0, size=(P, N)).astype(np.float32)
    return planes, scales


def random_query(rng, d, Pq):
    W = d // 64
    return (rng.integers(0, 2**64, size=(Pq, W), dtype=np.uint64),
            rng.uniform(0.01, 1.0, size=Pq).astype(np.float32))


def full_sort_topk(sc, k):
    """Definition of exact top-k: sort every (score, id) by score desc, id asc."""
    order = sorted(range(len(sc)), key=lambda z: (-sc[z], z))
    return order[:k]


# ---------------------------------------------------------------- P1: bitwise identity
def test_binary_dot_identity_random_words():
    rng = np.random.default_rng(1)
    for d in (64, 128, 256):
        for _ in range(200):
            x = rng.integers(0, 2**64, size=d // 64, dtype=np.uint64)
            y = rng.integers(0, 2**64, size=d // 64, dtype=np.uint64)
            naive = int(np.dot(unpack_pm1(x, d), unpack_pm1(y, d)))
            assert oracle.binary_dot(x, y) == naive


def test_binary_dot_identity_exhaustive_8bit():
    # all 2^8 x 2^8 patterns in the low byte; the other 56 dims agree (+1 each)
    for a in range(256):
        xa = np.array([a], dtype=np.uint64)
        va = unpack_pm1(xa, 64)
        for b in range(0, 256, 5):
            xb = np.array([b], dtype=np.uint64)
            assert oracle.binary_dot(xa, xb) == int(np.dot(va, unpack_pm1(xb, 64)))


def test_binary_dot_corrected_sign_and_shift():
    # n = 1-like case embedded in 64 dims: x = +1, y = -1 in one dim, equal elsewhere
    x = np.array([0xFFFFFFFFFFFFFFFF], dtype=np.uint64)
    y = np.array([0xFFFFFFFFFFFFFFFE], dtype=np.uint64)
    assert oracle.binary_dot(x, y) == 62          # 63 agreements - 1 disagreement
    assert oracle.binary_dot(x, x) == 64
    assert oracle.binary_dot(x, ~x) == -64


def test_popcounts_layout_and_values():
    rng = np.random.default_rng(2)
    planes, _ = random_corpus(rng, 37, 128, 3)
    qp, _ = random_query(rng, 128, 2)
    pc = oracle.popcounts(planes, qp)
    assert pc.shape == (37, 3, 2)
    for z in (0, 5, 36):
        for j in range(3):
            for i in range(2):
                dis = np.sum(unpack_pm1(planes[j, z], 128) != unpack_pm1(qp[i], 128))
                assert pc[z, j, i] == dis


# ---------------------------------------------------------------- P2: score == float dot of reconstructions
@pytest.mark.parametrize("d,P,Pq", [(64, 1, 1), (64, 3, 3), (64, 2, 3), (128, 4, 4), (128, 4, 1), (256, 2, 2)])
def test_score_equals_dot_of_reconstructed_vectors(d, P, Pq):
    rng = np.random.default_rng(100 + d + 10 * P + Pq)
    N = 300
    planes, scales = random_corpus(rng, N, d, P)
    qp, qs = random_query(rng, d, Pq)
    s = oracle.scores(planes, scales, qp, qs)
    qhat = reconstruct_query(qp, qs, d)
    for z in range(N):
        ref = float(np.dot(qhat, reconstruct(planes, scales, z, d)))
        assert s[z] == pytest.approx(ref, rel=1e-12, abs=1e-12)


def test_score_on_encoded_clustered_corpus_matches_float_dot():
    c = rbe_synth.centres_numpy(8, 64)
    x = rbe_synth.vectors_numpy(500, c, 0.3, seed=3)
    q = rbe_synth.vectors_numpy(1, c, 0.3, seed=4)
    planes, scales = oracle.encode(x, 3)
    qp, qs = oracle.encode(q, 3)
    s = oracle.scores(planes, scales, qp[:, 0], qs[:, 0])
    qhat = reconstruct_query(qp[:, 0], qs[:, 0], 64)
    ref = np.array([np.dot(qhat, reconstruct(planes, scales, z, 64)) for z in range(500)])
    np.testing.assert_allclose(s, ref, rtol=1e-12, atol=1e-12)
    # the 3-plane reconstruction approximates the true cosine
    assert np.corrcoef(s, x @ q[0])[0, 1] > 0.97


def test_scores_range_arguments():
    rng = np.random.default_rng(5)
    planes, scales = random_corpus(rng, 100, 64, 2)
    qp, qs = random_query(rng, 64, 2)
    full = oracle.scores(planes, scales, qp, qs)
    np.testing.assert_array_equal(oracle.scores(planes, scales, qp, qs, 17, 63), full[17:63])



@pytest.mark.parametrize("d,P,Pq", [(64, 3, 3), (64, 2, 3), (128, 4, 4)])
def test_scores_at_gathers_the_listed_ids(d, P, Pq):
    """scores_at(ids)[r] is the score of item ids[r]: against the dense scores for shuffled, repeated
    and boundary ids, and against the float64 dot product of the unpacked reconstructions (Eq. 14)
    for a handful.  Items are made distinguishable (a wrong gather index cannot hit an equal score)."""
    rng = np.random.default_rng(400 + d + P)
    N = 777
    planes, scales = random_corpus(rng, N, d, P)
    qp, qs = random_query(rng, d, Pq)
    dense = oracle.scores(planes, scales, qp, qs)
    assert np.unique(dense).size == N
    ids = np.concatenate([[0, N - 1, N - 1, 0, 1, N - 2], rng.permutation(N), rng.integers(0, N, size=300)]).astype(np.int64)
    got = oracle.scores_at(planes, scales, qp, qs, ids)
    np.testing.assert_array_equal(got, dense[ids])
    qv = reconstruct_query(qp, qs, d)
    for r in (0, 1, 5, 6, 400, ids.size - 1):
        z = int(ids[r])
        ref = float(np.dot(qv, reconstruct(planes, scales, z, d)))
        assert abs(got[r] - ref) <= 1e-12 * max(1.0, abs(ref))
    assert oracle.scores_at(planes, scales, qp, qs, np.empty(0, np.int64)).size == 0
    # one id at a time agrees with the batch call (no dependence on the list's length or order)
    for z in (0, 3, N - 1):
        assert oracle.scores_at(planes, scales, qp, qs, [z])[0] == dense[z]
    with pytest.raises(ValueError):
        oracle.scores_at(planes, scales, qp, qs, [N])
    with pytest.raises(ValueError):
        oracle.scores_at(planes, scales, qp, qs, [-1])


def test_scores_at_on_a_strided_corpus_view_uses_plane_major_indexing():
    """Plane j of item z sits at planes[j][z]: a corpus whose planes differ per j and per z in a
    known way (one plane equal to the query, the others its complement) gives hand-computable scores."""
    d, P, N = 64, 3, 50
    qp = np.array([[0x0123456789ABCDEF]], dtype=np.uint64)
    qs = np.array([1.0], dtype=np.float32)
    planes = np.empty((P, N, 1), dtype=np.uint64)
    scales = np.empty((P, N), dtype=np.float32)
    for z in range(N):
        for j in range(P):
            same = (z + j) % 3 == 0                      # exactly one plane of every item equals the query
            planes[j, z, 0] = qp[0, 0] if same else ~qp[0, 0]
            scales[j, z] = (j + 1) * 10 + z * 0.25       # exact in fp32
    ids = np.array([49, 0, 17, 17, 3], dtype=np.int64)
    expect = []
    for z in ids:
        expect.append(sum((1.0 if (z + j) % 3 == 0 else -1.0) * 64.0 * ((j + 1) * 10 + z * 0.25) for j in range(P)))
    np.testing.assert_array_equal(oracle.scores_at(planes, scales, qp, qs, ids), np.array(expect))


def test_recall_against_hand_counted_sets():
    assert oracle.recall([1, 2, 3], [1, 2, 3]) == 1.0
    assert oracle.recall([3, 2, 1], [1, 2, 3]) == 1.0                 # order does not matter
    assert oracle.recall([1, 2, 9], [1, 2, 3]) == 2 / 3
    assert oracle.recall([7, 8, 9], [1, 2, 3]) == 0.0
    assert oracle.recall([1, -1, -1], [1, 2, -1]) == 0.5             # -1 padding is no item on either side
    assert oracle.recall([-1, -1], [-1, -1]) == 1.0                  # nothing to find
    assert oracle.recall([], [4, 5]) == 0.0
    assert oracle.recall([4, 4, 4, 5], [4, 5, 6, 7]) == 0.5          # repeats count once
    assert oracle.recall(np.array([0, 5], dtype=np.int64), np.array([0, 1, 2, 5], dtype=np.int64)) == 0.5   # id 0 is an item

# ---------------------------------------------------------------- P3: the paper's worked expansions
def test_two_ingredient_expansion_unweighted():
    """Sec. 3.2 example: (b0_q + d0_q).(b0_k + d0_k) is the sum of the four
    binary dot products."""
    rng = np.random.default_rng(6)
    for _ in range(50):
        planes = rng.integers(0, 2**64, size=(2, 1, 1), dtype=np.uint64)
        qp = rng.integers(0, 2**64, size=(2, 1), dtype=np.uint64)
        ones = np.ones((2, 1), dtype=np.float32)
        s = oracle.scores(planes, ones, qp, ones[:, 0])[0]
        four = sum(oracle.binary_dot(qp[i], planes[j, 0]) for i in range(2) for j in range(2))
        direct = np.dot(unpack_pm1(qp[0], 64) + unpack_pm1(qp[1], 64),
                        unpack_pm1(planes[0, 0], 64) + unpack_pm1(planes[1, 0], 64))
        assert s == four == direct


def test_rbe_dot_product_expansion_with_residual_weights():
    """Eq. 14 with the paper's weights: b^t = b^0 + sum_{s<t} 2^-(s+1) d^s on both
    sides (u query residuals, v keyword residuals); the four groups of terms of
    the expansion, with the summation limits the definitions imply."""
    rng = np.random.default_rng(7)
    u, v = 2, 1                                     # rbe*: 3 query vectors, 2 keyword vectors
    qp = rng.integers(0, 2**64, size=(u + 1, 1), dtype=np.uint64)
    planes = rng.integers(0, 2**64, size=(v + 1, 1, 1), dtype=np.uint64)
    qs = np.array([2.0 ** -i for i in range(u + 1)], dtype=np.float32)
    ks = np.array([[2.0 ** -j] for j in range(v + 1)], dtype=np.float32)
    s = oracle.scores(planes, ks, qp, qs)[0]
    bd = oracle.binary_dot
    b0q, dq = qp[0], qp[1:]
    b0k, dk = planes[0, 0], planes[1:, 0]
    expansion = (bd(b0q, b0k)
                 + sum(0.5 ** (j + i + 2) * bd(dq[j], dk[i]) for j in range(u) for i in range(v))
                 + sum(0.5 ** (i + 1) * bd(b0q, dk[i]) for i in range(v))
                 + sum(0.5 ** (j + 1) * bd(b0k, dq[j]) for j in range(u)))
    assert s == pytest.approx(expansion, rel=1e-15)


def test_residual_weight_levels_and_cardinality():
    """Sec. 4.3: with weight 1/2 a two-ingredient embedding takes per-dimension
    values {-1.5,-0.5,0.5,1.5} and 4^n distinct vectors; without it {-2,0,2} and 3^n."""
    with open(os.path.join(GOLDEN, "paper_constants.txt")) as f:
        line = [l for l in f if l.startswith("two_ingredient_levels")][0]
    levels = sorted(float(t) for t in line.split("#")[0].split()[1:])
    for n in (1, 2, 3):
        weighted, plain = set(), set()
        for b in itertools.product((-1, 1), repeat=n):
            for dd in itertools.product((-1, 1), repeat=n):
                weighted.add(tuple(bi + 0.5 * di for bi, di in zip(b, dd)))
                plain.add(tuple(bi + di for bi, di in zip(b, dd)))
        assert len(weighted) == 4 ** n and len(plain) == 3 ** n
        assert sorted({v for t in weighted for v in t}) == levels
    # general claim: with j ingredient vectors the cardinality grows (2^j/(j+1))^n times
    for j in (2, 3, 4):
        w = {sum(0.5 ** t * s for t, s in enumerate(signs)) for signs in itertools.product((-1, 1), repeat=j)}
        p = {sum(signs) for signs in itertools.product((-1, 1), repeat=j)}
        assert len(w) == 2 ** j and len(p) == j + 1


# ---------------------------------------------------------------- P4: special cases
def test_single_plane_ranking_is_hamming_ranking():
    rng = np.random.default_rng(8)
    N = 2000
    planes = rng.integers(0, 2**64, size=(1, N, 1), dtype=np.uint64)
    scales = np.ones((1, N), dtype=np.float32)
    qp = rng.integers(0, 2**64, size=(1, 1), dtype=np.uint64)
    ids, sc = oracle.topk(planes, scales, qp, np.ones(1, np.float32), 50)
    ham = np.array([bin(int(planes[0, z, 0]) ^ int(qp[0, 0])).count("1") for z in range(N)])
    expect = sorted(range(N), key=lambda z: (ham[z], z))[:50]
    assert list(ids) == expect
    np.testing.assert_array_equal(sc, 64 - 2 * ham[ids])


def test_self_score_is_squared_norm_and_cosine_self_query_wins():
    c = rbe_synth.centres_numpy(4, 64)
    x = rbe_synth.vectors_numpy(400, c, 0.3, seed=9)
    planes, scales = oracle.encode(x, 3)
    nrm = oracle.recon_norms(planes, scales)
    for z in (0, 17, 399):
        s = oracle.scores(planes, scales, planes[:, z], scales[:, z], z, z + 1)[0]
        assert s == pytest.approx(nrm[z] ** 2, rel=1e-12)
        assert nrm[z] == pytest.approx(np.linalg.norm(reconstruct(planes, scales, z, 64)), rel=1e-12)
    cos_scales = oracle.fold_cosine(planes, scales)
    z = 123
    s = oracle.scores(planes, cos_scales, planes[:, z], scales[:, z])
    assert s[z] == pytest.approx(nrm[z], rel=1e-6)          # ||khat|| by Cauchy-Schwarz is the maximum
    assert np.all(s <= s[z] * (1 + 1e-6))


def test_paper_special_case_dyadic_weights_and_stored_norm():
    """The paper's score: weights 2^-t, one inverse norm per keyword (Sec. 5.1)."""
    rng = np.random.default_rng(10)
    N, d = 200, 64
    planes = rng.integers(0, 2**64, size=(2, N, 1), dtype=np.uint64)
    w = np.array([[1.0], [0.5]], dtype=np.float32) * np.ones((2, N), dtype=np.float32)
    scales = oracle.fold_cosine(planes, w)
    qp = rng.integers(0, 2**64, size=(3, 1), dtype=np.uint64)
    qs = np.array([1.0, 0.5, 0.25], dtype=np.float32)
    s = oracle.scores(planes, scales, qp, qs)
    qv = reconstruct_query(qp, qs, d)
    for z in range(0, N, 7):
        kv = unpack_pm1(planes[0, z], d) + 0.5 * unpack_pm1(planes[1, z], d)
        # ||b^1||^2 = 1.25 n + b^0 . d^0
        assert np.dot(kv, kv) == pytest.approx(1.25 * d + oracle.binary_dot(planes[0, z], planes[1, z]))
        assert s[z] == pytest.approx(np.dot(qv, kv) / np.linalg.norm(kv), rel=1e-6)


# ---------------------------------------------------------------- P5: invariants
def test_invariants():
    rng = np.random.default_rng(11)
    N, d, P, Pq = 500, 128, 3, 2
    planes, scales = random_corpus(rng, N, d, P)
    qp, qs = random_query(rng, d, Pq)
    s = oracle.scores(planes, scales, qp, qs)

    perm = rng.permutation(N)                              # item permutation
    np.testing.assert_array_equal(oracle.scores(planes[:, perm], scales[:, perm], qp, qs), s[perm])

    np.testing.assert_array_equal(oracle.scores(~planes, scales, ~qp, qs), s)   # complement both sides

    # the same rotation of the 64 bit positions of every word on both sides
    def rot(a, r):
        return ((a << np.uint64(r)) | (a >> np.uint64(64 - r)))
    np.testing.assert_array_equal(oracle.scores(rot(planes, 13), scales, rot(qp, 13), qs), s)
    # swapping the two words of every vector on both sides
    np.testing.assert_array_equal(oracle.scores(planes[:, :, ::-1], scales, qp[:, ::-1], qs), s)

    flipped = planes.copy()
    flipped[1] = ~flipped[1]                               # complement one corpus plane: its term changes sign
    s1 = oracle.scores(flipped, scales, qp, qs)
    only1 = scales.copy(); only1[0] = 0; only1[2] = 0
    term1 = oracle.scores(planes, only1, qp, qs)
    np.testing.assert_allclose(s1, s - 2 * term1, rtol=1e-12, atol=1e-12)

    lam = scales.copy(); lam[:, 7] *= np.float32(4.0)       # scale one item's planes by a power of two
    s2 = oracle.scores(planes, lam, qp, qs)
    assert s2[7] == 4.0 * s[7] and np.array_equal(np.delete(s2, 7), np.delete(s, 7))

    a = scales.copy(); a[1:] = 0                            # additivity over planes
    b = scales.copy(); b[0] = 0
    np.testing.assert_allclose(oracle.scores(planes, a, qp, qs) + oracle.scores(planes, b, qp, qs), s,
                               rtol=1e-12, atol=1e-12)


def test_duplicates_tie_and_order_by_id():
    x = rbe_synth.near_duplicates_numpy(300, 64, 5, seed=12)
    planes, scales = oracle.encode(x, 3)
    qp, qs = oracle.encode(x[:1], 3)
    ids, sc = oracle.topk(planes, scales, qp[:, 0], qs[:, 0], 40)
    s = oracle.scores(planes, scales, qp[:, 0], qs[:, 0])
    assert list(ids) == full_sort_topk(s, 40)
    runs = [list(g) for _, g in itertools.groupby(range(40), key=lambda r: sc[r])]
    assert any(len(r) > 1 for r in runs)
    for r in runs:
        assert list(ids[r]) == sorted(ids[r])


# ---------------------------------------------------------------- hybrid scoring (float query)
@pytest.mark.parametrize("d,P", [(64, 1), (64, 3), (128, 4)])
def test_float_query_score_is_dot_with_reconstruction(d, P):
    rng = np.random.default_rng(50 + d + P)
    N = 200
    planes, scales = random_corpus(rng, N, d, P)
    q = rng.standard_normal(d).astype(np.float32)
    s = oracle.scores_fq(planes, scales, q)
    for z in range(N):
        assert s[z] == pytest.approx(float(np.dot(q.astype(np.float64), reconstruct(planes, scales, z, d))), rel=1e-12, abs=1e-12)
    np.testing.assert_array_equal(oracle.scores_at_fq(planes, scales, q, [5, 0, 199]), s[[5, 0, 199]])
    ids, sc = oracle.topk_fq(planes, scales, q, 30)
    assert list(ids) == full_sort_topk(s, 30)
    np.testing.assert_array_equal(sc, s[ids])


def test_float_query_equal_to_reconstructed_binary_query_gives_binary_score():
    """If the float query is exactly the reconstruction sum_i c_i b_q^i of an RBE query, the hybrid
    score equals the all-binary score of Eq. 14 (dyadic c_i keep the reconstruction exact in fp32)."""
    rng = np.random.default_rng(51)
    planes, scales = random_corpus(rng, 300, 64, 3)
    qp = rng.integers(0, 2**64, size=(3, 1), dtype=np.uint64)
    qs = np.array([1.0, 0.5, 0.25], dtype=np.float32)
    qf = reconstruct_query(qp, qs, 64).astype(np.float32)
    np.testing.assert_allclose(oracle.scores_fq(planes, scales, qf), oracle.scores(planes, scales, qp, qs), rtol=1e-12, atol=1e-12)


# ---------------------------------------------------------------- P9: exact top-k
@pytest.mark.parametrize("N,k", [(1, 1), (10, 3), (10, 10), (10, 25), (1000, 1), (1000, 100), (5000, 4096)])
def test_topk_equals_full_sort(N, k):
    rng = np.random.default_rng(13 + N + k)
    planes, scales = random_corpus(rng, N, 64, 2)
    scales = np.round(scales, 1).astype(np.float32)       # coarse scales -> plenty of ties
    qp, qs = random_query(rng, 64, 2)
    s = oracle.scores(planes, scales, qp, qs)
    ids, sc = oracle.topk(planes, scales, qp, qs, k)
    expect = full_sort_topk(s, k)
    m = min(N, k)
    assert list(ids[:m]) == expect
    np.testing.assert_array_equal(sc[:m], s[expect])
    assert np.all(ids[m:] == -1) and np.all(np.isneginf(sc[m:]))
    if k == 1:
        assert ids[0] == int(np.flatnonzero(s == s.max())[0])


def test_topk_of_scores_and_subrange():
    rng = np.random.default_rng(14)
    s = np.round(rng.standard_normal(3000), 1)
    ids, sc = oracle.topk_of_scores(s, None, 77)
    assert list(ids) == full_sort_topk(s, 77)
    given = rng.permutation(3000).astype(np.int64) + 10
    ids2, _ = oracle.topk_of_scores(s, given, 77)
    expect = sorted(range(3000), key=lambda r: (-s[r], given[r]))[:77]
    assert list(ids2) == [int(given[r]) for r in expect]

    planes, scales = random_corpus(rng, 400, 64, 2)
    qp, qs = random_query(rng, 64, 2)
    full = oracle.scores(planes, scales, qp, qs)
    ids3, _ = oracle.topk(planes, scales, qp, qs, 10, 100, 250)
    assert list(ids3) == [100 + r for r in full_sort_topk(full[100:250], 10)]


# ---------------------------------------------------------------- P6: encoder
def test_encoder_identities():
    rng = np.random.default_rng(15)
    d, P = 128, 4
    x = rng.standard_normal((50, d)).astype(np.float32)
    x[3, 10] = 0.0                                          # rho(0) = -1 -> bit 0
    planes, scales = oracle.encode(x, P)
    assert (int(planes[0, 3, 0]) >> 10) & 1 == 0
    for z in range(50):
        r = x[z].astype(np.float64)
        for t in range(P):
            b = unpack_pm1(planes[t, z], d)
            assert np.all((b > 0) == (r > 0))
            alpha = float(scales[t, z])
            assert alpha == pytest.approx(np.mean(np.abs(r)), rel=1e-6)
            # least-squares optimum of ||r - alpha * sign(r)||^2 over alpha
            for other in (alpha * 0.9, alpha * 1.1):
                assert np.sum((r - alpha * b) ** 2) <= np.sum((r - other * b) ** 2)
            r_next = (r - alpha * b).astype(np.float32).astype(np.float64)
            # energy identity ||r'||^2 = ||r||^2 - d alpha^2
            assert np.sum(r_next ** 2) == pytest.approx(np.sum(r ** 2) - d * alpha ** 2, rel=1e-5, abs=1e-6)
            r = r_next
        recon = reconstruct(planes, scales, z, d)
        np.testing.assert_allclose(recon + r, x[z], atol=1e-5)
    # residual energy strictly decreases, so more planes approximate x better
    e = [np.mean(np.sum((x - np.stack([reconstruct(planes[:p], scales[:p], z, d) for z in range(50)])) ** 2, axis=1))
         for p in range(1, P + 1)]
    assert all(e[i + 1] < e[i] for i in range(P - 1))


def test_encoder_bit_order_lsb_first():
    x = -np.ones((1, 128), dtype=np.float32)
    x[0, 0] = 1; x[0, 65] = 1; x[0, 127] = 1
    planes, scales = oracle.encode(x, 1)
    assert int(planes[0, 0, 0]) == 1
    assert int(planes[0, 0, 1]) == (1 << 1) | (1 << 63)
    assert scales[0, 0] == 1.0


# ---------------------------------------------------------------- O4: near-lossless selector
def groups_by_reshape(sc, Tb, I, qlen):
    """The selector's partition written as array reshapes, independently of the oracle's loops
    (Algorithm 1, Sec. 6.2): pad the id axis to whole blocks of Tb*I ids, view it as
    [block][visit][thread] (a thread's visits are Tb apart), and bring the visits of one
    (block, thread) pair together.  Returns, per group, the ids of its best qlen existing items
    under (score desc, id asc), best first."""
    N = len(sc)
    n_blocks = -(-N // (Tb * I))
    ids = np.arange(n_blocks * Tb * I, dtype=np.int64)
    padded = np.full(ids.size, -np.inf)
    padded[:N] = sc
    member_ids = ids.reshape(n_blocks, I, Tb).transpose(0, 2, 1).reshape(n_blocks * Tb, I)
    member_sc = padded.reshape(n_blocks, I, Tb).transpose(0, 2, 1).reshape(n_blocks * Tb, I)
    # ids ascend along a group's row, so a stable sort by descending score breaks ties by id
    order = np.argsort(-member_sc, axis=1, kind="stable")
    best_ids = np.take_along_axis(member_ids, order, axis=1)[:, :qlen]
    return [[int(z) for z in row if z < N] for row in best_ids]


def forwarded_topk(sc, groups, k):
    alive = [z for g in groups for z in g]
    alive.sort(key=lambda z: (-sc[z], z))
    return alive[:k]


@pytest.mark.parametrize("N,Tb,I,k", [(24, 4, 3, 5), (25, 4, 3, 8), (1000, 8, 16, 20), (1000, 256, 2, 600), (70000, 256, 256, 100)])
def test_nearlossless_matches_partition_by_reshape(N, Tb, I, k):
    rng = np.random.default_rng(16 + N)
    planes, scales = random_corpus(rng, N, 64, 2)
    scales = np.round(scales, 1).astype(np.float32)
    qp, qs = random_query(rng, 64, 2)
    s = oracle.scores(planes, scales, qp, qs)
    ids, sc, w_ids, w_sc = oracle.nearlossless(planes, scales, qp, qs, k, I=I, Tb=Tb, return_winners=True)
    groups = groups_by_reshape(s, Tb, I, 1)
    expect = forwarded_topk(s, groups, k)
    m = len(expect)
    assert list(ids[:m]) == expect and np.all(ids[m:] == -1)
    np.testing.assert_array_equal(sc[:m], s[expect])
    assert [int(w) for w in w_ids] == [(g[0] if g else -1) for g in groups]
    assert oracle.n_groups(N, I, Tb) == len(groups)
    # the group of an id, from the id alone (the closed form the GPU tests use)
    z = np.arange(N)
    gz = (z // (Tb * I)) * Tb + (z % Tb)
    for g in (0, len(groups) // 2, len(groups) - 1):
        members = z[gz == g]
        if members.size:
            best = min(members, key=lambda m_: (-s[m_], m_))
            assert groups[g] == [int(best)]
    # a subset of the exact top-k can only lose items, never invent better ones
    exact, exact_sc = oracle.topk(planes, scales, qp, qs, k)
    hit = len(set(ids[:m].tolist()) & set(exact.tolist()))
    assert oracle.recall(ids, exact) == hit / len([e for e in exact if e >= 0])
    assert np.all(sc[:m] <= exact_sc[:m])


def test_nearlossless_I1_is_exact():
    rng = np.random.default_rng(17)
    planes, scales = random_corpus(rng, 3000, 64, 3)
    qp, qs = random_query(rng, 64, 3)
    a, _ = oracle.nearlossless(planes, scales, qp, qs, 50, I=1, Tb=256)
    b, _ = oracle.topk(planes, scales, qp, qs, 50)
    assert list(a) == list(b)


@pytest.mark.parametrize("N,Tb,I,k,qlen", [(24, 4, 3, 5, 2), (25, 4, 3, 30, 2), (1000, 8, 16, 40, 2), (1000, 8, 16, 40, 3),
                                           (1000, 256, 2, 600, 2), (70000, 256, 256, 100, 2), (500, 4, 5, 50, 5)])
def test_nearlossless_longer_queue_matches_partition_by_reshape(N, Tb, I, k, qlen):
    rng = np.random.default_rng(116 + N + qlen)
    planes, scales = random_corpus(rng, N, 64, 2)
    scales = np.round(scales, 1).astype(np.float32)       # many exact ties
    qp, qs = random_query(rng, 64, 2)
    s = oracle.scores(planes, scales, qp, qs)
    ids, sc, w_ids, w_sc = oracle.nearlossless(planes, scales, qp, qs, k, I=I, Tb=Tb, return_winners=True, queue_len=qlen)
    groups = groups_by_reshape(s, Tb, I, qlen)
    expect = forwarded_topk(s, groups, k)
    m = len(expect)
    assert list(ids[:m]) == expect and np.all(ids[m:] == -1)
    np.testing.assert_array_equal(sc[:m], s[expect])
    for g, q in enumerate(groups):
        assert [int(v) for v in w_ids[g][:len(q)]] == q and np.all(w_ids[g][len(q):] == -1)
        np.testing.assert_array_equal(w_sc[g][:len(q)], s[q])
    # a longer queue keeps a superset of what a shorter one keeps
    shorter, _ = oracle.nearlossless(planes, scales, qp, qs, k, I=I, Tb=Tb, queue_len=qlen - 1)
    exact, _ = oracle.topk(planes, scales, qp, qs, k)
    assert oracle.recall(ids, exact) >= oracle.recall(shorter, exact)
    if qlen >= I:                                          # every item is forwarded: the selector is exact
        assert list(ids) == list(exact)


def test_expected_recall_with_longer_queue_by_enumeration():
    """Tiny case, every placement enumerated: C = 12 slots in threads of I = 3, N = 4 relevant items;
    a thread with n relevant items keeps min(n, p)."""
    from itertools import combinations
    C, I, N = 12, 3, 4
    for p in (1, 2, 3):
        kept = 0
        total = 0
        for placement in combinations(range(C), N):
            per_thread = [0] * (C // I)
            for slot in placement:
                per_thread[slot // I] += 1
            kept += sum(min(n, p) for n in per_thread)
            total += 1
        assert oracle.expected_recall(N, C, I, queue_len=p) == pytest.approx(kept / (total * N), abs=1e-12)
    assert oracle.expected_recall(N, C, I, queue_len=3) == 1.0
    # the paper's operating point: a second queue entry removes almost all of the (already small) loss
    r1 = oracle.expected_recall(1000, 10**9, 256, queue_len=1)
    r2 = oracle.expected_recall(1000, 10**9, 256, queue_len=2)
    assert r1 < r2 < 1.0 and 1 - r2 < 1e-7 and 1 - r1 == pytest.approx(1.274e-4, rel=1e-2)


# ---------------------------------------------------------------- P7: Appendix A
def test_table7_values():
    rows = {}
    with open(os.path.join(GOLDEN, "appendix_a_table7.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                l, pct = line.split()
                rows[int(l)] = float(pct)
    assert sorted(rows) == [0, 1, 2]
    for l, pct in rows.items():
        got = 100.0 * oracle.miss_probability(l, N=1000, C=10**9, I=256)
        assert abs(got - pct) <= 1.1e-3, (l, got, pct)      # the table truncates 88.0396 to 88.039


def test_eq16_against_closed_forms():
    """L = 0, 1, 2 written out by hand from Eq. 16.  Evaluated with log-gamma, whose
    cancellation at arguments ~1e9 leaves about 1e-6 relative error."""
    N, C, I = 1000, 10**9, 256
    T = C // I
    lg = math.lgamma

    def lchoose(n, r):
        return lg(n + 1) - lg(r + 1) - lg(n - r + 1)
    p0 = math.exp(lchoose(T, N) + N * math.log(I) - lchoose(C, N))
    p1 = math.exp(lchoose(T, N - 1) + math.log(N - 1) + math.log(math.comb(I, 2)) + (N - 2) * math.log(I) - lchoose(C, N))
    a = math.exp(lchoose(T, N - 2) + math.log(N - 2) + math.log(math.comb(I, 3)) + (N - 3) * math.log(I) - lchoose(C, N))
    b = math.exp(lchoose(T, N - 2) + math.log(math.comb(N - 2, 2)) + 2 * math.log(math.comb(I, 2)) + (N - 4) * math.log(I) - lchoose(C, N))
    p2 = a + b
    assert float(oracle.prob_threads_hit(N, N, C, I)) == pytest.approx(p0, rel=1e-5)
    assert float(oracle.prob_threads_hit(N - 1, N, C, I)) == pytest.approx(p1, rel=1e-5)
    assert float(oracle.prob_threads_hit(N - 2, N, C, I)) == pytest.approx(p2, rel=1e-5)


def test_eq16_by_enumerating_compositions_and_by_brute_force():
    def compositions(total, parts):
        if parts == 1:
            yield (total,)
            return
        for first in range(1, total - parts + 2):
            for rest in compositions(total - first, parts - 1):
                yield (first,) + rest

    for (C, I, N) in [(12, 3, 3), (12, 4, 5), (16, 4, 4), (20, 5, 6)]:
        T = C // I
        # brute force over every placement of the N relevant items
        count = {}
        for placement in itertools.combinations(range(C), N):
            m = len({slot // I for slot in placement})
            count[m] = count.get(m, 0) + 1
        total = math.comb(C, N)
        for M in range(0, N + 1):
            by_eq16 = Fraction(0)
            if 1 <= M <= T:
                by_eq16 = Fraction(math.comb(T, M) * sum(math.prod(math.comb(I, n) for n in comp)
                                                         for comp in compositions(N, M)), total)
            assert oracle.prob_threads_hit(M, N, C, I) == by_eq16 == Fraction(count.get(M, 0), total)
        assert sum(oracle.prob_threads_hit(M, N, C, I) for M in range(N + 1)) == 1
        e_rec = sum(M * Fraction(count.get(M, 0), total) for M in range(N + 1)) / N
        assert oracle.expected_recall(N, C, I) == pytest.approx(float(e_rec), rel=1e-12)


def test_expected_recall_matches_paper_measurement():
    with open(os.path.join(GOLDEN, "paper_constants.txt")) as f:
        consts = {l.split()[0]: l.split("#")[0].split()[1:] for l in f if l.strip() and not l.startswith("#")}
    side, tb, ipt = int(consts["grid_side"][0]), int(consts["threads_per_block"][0]), int(consts["items_per_thread"][0])
    slots = side * side * tb * ipt
    assert slots == 1_212_153_856 and round(slots / 1e9, 1) == float(consts["keywords_billion"][0])
    r = oracle.expected_recall(1000, slots, ipt)
    assert round(100 * r, 2) == float(consts["recall_at_1000_percent"][0])
    # first-order approximation 1 - (N-1)(I-1) / (2 (C-1))
    assert r == pytest.approx(1 - 999 * 255 / (2 * (slots - 1)), abs=1e-7)
    # memory figures of Sec. 5.3 (GiB)
    assert round(10**9 * 64 * 2 / 8 / 2**30, 2) == float(consts["memory_rbe_gb"][0])
    assert round(10**9 * 64 * 4 / 2**30) == float(consts["memory_float_gb"][0])


def test_measured_recall_of_oracle_selector_tracks_appendix_a():
    """Random scores in random order: recall of the oracle's selector averaged
    over queries agrees with E[M]/N (binomial tolerance)."""
    rng = np.random.default_rng(18)
    N, I, Tb, k = 65536, 16, 256, 200
    planes, scales = random_corpus(rng, N, 64, 2)
    recs = []
    for _ in range(12):
        qp, qs = random_query(rng, 64, 2)
        exact, _ = oracle.topk(planes, scales, qp, qs, k)
        nl, _ = oracle.nearlossless(planes, scales, qp, qs, k, I=I, Tb=Tb)
        recs.append(oracle.recall(nl, exact))
    expect = oracle.expected_recall(k, N, I)
    assert abs(np.mean(recs) - expect) < 4 * math.sqrt(expect * (1 - expect) / (k * len(recs))) + 1e-3


# ---------------------------------------------------------------- input generator vs encoder
def test_torch_packer_agrees_with_oracle_encoder():
    import torch
    c = rbe_synth.centres_torch(16, 128, "cpu")
    x = rbe_synth.vectors_torch(2000, c, 0.3, seed=19)
    pl, sc = rbe_synth.pack_planes_torch(x, 4)
    opl, osc = oracle.encode(x.numpy(), 4)
    # bits may differ only where a residual is within rounding of zero
    diff_bits = int(sum(bin(int(v)).count("1") for v in (pl.numpy().view(np.uint64) ^ opl).ravel()))
    assert diff_bits <= 4
    np.testing.assert_allclose(sc.numpy(), osc, rtol=1e-5)
    assert torch.allclose(torch.linalg.vector_norm(x, dim=1), torch.ones(2000), atol=1e-5)
