"""Full-size parity: the 1e9-item configurations, searched in the launch
configuration bench.py times, checked against the CPU oracle.

The corpus is generated on the device in seeded chunks (the same chunks can be
regenerated at will), loaded into the library, and streamed back chunk by chunk
for the oracle.  At 1e9 items every query of every call (the one-query call, the
16-query matrix-core call, the 8-query k = 4000 call) gets a full oracle scan of
every item; at the other sizes a spread of queries does, and the remaining ones are
checked on what the oracle can compute one by one: the oracle score of every
returned id, and completeness over sampled chunks (no item of a sampled chunk may
beat the returned k-th score by more than the tolerance).

The oracle itself stays single-threaded C; the harness calls it from several host
threads on disjoint item ranges of a chunk (ctypes releases the interpreter lock
during the call) and merges the per-range results with oracle.topk_of_scores."""
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest

import oracle
import paper_1802_06466_amd as rbe
import rbe_synth
from parity import REL

pytestmark = pytest.mark.gpu

CHUNK = 4_000_000
N_THREADS = max(1, min(16, os.cpu_count() or 1))
POOL = ThreadPoolExecutor(N_THREADS)


def ranges(n, parts=N_THREADS):
    edges = np.linspace(0, n, parts + 1).astype(np.int64)
    return [(int(a), int(b)) for a, b in zip(edges[:-1], edges[1:]) if b > a]


def build(N, d, P, n_clusters, sigma, progress, flags=0):
    import torch
    dev = torch.device("cuda:0")
    centres = rbe_synth.centres_torch(n_clusters, d, dev)
    ix = rbe.rbe_index_create(N, d, P, flags)
    for c, z0 in enumerate(range(0, N, CHUNK)):
        n = min(CHUNK, N - z0)
        x = rbe_synth.vectors_torch(n, centres, sigma, rbe_synth.SEED_ITEMS, c)
        planes, scales = rbe_synth.pack_planes_torch(x, P)
        rbe.rbe_load_chunk(ix, z0, planes, None if flags & rbe.RBE_DYADIC else scales)
        if c % 50 == 0:
            print(f"  {progress}: loaded {z0 + n} items", flush=True)
    rbe.rbe_finalize(ix)
    torch.cuda.empty_cache()
    return ix, centres


def chunk_on_host(c, N, centres, sigma, P, dyadic_cosine=False):
    """Chunk c regenerated for the oracle.  dyadic_cosine: the planes alone are the corpus (weights
    2^-j); the oracle gets those weights divided by the reconstructed norm (Sec. 5.1)."""
    z0 = c * CHUNK
    n = min(CHUNK, N - z0)
    x = rbe_synth.vectors_torch(n, centres, sigma, rbe_synth.SEED_ITEMS, c)
    planes, scales = rbe_synth.pack_planes_torch(x, P)
    planes = planes.cpu().numpy().view(np.uint64)
    if dyadic_cosine:
        return z0, planes, None          # oracle scales are derived per subset, see dyadic_cosine_scales
    return z0, planes, scales.cpu().numpy()


def dyadic_cosine_scales(planes):
    """Scales the oracle scores a dyadic + stored-norm corpus with: 2^-j divided by the norm of the
    reconstruction (Sec. 5.1), by oracle.fold_cosine on disjoint item ranges."""
    P, n = planes.shape[0], planes.shape[1]
    w = np.array([2.0 ** -j for j in range(P)], dtype=np.float32)[:, None] * np.ones((P, n), dtype=np.float32)
    if n < 100_000:
        return oracle.fold_cosine(planes, w)
    out = np.empty((P, n), dtype=np.float32)
    def part(a, b):
        out[:, a:b] = oracle.fold_cosine(np.ascontiguousarray(planes[:, a:b]), np.ascontiguousarray(w[:, a:b]))
    list(POOL.map(lambda r: part(*r), ranges(n)))
    return out


def queries(centres, n, sigma, P):
    x = rbe_synth.vectors_torch(n, centres, sigma, rbe_synth.SEED_QUERIES, 7).cpu().numpy()
    enc = [rbe.rbe_encode_query(x[i], P) for i in range(n)]
    return np.stack([e[0] for e in enc]), np.stack([e[1] for e in enc])


def verify(N, centres, sigma, P, qp, qs, k, ids, sc, full_scan_queries, sampled_chunks, label, dyadic_cosine=False):
    """ids/sc: [Q][k] results.  Queries listed in full_scan_queries get the exact oracle top-k
    over every chunk; all queries get per-id score checks and completeness on sampled_chunks."""
    Q = qp.shape[0]
    n_chunks = -(-N // CHUNK)
    true_sc = np.full((Q, k), np.nan)
    merged = {q: (np.empty(0, np.int64), np.empty(0)) for q in full_scan_queries}
    kth = sc[:, k - 1].astype(np.float64)
    for c in range(n_chunks):
        z0, planes, scales = chunk_on_host(c, N, centres, sigma, P, dyadic_cosine)
        n = planes.shape[1]
        need_all = bool(merged) or c in sampled_chunks
        if dyadic_cosine and need_all:
            scales = dyadic_cosine_scales(planes)
        parts = ranges(n)
        topk_jobs, dense_jobs = {}, {}
        for q in range(Q):
            sel = np.flatnonzero((ids[q] >= z0) & (ids[q] < z0 + n))
            if sel.size:
                loc = ids[q][sel] - z0
                if scales is None:        # only the returned items of this chunk are needed
                    sub = np.ascontiguousarray(planes[:, loc])
                    true_sc[q, sel] = oracle.scores_at(sub, dyadic_cosine_scales(sub), qp[q], qs[q], np.arange(loc.size))
                else:
                    true_sc[q, sel] = oracle.scores_at(planes, scales, qp[q], qs[q], loc)
            if q in merged:
                topk_jobs[q] = [POOL.submit(oracle.topk, planes, scales, qp[q], qs[q], k, a, b) for a, b in parts]
            elif c in sampled_chunks:
                dense_jobs[q] = [POOL.submit(oracle.scores, planes, scales, qp[q], qs[q], a, b) for a, b in parts]
        for q, jobs in topk_jobs.items():
            got = [j.result() for j in jobs]                 # ids are chunk-local item numbers
            a_ids = np.concatenate([merged[q][0]] + [g[0][g[0] >= 0] + z0 for g in got])
            a_sc = np.concatenate([merged[q][1]] + [g[1][g[0] >= 0] for g in got])
            merged[q] = oracle.topk_of_scores(a_sc, a_ids, k)
        for q, jobs in dense_jobs.items():
            s = np.concatenate([j.result() for j in jobs])
            eps = REL * abs(kth[q])
            better = np.flatnonzero(s > kth[q] + eps) + z0
            assert set(better.tolist()) <= set(ids[q].tolist()), f"{label}: query {q} missed an item of chunk {c}"
        if c % 50 == 0:
            print(f"  {label}: oracle at chunk {c}/{n_chunks}", flush=True)
    for q in range(Q):
        assert np.unique(ids[q]).size == k and ids[q].min() >= 0 and ids[q].max() < N
        np.testing.assert_allclose(sc[q], true_sc[q], rtol=REL, err_msg=f"{label}: query {q} scores")
        assert np.all(sc[q][:-1] >= sc[q][1:])
    for q, (o_ids, o_sc) in merged.items():
        eps = REL * abs(o_sc[-1])
        assert set(o_ids[o_sc > o_sc[-1] + eps].tolist()) <= set(ids[q].tolist()), f"{label}: query {q} missed a top item"
        assert np.all(true_sc[q] >= o_sc[-1] - eps), f"{label}: query {q} returned an item below the k-th best"
    print(f"  {label}: full oracle scans for queries {sorted(merged)} agree", flush=True)


def test_1e7_items_batch32_top1000_full_oracle():
    """10,000,000 items, d=64, 3 planes, 1024 clusters, 32 queries, k=1000: every query against a
    full oracle scan (host-generated corpus, oracle encoder)."""
    from parity import check_batch
    N, d, P, k, Q = 10_000_000, 64, 3, 1000, 32
    c = rbe_synth.centres_numpy(1024, d)
    planes = np.empty((P, N, 1), dtype=np.uint64)
    scales = np.empty((P, N), dtype=np.float32)
    step = 2_000_000
    for i, z0 in enumerate(range(0, N, step)):
        x = rbe_synth.vectors_numpy(step, c, 0.3, seed=rbe_synth.SEED_ITEMS, chunk=i)
        pl, sc = oracle.encode(x, P)
        planes[:, z0:z0 + step] = pl
        scales[:, z0:z0 + step] = sc
    print("  1e7: corpus encoded", flush=True)
    q = rbe_synth.vectors_numpy(Q, c, 0.3, seed=rbe_synth.SEED_QUERIES)
    qp = np.stack([rbe.rbe_encode_query(q[i], P)[0] for i in range(Q)])
    qs = np.stack([rbe.rbe_encode_query(q[i], P)[1] for i in range(Q)])
    ix = rbe.rbe_load_corpus(planes, scales)
    ids, sc = rbe.rbe_search(ix, qp, qs, k)
    assert not rbe.rbe_get_search_stats(ix)["fallback"]
    rbe.rbe_free(ix)
    check_batch(planes, scales, qp, qs, k, ids, sc)


def test_1e8_items_d128_4planes_batch64_top1000():
    N, d, P, k, sigma, Q = 100_000_000, 128, 4, 1000, 0.3, 64
    ix, centres = build(N, d, P, 4096, sigma, "1e8 d128")
    qp, qs = queries(centres, Q, sigma, P)
    ids, sc = rbe.rbe_search(ix, qp, qs, k)
    assert not rbe.rbe_get_search_stats(ix)["fallback"]
    rbe.rbe_free(ix)
    verify(N, centres, sigma, P, qp, qs, k, ids, sc, full_scan_queries=list(range(0, 64, 3)) + [63], sampled_chunks={1, 12},
           label="1e8 d128 k=1000")


def test_1e9_items_single_query_and_batch16_top1000():
    N, d, P, k, sigma = 1_000_000_000, 64, 3, 1000, 0.3
    ix, centres = build(N, d, P, 4096, sigma, "1e9 sigma 0.3")
    qp, qs = queries(centres, 17, sigma, P)
    ids1, sc1 = rbe.rbe_search(ix, qp[:1], qs[:1], k)                    # the timed configuration: one query
    st = rbe.rbe_get_search_stats(ix)
    assert not st["fallback"] and st["n_levels"] - st["last_level_parts"] == 3
    ids16, sc16 = rbe.rbe_search(ix, qp[1:], qs[1:], k)                  # batch of 16
    near, nsc = rbe.rbe_search(ix, qp[:1], qs[:1], k, mode=rbe.RBE_SELECT_NEARLOSSLESS, group_size_I=256)
    rbe.rbe_free(ix)
    ids = np.concatenate([ids1, ids16]); sc = np.concatenate([sc1, sc16])
    # full oracle scans of all 1e9 items for every query: the one-query call and all 16 of the matrix-core call
    verify(N, centres, sigma, P, qp, qs, k, ids, sc, full_scan_queries=list(range(17)), sampled_chunks=set(),
           label="1e9 k=1000")
    # the near-lossless result loses at most a handful of the exact top 1000 (Appendix A: 0.13 expected)
    lost = k - len(set(near[0].tolist()) & set(ids1[0].tolist()))
    assert lost <= 4
    assert np.all(np.isin(near[0], ids1[0]) | (nsc[0] <= sc1[0][-1]))


def test_1e9_near_duplicate_clusters_batch8_top4000():
    N, d, P, k, sigma = 1_000_000_000, 64, 3, 4000, 0.05
    ix, centres = build(N, d, P, 4096, sigma, "1e9 sigma 0.05")
    qp, qs = queries(centres, 8, sigma, P)
    ids, sc = rbe.rbe_search(ix, qp, qs, k)
    assert not rbe.rbe_get_search_stats(ix)["fallback"]
    near, _ = rbe.rbe_search(ix, qp, qs, k, mode=rbe.RBE_SELECT_NEARLOSSLESS, group_size_I=256)
    rbe.rbe_free(ix)
    verify(N, centres, sigma, P, qp, qs, k, ids, sc, full_scan_queries=list(range(8)), sampled_chunks=set(),
           label="1e9 k=4000")
    rec = np.mean([len(set(near[q].tolist()) & set(ids[q].tolist())) / k for q in range(8)])
    expect = oracle.expected_recall(k, 15259 * 65536, 256)
    print(f"  near-lossless recall {rec:.5f}, Appendix A predicts {expect:.5f}", flush=True)
    assert abs(rec - expect) < 1.5e-3


def test_paper_operating_point_1212153856_items_dyadic():
    """The paper's own operating point at full size: 136^2 x 256^2 keywords, 2 keyword + 3 query bits per
    dimension, residual weights 2^-t, stored inverse norm (20 B per keyword).  One query (shift-add kernel),
    16 queries (matrix cores, one query half) and the near-lossless selector; every returned score against
    the oracle, completeness on sampled chunks."""
    N, d, P, Pq, k, sigma = 136 * 136 * 256 * 256, 64, 2, 3, 1000, 0.3
    ix, centres = build(N, d, P, 4096, sigma, "paper point", flags=rbe.RBE_DYADIC | rbe.RBE_COSINE)
    qp, _ = queries(centres, 17, sigma, Pq)
    qs = np.tile(np.array([2.0 ** -i for i in range(Pq)], dtype=np.float32), (17, 1))
    ids1, sc1 = rbe.rbe_search(ix, qp[:1], None, k)
    assert not rbe.rbe_get_search_stats(ix)["fallback"]
    ids16, sc16 = rbe.rbe_search(ix, qp[1:], None, k)
    near, nsc = rbe.rbe_search(ix, qp[:1], None, k, mode=rbe.RBE_SELECT_NEARLOSSLESS, group_size_I=256)
    rbe.rbe_free(ix)
    ids = np.concatenate([ids1, ids16]); sc = np.concatenate([sc1, sc16])
    # full oracle scans (norm fold of every item included) for the one-query call and one query of the 16-query call
    verify(N, centres, sigma, P, qp, qs, k, ids, sc, full_scan_queries=[0, 1, 9, 16],
           sampled_chunks={0, 61, 150, 303}, label="paper point", dyadic_cosine=True)
    lost = k - len(set(near[0].tolist()) & set(ids1[0].tolist()))
    assert lost <= 4
