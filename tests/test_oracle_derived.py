"""Pins of the derived-quantizer oracle (thesis chapter 6) against things other than itself:
literal simulations of the data structures of Alg. 5, brute force from the definitions, the
properties Alg. 4 promises, and special cases that reduce to the plain ADC search."""
import heapq

import numpy as np
import pytest

from oracle import derived_oracle as dq
from oracle import pq_oracle as orc


def rng(seed):
    return np.random.default_rng(seed)


# ---------------------------------------------------------------------------------------------
# Alg. 4
def test_same_size_partition_and_property_p1_small_figure_shape():
    """k = 16, kbar = 4 as in the figure of Section 6.2.2: four clusters of four centroids,
    index low bits = cluster (P1), derived centroid = mean of its cluster."""
    r = rng(1)
    temp = r.normal(size=(16, 2)).astype(np.float32)
    cbar, assign = dq.kmeans_same_size(temp, 4, 5, [0, 5, 10, 15])
    assert sorted(np.bincount(assign, minlength=4).tolist()) == [4, 4, 4, 4]
    final = dq.build_final_codebook(temp, assign, 4)
    # every temporary centroid appears exactly once
    assert sorted(map(tuple, final.tolist())) == sorted(map(tuple, temp.tolist()))
    for i in range(16):
        src = np.nonzero((temp == final[i]).all(1))[0][0]
        assert assign[src] == (i & 3)                       # P1
    for l in range(4):
        np.testing.assert_allclose(cbar[l], final[l::4].astype(np.float64).mean(0), rtol=1e-6)
    # members of a cluster keep their temporary order: index >> 2 counts them
    for l in range(4):
        members = np.nonzero(assign == l)[0]
        for i, src in enumerate(members):
            assert np.array_equal(final[(i << 2) | l], temp[src])


def test_same_size_assignment_prefers_the_closest_pairs():
    """Two tight pairs and capacity two: the greedy hand-out must not split a pair."""
    pts = np.array([[0.0], [0.1], [10.0], [10.1]], np.float32)
    cbar, assign = dq.kmeans_same_size(pts, 2, 3, [0, 2])
    assert assign[0] == assign[1] and assign[2] == assign[3] and assign[0] != assign[2]
    np.testing.assert_allclose(np.sort(cbar[:, 0]), [0.05, 10.05], rtol=1e-6)


def test_train_derived_quantizer_of_a_vector_is_the_low_bits_of_its_code():
    """Section 6.2.2, last paragraph: the derived quantizer needs no second encoding; the low
    bits of the code name a cluster whose members include the code's centroid."""
    r = rng(2)
    x = r.normal(size=(600, 4)).astype(np.float32)
    final, cbar = dq.train_derived(x, 64, 8, 3, np.arange(64) * 9, np.arange(8) * 8)
    codes = dq.encode16(x[:50], final[None])
    for c in codes[:, 0]:
        group = final[(np.arange(64) & 7) == (int(c) & 7)]
        assert any(np.array_equal(final[int(c)], g) for g in group)
    # the derived centroid is the mean of the 8 members of its cluster
    for l in range(8):
        np.testing.assert_allclose(cbar[l], final[l::8].astype(np.float64).mean(0), rtol=1e-5, atol=1e-6)


# ---------------------------------------------------------------------------------------------
# Alg. 5, Step 1.3: capped buckets, simulated literally
class CappedBuckets:
    """One list of ids per integer distance; vectors above the bucket of the r2-th farthest kept
    vector are discarded (Section 6.2.3, Step 1.3)."""

    def __init__(self, r2, nbuckets):
        self.r2 = r2
        self.buckets = [[] for _ in range(nbuckets)]
        self.bound = nbuckets - 1
        self.kept = 0

    def put(self, d, i):
        if d > self.bound:
            return
        self.buckets[d].append(i)
        self.kept += 1
        # lower the bound while the buckets below it already hold r2 vectors
        while self.kept - len(self.buckets[self.bound]) >= self.r2:
            self.kept -= len(self.buckets[self.bound])
            self.buckets[self.bound] = []
            self.bound -= 1

    def take(self):
        out, count, b = [], 0, 0
        while count < self.r2 and b < len(self.buckets):
            out += self.buckets[b]
            count += len(self.buckets[b])
            b += 1
        return b - 1, out


@pytest.mark.parametrize("n,r2,top", [(500, 40, 30), (500, 40, 3), (64, 100, 20), (300, 1, 9), (1000, 999, 50)])
def test_candidates_equal_literal_capped_buckets(n, r2, top):
    r = rng(n + r2)
    sums = r.integers(0, top, n)
    cb = CappedBuckets(r2, top)
    for i, d in enumerate(sums):
        cb.put(int(d), i)
    last, ids = cb.take()
    s_star, got = dq.candidates(sums, r2)
    assert sorted(ids) == got.tolist()
    if n >= r2:
        assert last == s_star
        assert (sums < s_star).sum() < r2 <= (sums <= s_star).sum()
    else:
        assert len(got) == n


def test_candidates_empty_database():
    s_star, ids = dq.candidates(np.empty(0, np.int64), 10)
    assert s_star == -1 and len(ids) == 0


# ---------------------------------------------------------------------------------------------
# Alg. 5, Step 2: lazily filled tables and a binary heap, simulated literally
def test_rerank_equals_lazily_filled_tables_with_a_heap():
    r = rng(5)
    m, k, dsub, n, topk = 3, 512, 4, 400, 7
    cb = r.normal(size=(m, k, dsub)).astype(np.float32)
    codes = r.integers(0, k, (n, m)).astype(np.uint16)
    codes[10] = codes[3]                                   # equal distances: the smaller id wins
    y = r.normal(size=m * dsub).astype(np.float32)
    cand = np.sort(r.choice(n, 150, replace=False))
    cand = np.union1d(cand, [3, 10])
    table = np.full((m, k), -1.0, np.float32)
    computed = 0
    heap = []                                              # max-heap on (distance, id) through negation
    for i in cand:
        d = 0.0
        for j in range(m):
            c = int(codes[i, j])
            if table[j, c] == -1.0:
                diff = y[j * dsub:(j + 1) * dsub].astype(np.float64) - cb[j, c].astype(np.float64)
                table[j, c] = np.float32((diff * diff).sum())
                computed += 1
            d += float(table[j, c])
        d = float(np.float32(d))
        item = (-d, -int(i))
        if len(heap) < topk:
            heapq.heappush(heap, item)
        elif item > heap[0]:
            heapq.heapreplace(heap, item)
    ref = sorted((-a, -b) for a, b in heap)
    got_d, got_i = dq.rerank_exact(codes, cand, cb, y, topk)
    assert [i for _, i in ref] == got_i.tolist()
    np.testing.assert_array_equal(np.array([d for d, _ in ref], np.float32), got_d)
    assert computed < m * k                                # only the entries the candidates touch


def test_rerank_pads_when_candidates_are_few():
    r = rng(6)
    cb = r.normal(size=(2, 300, 2)).astype(np.float32)
    codes = r.integers(0, 300, (5, 2)).astype(np.uint16)
    d, i = dq.rerank_exact(codes, np.array([4, 1]), cb, r.normal(size=4).astype(np.float32), 4)
    assert i[2:].tolist() == [-1, -1] and np.isinf(d[2:]).all() and set(i[:2].tolist()) == {1, 4}


# ---------------------------------------------------------------------------------------------
# adc_low_bits and qmax against the plain ADC routines on the low bytes
def test_low_bits_sums_and_qmax_equal_plain_adc_on_the_low_bytes():
    r = rng(7)
    nq, m, n = 5, 4, 3000
    codes = r.integers(0, 65536, (n, m)).astype(np.uint16)
    dluts = (r.random((nq, m, 256)) * 50).astype(np.float32)
    qluts = r.integers(0, 256, (nq, m, 256)).astype(np.uint8)
    low = (codes & 255).astype(np.uint8)
    sums = dq.low_bits_sums(codes, qluts)
    for q in range(nq):
        np.testing.assert_array_equal(sums[q], orc.adc_all_u8(low, orc.CODES_U8, qluts[q]))
        brute = [sum(int(qluts[q, j, codes[i, j] % 256]) for j in range(m)) for i in range(0, n, 97)]
        assert brute == sums[q, ::97].tolist()
    qmax = dq.derived_qmax(codes, dluts, 700)
    for q in range(nq):
        assert qmax[q] == orc.adc_all_f32(low[:700], orc.CODES_U8, dluts[q]).max()


# ---------------------------------------------------------------------------------------------
# whole search
def make_problem(seed, n, m, k, kbar, dsub, nq):
    """Codebooks with property P1 by construction: cluster centres, members scattered around them."""
    r = rng(seed)
    centres = r.normal(size=(m, kbar, dsub)) * 4
    cb = np.empty((m, k, dsub), np.float32)
    for i in range(k):
        cb[:, i] = centres[:, i % kbar] + r.normal(size=(m, dsub)) * 0.5
    cbar = np.stack([np.stack([cb[j, l::kbar].astype(np.float64).mean(0) for l in range(kbar)]) for j in range(m)])
    codes = r.integers(0, k, (n, m)).astype(np.uint16)
    queries = (r.normal(size=(nq, m * dsub)) * 4).astype(np.float32)
    return cb, cbar.astype(np.float32), codes, queries


def test_search_against_brute_force_from_the_definitions():
    m, k, kbar, dsub, n, nq, r2, topk = 4, 1024, 256, 3, 700, 3, 60, 10
    cb, cbar, codes, queries = make_problem(11, n, m, k, kbar, dsub, nq)
    out_d, out_i, s_star, cands, dluts, qmax, qluts = dq.search(codes, cbar, cb, queries, r2, topk)
    for q in range(nq):
        y = queries[q].astype(np.float64)
        # Step 1.1: compact tables straight from Eq. (tables)
        D = np.array([[((y[j * dsub:(j + 1) * dsub] - cbar[j, i].astype(np.float64)) ** 2).sum() for i in range(kbar)]
                      for j in range(m)]).astype(np.float32)
        np.testing.assert_allclose(D, dluts[q], rtol=1e-6)
        # Step 1.2: 255 bins between the smallest table entry and the greatest of the first r2 distances
        first = [np.float32(sum(float(dluts[q, j, codes[i, j] & 255]) for j in range(m))) for i in range(r2)]
        assert qmax[q] == max(first)
        qmin = dluts[q].min()
        width = (np.float64(qmax[q]) - np.float64(qmin)) / 255.0
        binned = np.minimum(255, np.floor((dluts[q].astype(np.float64) - qmin) / width))
        assert np.abs(binned - qluts[q]).max() <= 1           # float32 sequence vs float64: a bin edge may move
        # Step 1.3: integer distances, buckets in increasing order until r2 vectors are in
        s = np.array([sum(int(qluts[q, j, codes[i, j] & 255]) for j in range(m)) for i in range(n)])
        order = np.sort(s)
        assert s_star[q] == order[r2 - 1]
        assert cands[q].tolist() == np.nonzero(s <= order[r2 - 1])[0].tolist()
        # Step 2: precise distances of the candidates, r smallest
        exact = {}
        for i in cands[q]:
            t = 0.0
            for j in range(m):
                diff = y[j * dsub:(j + 1) * dsub] - cb[j, codes[i, j]].astype(np.float64)
                t += float(np.float32((diff * diff).sum()))
            exact[int(i)] = np.float32(t)
        best = sorted(exact.items(), key=lambda kv: (kv[1], kv[0]))[:topk]
        assert [i for i, _ in best] == out_i[q].tolist()
        np.testing.assert_array_equal(np.array([d for _, d in best], np.float32), out_d[q])
        # and the precise distance is the distance to the reconstructed vector (Eq. adc2)
        i0 = int(out_i[q, 0])
        recon = np.concatenate([cb[j, codes[i0, j]] for j in range(m)]).astype(np.float64)
        np.testing.assert_allclose(out_d[q, 0], ((y - recon) ** 2).sum(), rtol=1e-5)


def test_search_with_every_code_as_candidate_is_the_plain_adc_search():
    """kbar = k = 256 and r2 >= n: derived and full quantizers coincide, every vector is reranked,
    so the result is the plain 8-bit ADC search with the full tables."""
    r = rng(13)
    m, k, dsub, n, nq, topk = 4, 256, 4, 900, 4, 15
    cb = r.normal(size=(m, k, dsub)).astype(np.float32)
    codes = r.integers(0, k, (n, m)).astype(np.uint16)
    queries = r.normal(size=(nq, m * dsub)).astype(np.float32)
    out_d, out_i, s_star, cands = dq.search(codes, cb, cb, queries, n + 5, topk)[:4]
    ref_d, ref_i = orc.adc_scan_topk_f32(codes.astype(np.uint8), orc.CODES_U8, orc.build_luts(queries, cb), topk)
    np.testing.assert_array_equal(out_i, ref_i)
    np.testing.assert_array_equal(out_d, ref_d)
    assert all(len(c) == n for c in cands)


def test_candidate_set_contains_the_r2_best_integer_distances_and_whole_last_bucket():
    m, k, kbar, dsub, n, nq, r2 = 4, 512, 256, 2, 5000, 2, 300
    cb, cbar, codes, queries = make_problem(17, n, m, k, kbar, dsub, nq)
    _, _, s_star, cands, _, _, qluts = dq.search(codes, cbar, cb, queries, r2, 5)
    sums = dq.low_bits_sums(codes, qluts)
    for q in range(nq):
        assert len(cands[q]) >= r2
        assert sums[q][cands[q]].max() == s_star[q]
        outside = np.setdiff1d(np.arange(n), cands[q])
        assert sums[q][outside].min() > s_star[q]
