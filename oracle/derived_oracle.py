"""CPU oracle of the search with derived quantizers (thesis chapter 6).

TEST INFRASTRUCTURE ONLY: the test-suite, the smoke check and the benchmark's
CPU-baseline leg may import this module; the GPU library and its Python binding
never do.  Plain numpy, float sums in float64 rounded once to float32, integer
work in integers; nothing here is blocked, fused or reordered.

What it follows:
  - Section 6.2.2, Alg. 4 (training): k-means, partition of the temporary codebook into
    clusters of identical size, final codebook ordered so that the low bits of a centroid's
    index name its cluster (property P1).
  - Section 6.2.3, Alg. 5 (search): compact tables from the derived codebooks (Step 1.1),
    their 8-bit quantisation with qmax = the greatest distance among the first r2 codes
    (Step 1.2), scan with adc_low_bits into buckets indexed by the integer distance
    (Step 1.3), precise distances with the full codebooks for the vectors of the buckets
    taken in increasing order until r2 vectors have been processed (Step 2).

Readings (the thesis leaves these open):
  - kmeans_same_size is cited, not specified: Lloyd iterations whose assignment step hands
    out the (point, cluster) pairs in order of increasing distance (ties: smaller point,
    then smaller cluster) while the cluster still has room.
  - The rerank loop of Alg. 5 finishes the bucket in which the r2-th vector falls, so the
    candidate set is every code whose integer distance is at most that bucket's; the
    sentence of Step 2 that speaks of r2 vectors is read as the loop's entry condition.
  - Integer distances are plain sums of the 8-bit entries (no saturation), so bucket
    indexes run to m * 255; the tables are quantised as everywhere else in this oracle.
  - Ties of the final distances go to the smaller id.

Parity status: pinned by tests/test_oracle_derived.py (literal capped-buckets simulation,
lazily filled tables, brute force from the definitions, property P1, closed forms).
Recall on the thesis's datasets: parity unpinned (datasets unavailable).
"""
import numpy as np

from oracle import pq_oracle as orc


# ---------------------------------------------------------------------------------------------
# Section 6.2.2, Alg. 4: training
def kmeans_same_size(points, kbar, iters, init_idx):
    """Step 2 of Alg. 4: kbar clusters of identical size len(points) / kbar.

    Returns (centroids [kbar][dim] float32, assign [len(points)] int64).  Each centroid is the
    mean of its cluster ("centroids of centroids" when the points are a codebook)."""
    pts = np.asarray(points, dtype=np.float64)
    k = len(pts)
    assert k % kbar == 0
    cap = k // kbar
    cent = pts[np.asarray(init_idx, dtype=np.int64)].copy()
    assign = np.full(k, -1, np.int64)
    for _ in range(max(1, iters)):
        dist = ((pts[:, None, :] - cent[None, :, :]) ** 2).sum(-1)          # [k][kbar]
        order = np.lexsort((np.tile(np.arange(kbar), k), np.repeat(np.arange(k), kbar), dist.ravel()))
        assign[:] = -1
        room = np.full(kbar, cap, np.int64)
        left = k
        for flat in order:
            p, c = divmod(int(flat), kbar)
            if assign[p] < 0 and room[c] > 0:
                assign[p] = c
                room[c] -= 1
                left -= 1
                if left == 0:
                    break
        for c in range(kbar):
            cent[c] = pts[assign == c].mean(axis=0)
    return cent.astype(np.float32), assign


def build_final_codebook(temp_codebook, assign, kbar):
    """Step 3 of Alg. 4: the i-th member (in temporary-index order) of cluster l gets the
    index (i << log2(kbar)) | l, so the low bits of an index name the cluster (P1)."""
    temp = np.asarray(temp_codebook, dtype=np.float32)
    k = len(temp)
    bbar = int(kbar).bit_length() - 1
    assert 1 << bbar == kbar
    final = np.empty_like(temp)
    for l in range(kbar):
        members = np.nonzero(assign == l)[0]
        for i, src in enumerate(members):
            final[(i << bbar) | l] = temp[src]
    assert k == kbar * (k // kbar)
    return final


def train_derived(x_sub, k, kbar, iters, init_idx, init_idx_bar, iters_bar=3):
    """Alg. 4 for one sub-space: (final codebook [k][dim], derived codebook [kbar][dim])."""
    temp = orc.kmeans(x_sub, k, iters, init_idx)                              # Step 1
    cbar, assign = kmeans_same_size(temp, kbar, iters_bar, init_idx_bar)       # Step 2
    return build_final_codebook(temp, assign, kbar), cbar                      # Step 3


def encode16(x, codebooks):
    """Section 2.3.1 encoder with codebooks of up to 65536 centroids: uint16 [n][m];
    nearest centroid per sub-space in float64, ties to the smaller index."""
    x = np.asarray(x, dtype=np.float64)
    m, k, dsub = codebooks.shape
    codes = np.empty((len(x), m), np.uint16)
    for j in range(m):
        cj = codebooks[j].astype(np.float64)
        for i0 in range(0, len(x), 256):
            xs = x[i0:i0 + 256, j * dsub:(j + 1) * dsub]
            dist = ((xs[:, None, :] - cj[None, :, :]) ** 2).sum(-1)
            codes[i0:i0 + 256, j] = dist.argmin(1)
    return codes


# ---------------------------------------------------------------------------------------------
# Section 6.2.3, Alg. 5: search
def low_bits(codes16, bbar=8):
    return (np.asarray(codes16, dtype=np.uint16) & np.uint16((1 << bbar) - 1)).astype(np.int64)


def derived_qmax(codes16, dluts, r2):
    """Step 1.2: the greatest distance (compact float tables, low bits of the indexes) between
    each query and the first r2 codes.  dluts [nq][m][256] float32 -> float32 [nq]."""
    low = low_bits(codes16[:r2])
    nq, m, _ = dluts.shape
    out = np.empty(nq, np.float32)
    for q in range(nq):
        d = np.zeros(len(low), np.float64)
        for j in range(m):
            d += dluts[q, j][low[:, j]].astype(np.float64)
        out[q] = np.float32(d.astype(np.float32).max()) if len(low) else np.float32(0)
    return out


def low_bits_sums(codes16, qluts):
    """adc_low_bits of Alg. 5 for every code: uint32 [nq][n], plain integer sums."""
    low = low_bits(codes16)
    nq, m, _ = qluts.shape
    out = np.zeros((nq, len(low)), np.uint32)
    for q in range(nq):
        for j in range(m):
            out[q] += qluts[q, j][low[:, j]].astype(np.uint32)
    return out


def candidates(sums, r2):
    """Step 1.3 + the bucket loop of Step 2 for one query: the bucket in which the r2-th vector
    falls, and the ids of every code in the buckets up to and including it (ascending ids).
    Fewer than r2 codes: all of them, and the last occupied bucket."""
    sums = np.asarray(sums, dtype=np.int64)
    if len(sums) == 0:
        return -1, np.empty(0, np.int64)
    hist = np.bincount(sums)
    cum = np.cumsum(hist)
    s_star = int(np.searchsorted(cum, min(r2, len(sums))))
    return s_star, np.nonzero(sums <= s_star)[0].astype(np.int64)


def rerank_exact(codes16, cand_ids, codebooks, query, topk):
    """Step 2: distance of every candidate from the full codebooks,
    sum_j || y^j - C^j[c[j]] ||^2 with each term rounded to float32 as a table entry would be
    (Eq. tables) and the m terms added in float64, rounded once (Eq. adc1); the topk smallest
    (distance, id).  Padded with (+inf, -1)."""
    m, k, dsub = codebooks.shape
    y = np.asarray(query, dtype=np.float64)
    cand_ids = np.asarray(cand_ids, dtype=np.int64)
    d = np.zeros(len(cand_ids), np.float64)
    for j in range(m):
        cent = codebooks[j][codes16[cand_ids, j].astype(np.int64)].astype(np.float64)
        term = ((y[None, j * dsub:(j + 1) * dsub] - cent) ** 2).sum(-1)
        d += term.astype(np.float32).astype(np.float64)
    d = d.astype(np.float32)
    order = np.lexsort((cand_ids, d))[:topk]
    out_d = np.full(topk, np.inf, np.float32)
    out_i = np.full(topk, -1, np.int64)
    out_d[:len(order)] = d[order]
    out_i[:len(order)] = cand_ids[order]
    return out_d, out_i


def search(codes16, derived_codebooks, codebooks, queries, r2, topk):
    """nns_derived of Alg. 5 for a batch of queries.
    Returns dist [nq][topk], ids [nq][topk], s_star [nq], cand (list of id arrays), and the
    intermediate tables (dluts, qmax, qluts) so that a test can feed the same bits to both sides."""
    queries = np.asarray(queries, dtype=np.float32)
    dluts = orc.build_luts(queries, derived_codebooks)                        # Step 1.1
    qmax = derived_qmax(codes16, dluts, r2)                                   # Step 1.2
    qluts, _, _ = orc.quantize_luts(dluts, qmax)
    return search_from_tables(codes16, qluts, codebooks, queries, r2, topk) + (dluts, qmax, qluts)


def search_from_tables(codes16, qluts, codebooks, queries, r2, topk):
    """Steps 1.3 and 2 from given 8-bit tables."""
    nq = len(queries)
    sums = low_bits_sums(codes16, qluts)
    out_d = np.empty((nq, topk), np.float32)
    out_i = np.empty((nq, topk), np.int64)
    s_star = np.empty(nq, np.int64)
    cands = []
    for q in range(nq):
        s_star[q], ids = candidates(sums[q], r2)                              # Step 1.3
        cands.append(ids)
        out_d[q], out_i[q] = rerank_exact(codes16, ids, codebooks, queries[q], topk)   # Step 2
    return out_d, out_i, s_star, cands
