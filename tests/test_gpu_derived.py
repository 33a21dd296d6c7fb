"""Search with derived quantizers (chapter 6, Alg. 5) on the GPU against the oracle.

Stage-wise bit-exactness: the compact float tables are taken from the GPU (pq_build_luts, the same
kernel the search runs inside) and handed to the oracle, so that qmax, the 8-bit tables, every
integer distance, the bucket b* and the candidate set must agree bit for bit; the precise distances
of Step 2 agree within 1e-5 and the final ids up to ties inside that tolerance."""
import numpy as np
import pytest
import torch

from oracle import derived_oracle as dq
from oracle import pq_oracle as orc
from paper_1712_02912_amd import binding
from util import check_float_topk_ranked

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    c = binding.Context(0)
    yield c
    torch.cuda.synchronize()
    c.close()


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def make_problem(seed, n, k, dsub, nq, distinct=None):
    """Codebooks with property P1 by construction (index low byte = cluster), random codes."""
    r = np.random.default_rng(seed)
    m, kbar = 4, 256
    centres = r.normal(size=(m, kbar, dsub)) * 4
    cb = (centres[:, np.arange(k) % kbar, :] + r.normal(size=(m, k, dsub)) * 0.7).astype(np.float32)
    cbar = np.stack([np.stack([cb[j, l::kbar].astype(np.float64).mean(0) for l in range(kbar)]) for j in range(m)])
    if distinct:
        pool = r.integers(0, k, (distinct, m))
        codes = pool[r.integers(0, distinct, n)].astype(np.uint16)
    else:
        codes = r.integers(0, k, (n, m)).astype(np.uint16)
    queries = (r.normal(size=(nq, m * dsub)) * 4).astype(np.float32)
    return cb, cbar.astype(np.float32), codes, queries


def run_case(ctx, cb, cbar, codes, queries, r2, topk):
    n, nq = len(codes), len(queries)
    d_cbar, d_cb, d_q = dev(cbar), dev(cb), dev(queries)
    d_codes = dev(codes.view(np.int16)) if n else torch.empty((0, 4), dtype=torch.int16, device="cuda")
    # oracle from the GPU's compact tables
    dluts = ctx.pq_build_luts(d_q, d_cbar)
    torch.cuda.synchronize()
    dluts = dluts.cpu().numpy()
    np.testing.assert_allclose(dluts, orc.build_luts(queries, cbar), rtol=1e-5, atol=1e-30)
    qmax = dq.derived_qmax(codes, dluts, r2)
    qluts, _, _ = orc.quantize_luts(dluts, qmax)
    od, oi, s_star, cands = dq.search_from_tables(codes, qluts, cb, queries, r2, topk)
    cap = max([len(c) for c in cands] + [1])
    gd, gi, bucket, ncand, cand = ctx.pq_derived_search(d_codes, d_cbar, d_cb, d_q, r2, topk, cand_cap=cap)
    torch.cuda.synchronize()
    gd, gi, bucket, ncand, cand = (t.cpu().numpy() for t in (gd, gi, bucket, ncand, cand))
    for q in range(nq):
        assert ncand[q] == len(cands[q]), f"query {q}: candidate count"
        if n:
            assert bucket[q] == s_star[q], f"query {q}: bucket"
        got = np.sort(cand[q][:ncand[q]])
        assert np.array_equal(got, cands[q]), f"query {q}: candidate set"
        assert np.all(cand[q][ncand[q]:] == -1)
        check_float_topk_ranked(gd[q], gi[q], od[q], oi[q])
    return ncand


def test_derived_search_several_tiles_ragged_tail_two_query_groups(ctx):
    cb, cbar, codes, queries = make_problem(3, 50_003, 1024, 8, 13)
    ncand = run_case(ctx, cb, cbar, codes, queries, 500, 10)
    assert ncand.min() >= 500
    # the same context again with a smaller problem (workspace kept, counters reset)
    run_case(ctx, cb, cbar, codes[:4097], queries[:3], 64, 5)


def test_derived_search_short_subvectors_direct_tables_kernel(ctx):
    cb, cbar, codes, queries = make_problem(5, 20_000, 512, 4, 9)
    run_case(ctx, cb, cbar, codes, queries, 300, 20)


@pytest.mark.parametrize("n,r2,topk", [(300, 1000, 10), (5000, 1, 1), (129, 129, 128), (2048, 2048, 7), (1, 5, 3)])
def test_derived_search_edges(ctx, n, r2, topk):
    cb, cbar, codes, queries = make_problem(7 + n, n, 768, 8, 4)
    run_case(ctx, cb, cbar, codes, queries, r2, topk)


def test_derived_search_empty_database(ctx):
    cb, cbar, codes, queries = make_problem(9, 0, 256, 8, 3)
    gd, gi, bucket, ncand, _ = ctx.pq_derived_search(torch.empty((0, 4), dtype=torch.int16, device="cuda"), dev(cbar),
                                                     dev(cb), dev(queries), 10, 4)
    torch.cuda.synchronize()
    assert torch.isinf(gd).all() and (gi == -1).all() and (ncand == 0).all()


def test_derived_search_huge_buckets_of_identical_codes(ctx):
    """40 distinct codes only: the bucket of the r2-th vector holds thousands of vectors, all of
    them candidates; precise distances tie massively and ids decide."""
    cb, cbar, codes, queries = make_problem(11, 60_000, 1024, 8, 10, distinct=40)
    ncand = run_case(ctx, cb, cbar, codes, queries, 700, 50)
    assert ncand.max() > 1400


def test_derived_search_full_size_codebooks(ctx):
    """k = 65536 centroids of 32 dimensions per sub-quantizer (d = 128), as in Section 6.3."""
    cb, cbar, codes, queries = make_problem(13, 200_000, 65536, 32, 16)
    run_case(ctx, cb, cbar, codes, queries, 2000, 100)


def test_derived_search_descending_order_worst_case_for_the_bound(ctx):
    """Codes ordered from far to near for query 0: every vector passes the bound of its time."""
    cb, cbar, codes, queries = make_problem(15, 40_000, 1024, 8, 2)
    dl = orc.build_luts(queries[:1], cbar)[0]
    low = (codes & 255).astype(np.int64)
    dist = sum(dl[j][low[:, j]].astype(np.float64) for j in range(4))
    codes = codes[np.argsort(-dist, kind="stable")]
    run_case(ctx, cb, cbar, codes, queries, 400, 10)


def test_derived_search_errors(ctx):
    cb, cbar, codes, queries = make_problem(17, 3000, 256, 8, 2)
    args = (dev(codes.view(np.int16)), dev(cbar), dev(cb), dev(queries))
    with pytest.raises(binding.PqError) as e:
        ctx.pq_derived_search(*args, 500, 10, cand_cap=100)     # every query has at least 500 candidates
    assert e.value.code == -2
    with pytest.raises(binding.PqError) as e:
        ctx.pq_derived_search(*args, 500, 200)                  # topk above 128
    assert e.value.code == -3
    with pytest.raises(binding.PqError) as e:
        ctx.pq_derived_search(*args, 0, 10)                     # r2 < 1
    assert e.value.code == -1
    z = lambda *s, dt=torch.float32: torch.zeros(s, dtype=dt, device="cuda")
    with pytest.raises(binding.PqError) as e:                   # m = 8 is outside the covered shapes
        ctx.pq_derived_search(z(10, 8, dt=torch.int16), z(8, 256, 4), z(8, 256, 4), z(1, 32), 5, 2)
    assert e.value.code == -3
    # the context still works after the errors
    run_case(ctx, cb, cbar, codes, queries, 100, 10)


def test_derived_search_bench_configuration_sampled(ctx):
    """The workload bench.py --derived times (25 M codes, 1000 queries, k = 65536, r2 = 10000, top-100):
    bucket, candidate count, candidate set and result of three sampled queries against the oracle."""
    from paper_1712_02912_amd import datagen
    mix = datagen.sift_like()
    n, nq, r2, topk = 25_000_000, 1000, 10000, 100
    cb, cbar = datagen.clustered_codebooks(mix, 4, 65536)
    queries = mix.sample(nq, datagen.SEED_QUERIES)
    gen = torch.Generator(device="cuda").manual_seed(datagen.SEED_CODES + 5)
    d_codes = torch.randint(-32768, 32768, (n, 4), dtype=torch.int16, device="cuda", generator=gen)
    d_cbar, d_cb, d_q = dev(cbar), dev(cb), dev(queries)
    cap = 40000
    gd, gi, bucket, ncand, cand = ctx.pq_derived_search(d_codes, d_cbar, d_cb, d_q, r2, topk, cand_cap=cap)
    dluts = ctx.pq_build_luts(d_q, d_cbar)
    torch.cuda.synchronize()
    codes = d_codes.cpu().numpy().view(np.uint16)
    dluts = dluts.cpu().numpy()
    sample = [0, 499, 999]
    qmax = dq.derived_qmax(codes, dluts[sample], r2)
    qluts, _, _ = orc.quantize_luts(dluts[sample], qmax)
    od, oi, s_star, cands = dq.search_from_tables(codes, qluts, cb, queries[sample], r2, topk)
    gd, gi, bucket, ncand = gd.cpu().numpy(), gi.cpu().numpy(), bucket.cpu().numpy(), ncand.cpu().numpy()
    assert ncand.min() >= r2 and ncand.max() <= cap
    for i, q in enumerate(sample):
        assert bucket[q] == s_star[i] and ncand[q] == len(cands[i])
        assert np.array_equal(np.sort(cand[q, :ncand[q]].cpu().numpy()), cands[i])
        check_float_topk_ranked(gd[q], gi[q], od[i], oi[i])


# ------------------------------------------------------------ 640 queries and more: 16 queries per pass over the codes
# (the last case has more queries than the 1024 that the offsets of the candidate lists are summed over at a time)
@pytest.mark.parametrize("n,nq,r2,topk", [(30_003, 650, 300, 10), (8_193, 641, 2000, 50), (300, 640, 1000, 5),
                                          (70_001, 777, 64, 128), (4_001, 2_301, 150, 5)])
def test_derived_search_many_queries(ctx, n, nq, r2, topk):
    cb, cbar, codes, queries = make_problem(21 + n, n, 1024, 8, nq)
    run_case(ctx, cb, cbar, codes, queries, r2, topk)


def test_derived_search_many_queries_identical_codes_and_worst_case_order(ctx, opts):
    # 40 distinct codes: buckets of thousands of vectors, all candidates
    cb, cbar, codes, queries = make_problem(23, 40_000, 1024, 8, 643, distinct=40)
    ncand = run_case(ctx, cb, cbar, codes, queries, 700, 20)
    assert ncand.max() > 1400
    # far to near for query 0: every vector passes the bound of its time
    cb, cbar, codes, queries = make_problem(25, 40_000, 1024, 8, 640)
    dl = orc.build_luts(queries[:1], cbar)[0]
    low = (codes & 255).astype(np.int64)
    dist = sum(dl[j][low[:, j]].astype(np.float64) for j in range(4))
    codes = codes[np.argsort(-dist, kind="stable")]
    run_case(ctx, cb, cbar, codes, queries, 400, 10)
    # the 8-query kernel for the same input (switch)
    opts.set("scan_q8", 0)
    run_case(ctx, cb, cbar, codes, queries, 400, 10)
