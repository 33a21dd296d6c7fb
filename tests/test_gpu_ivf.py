"""IVFADC search (Index + Tables + Scan with an inverted index) against the oracle."""
import numpy as np
import pytest
import torch

from oracle import pq_oracle as orc
from paper_1712_02912_amd import binding, datagen
from util import RTOL, check_float_topk_ranked

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    c = binding.Context(0)
    yield c
    torch.cuda.synchronize()
    c.close()


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def check_probes(queries, coarse, gpu_probes, nprobe):
    """Probed lists equal the oracle's up to ties of the coarse distances inside 1e-6 relative."""
    ref, ref_d = orc.ivf_probe(queries, coarse, nprobe)
    c64 = coarse.astype(np.float64)
    cd = np.stack([((q.astype(np.float64)[None, :] - c64) ** 2).sum(-1) for q in queries])
    for q in range(len(queries)):
        if np.array_equal(gpu_probes[q], ref[q]):
            continue
        assert len(set(gpu_probes[q].tolist())) == nprobe
        tau = cd[q][ref[q][-1]]
        assert np.all(cd[q][gpu_probes[q]] <= tau * (1 + 1e-6))
        np.testing.assert_allclose(cd[q][gpu_probes[q]], cd[q][ref[q]], rtol=1e-6)


def run_ivf(ctx, queries, coarse, offsets, codes, ids, cb, nprobe, topk):
    d, i, p = ctx.ivf_adc_search(dev(coarse), dev(offsets), dev(codes), None if ids is None else dev(ids), dev(cb),
                                 binding.CODES_U8, dev(queries), nprobe, topk, return_probes=True)
    torch.cuda.synchronize()
    gd, gi, gp = d.cpu().numpy(), i.cpu().numpy(), p.cpu().numpy()
    check_probes(queries, coarse, gp, nprobe)
    # the scan is compared on the lists the GPU probed, so that a coarse tie cannot move the result
    od, oi = orc.ivf_scan(queries, coarse, offsets, codes, ids, cb, orc.CODES_U8, gp, topk)
    for q in range(len(queries)):
        check_float_topk_ranked(gd[q], gi[q], od[q], oi[q])
    return gd, gi


def make_index(n, d, m, nlist, seed, ntrain=4000, encoded=True):
    mix = datagen.Mixture(d, 16, (0.0, 128.0), (8.0, 32.0), (0.0, 255.0), seed=seed)
    base = mix.sample(n, seed + 1)
    coarse = orc.kmeans(base[:ntrain], nlist, 3, np.arange(nlist, dtype=np.int64) * (ntrain // nlist))
    assign = ((base[:, None, :].astype(np.float32) - coarse[None]) ** 2).sum(-1).argmin(1)
    resid = base - coarse[assign]
    cb = orc.pq_train(resid[:ntrain], m, 256, 3, datagen.kmeans_init_idx(ntrain, m, 256, seed + 2))
    order = np.argsort(assign, kind="stable")
    codes = orc.pq_encode(resid[order], cb)
    offsets = datagen.offsets_from_sizes(np.bincount(assign, minlength=nlist))
    return mix, coarse, cb, codes, order.astype(np.int64), offsets


@pytest.mark.parametrize("m", [8, 16])
def test_ivf_encoded_small(ctx, m):
    mix, coarse, cb, codes, order, offsets = make_index(20000, 64, m, 40, seed=21 + m)
    queries = mix.sample(13, 99)
    for nprobe, topk in ((1, 10), (8, 100), (40, 128), (5, 1)):
        run_ivf(ctx, queries, coarse, offsets, codes, order, cb, nprobe, topk)
    run_ivf(ctx, queries, coarse, offsets, codes, None, cb, 8, 50)


def test_ivf_all_lists_equals_flat_scan_of_residual_tables(ctx):
    """nprobe = nlist: every code is scanned once with the tables of its own list."""
    mix, coarse, cb, codes, order, offsets = make_index(8000, 64, 8, 16, seed=31)
    queries = mix.sample(6, 98)
    gd, gi = run_ivf(ctx, queries, coarse, offsets, codes, None, cb, 16, 20)
    # brute force straight from the definition: || (y - centroid_l(n)) - decode(code_n) ||^2
    list_of = np.repeat(np.arange(16), np.diff(offsets))
    decoded = np.concatenate([cb[j][codes[:, j]] for j in range(8)], axis=1).astype(np.float64)
    for q in range(len(queries)):
        r = (queries[q][None, :] - coarse[list_of]).astype(np.float64)
        dd = ((r - decoded) ** 2).sum(1)
        np.testing.assert_allclose(gd[q], np.sort(dd)[:20], rtol=1e-5)


@pytest.mark.parametrize("prune", [0, 1])
def test_ivf_skewed_lists_many_chunks_and_empty_lists(ctx, opts, prune):
    """Zipf-like list sizes with one list long enough to be cut into chunks, odd list boundaries, empty lists."""
    opts.set("ivf_prune", prune)
    r = np.random.default_rng(41)
    d, m, nlist = 32, 8, 24
    sizes = np.array([700_001, 90_003, 7, 0, 1, 33_333, 0, 129, 128, 127] + [1000 + 37 * i for i in range(14)])
    offsets = datagen.offsets_from_sizes(sizes)
    n = int(offsets[-1])
    codes = r.integers(0, 256, (n, m), dtype=np.uint8)
    coarse = (r.random((nlist, d)) * 100).astype(np.float32)
    cb = (r.random((m, 256, d // m)) * 30).astype(np.float32)
    queries = (r.random((9, d)) * 100).astype(np.float32)
    ids = r.permutation(n).astype(np.int64)
    run_ivf(ctx, queries, coarse, offsets, codes, ids, cb, 24, 100)
    run_ivf(ctx, queries, coarse, offsets, codes, None, cb, 6, 17)


def test_ivf_fewer_codes_than_topk(ctx):
    r = np.random.default_rng(43)
    d, m, nlist = 16, 8, 4
    offsets = datagen.offsets_from_sizes(np.array([3, 0, 2, 1]))
    codes = r.integers(0, 256, (6, m), dtype=np.uint8)
    coarse = r.random((nlist, d)).astype(np.float32)
    cb = r.random((m, 256, d // m)).astype(np.float32)
    queries = r.random((3, d)).astype(np.float32)
    gd, gi = run_ivf(ctx, queries, coarse, offsets, codes, None, cb, 4, 10)
    assert np.all(gi[:, 6:] == -1) and np.all(np.isinf(gd[:, 6:]))


def test_ivf_errors(ctx):
    z = lambda *s, dt=torch.float32: torch.zeros(s, dtype=dt, device="cuda")
    with pytest.raises(binding.PqError) as e:
        ctx.ivf_adc_search(z(4, 16), z(5, dt=torch.int64), z(6, 8, dt=torch.uint8), None, z(8, 256, 2), binding.CODES_U8,
                           z(1, 16), 5, 3)
    assert e.value.code == -2      # nprobe > nlist
    with pytest.raises(binding.PqError) as e:
        ctx.ivf_adc_search(z(4, 16), z(5, dt=torch.int64), z(6, 4, dt=torch.uint8), None, z(4, 256, 4), binding.CODES_U8,
                           z(1, 16), 2, 3)
    assert e.value.code == -3      # m = 4 is outside the covered shapes


def test_ivf_many_lists_probe_selection(ctx):
    """16 384 lists (the probe selection's sampled-threshold path), random codes, Zipf-like list sizes."""
    r = np.random.default_rng(61)
    d, m, nlist, n = 32, 8, 16384, 300_000
    sizes = datagen.zipf_list_sizes(n, nlist)
    offsets = datagen.offsets_from_sizes(sizes)
    codes = r.integers(0, 256, (n, m), dtype=np.uint8)
    coarse = (r.random((nlist, d)) * 100).astype(np.float32)
    cb = (r.random((m, 256, d // m)) * 20 - 10).astype(np.float32)
    queries = (r.random((40, d)) * 100).astype(np.float32)
    queries[3] = coarse[77]                      # a query on top of a centroid
    coarse[200:232] = coarse[100:132]            # duplicate centroids: exact ties of coarse distances
    for nprobe, topk in ((1, 10), (16, 100), (64, 128)):
        run_ivf(ctx, queries, coarse, offsets, codes, None, cb, nprobe, topk)



def test_ivf_queries_served_in_several_batches(ctx, opts):
    """A 1 GiB workspace holds about 600 queries of this shape: 1500 queries take three batches."""
    opts.set("ivf_ws_gib", 1)
    r = np.random.default_rng(67)
    d, m, nlist, n, nq = 32, 8, 16384, 200_000, 1500
    sizes = datagen.zipf_list_sizes(n, nlist)
    offsets = datagen.offsets_from_sizes(sizes)
    codes = r.integers(0, 256, (n, m), dtype=np.uint8)
    coarse = (r.random((nlist, d)) * 100).astype(np.float32)
    cb = (r.random((m, 256, d // m)) * 20 - 10).astype(np.float32)
    queries = (r.random((nq, d)) * 100).astype(np.float32)
    run_ivf(ctx, queries, coarse, offsets, codes, None, cb, 64, 20)


@pytest.mark.parametrize("env", [{"ivf_block_waves": 16}, {"ivf_prune": 1}, {"ivf_prune": 0},
                                 {"ivf_prune": 1, "ivf_short_max": 0}, {"ivf_prune": 0, "ivf_short_max": 0},
                                 {"ivf_prune": 1, "ivf_block_waves": 16}])
@pytest.mark.parametrize("m", [8, 16])
def test_ivf_switches_lower_bound_loop_and_block_shape(ctx, opts, env, m):
    """The inverted-list scan on 16-bit lower bounds (8 pairs per item) and in blocks of 16 waves."""
    for k, v in env.items():
        opts.set(k, v)
    mix, coarse, cb, codes, order, offsets = make_index(20000, 64, m, 40, seed=71 + m)
    queries = mix.sample(11, 97)
    run_ivf(ctx, queries, coarse, offsets, codes, order, cb, 8, 100)
    run_ivf(ctx, queries, coarse, offsets, codes, None, cb, 40, 7)


@pytest.mark.parametrize("prune", [0, 1])
def test_ivf_pairs_that_cannot_contribute_and_unseeded_queries(ctx, opts, prune):
    """Far lists whose table minima already exceed the query's first bound (nothing of them may enter the
    result), and a query whose nearest lists hold fewer than topk codes (no first bound, no pruning)."""
    opts.set("ivf_prune", prune)
    r = np.random.default_rng(73)
    d, m, nlist = 32, 8, 12
    sizes = np.array([5000, 4000, 3, 2, 6000, 2500, 1, 0, 3000, 3500, 2000, 4500])
    offsets = datagen.offsets_from_sizes(sizes)
    n = int(offsets[-1])
    codes = r.integers(0, 256, (n, m), dtype=np.uint8)
    coarse = (r.random((nlist, d)) * 10).astype(np.float32)
    coarse[4:] += 400.0                               # a far group of lists: residuals there are huge
    cb = (r.random((m, 256, d // m)) * 4 - 2).astype(np.float32)
    queries = (r.random((7, d)) * 10).astype(np.float32)
    queries[5] = coarse[2] + 0.01                     # nearest lists are the tiny ones
    queries[6] = coarse[6] + 0.01
    for nprobe, topk in ((12, 100), (6, 10), (3, 128)):
        run_ivf(ctx, queries, coarse, offsets, codes, None, cb, nprobe, topk)


@pytest.mark.parametrize("m", [8, 16])
def test_ivf_lists_beyond_4_gib_of_codes(ctx, m):
    """Lists whose codes start more than 2^32 bytes into the code array (row 2^29 with 8-byte codes, 2^28 with
    16-byte codes): byte offsets of list chunks are 64-bit.  One huge list with a far centroid fills the front
    of the array and is never probed; the probed lists lie behind it.  The oracle runs on those lists alone,
    with the rows of the full array as ids."""
    r = np.random.default_rng(83 + m)
    d, nlist, nq = 32, 40, 12
    filler = (1 << 32) // m + 12_345                       # rows of list 0
    sizes = np.array([filler] + [3000 + 211 * i for i in range(nlist - 1)])
    sizes[7] = 0
    sizes[11] = 150_001                                    # a list cut into chunks
    offsets = datagen.offsets_from_sizes(sizes)
    n = int(offsets[-1])
    gen = torch.Generator(device="cuda").manual_seed(830 + m)
    codes_d = torch.randint(0, 256, (n, m), dtype=torch.uint8, device="cuda", generator=gen)
    tail = codes_d[filler:].cpu().numpy()                  # the probed lists' codes
    coarse = (r.random((nlist, d)) * 100).astype(np.float32)
    coarse[0] += 10_000.0                                  # never among the nearest lists
    cb = (r.random((m, 256, d // m)) * 20 - 10).astype(np.float32)
    queries = (r.random((nq, d)) * 100).astype(np.float32)
    for nprobe, topk in ((8, 100), (39, 20)):
        gd, gi, gp = ctx.ivf_adc_search(dev(coarse), dev(offsets), codes_d, None, dev(cb), binding.CODES_U8, dev(queries),
                                        nprobe, topk, return_probes=True)
        torch.cuda.synchronize()
        gd, gi, gp = gd.cpu().numpy(), gi.cpu().numpy(), gp.cpu().numpy()
        assert np.all(gp > 0), "the filler list must not be probed"
        check_probes(queries, coarse, gp, nprobe)
        assert gi.min() >= filler
        od, oi = orc.ivf_scan(queries, coarse[1:], offsets[1:] - filler, tail, np.arange(filler, n, dtype=np.int64), cb,
                              orc.CODES_U8, gp - 1, topk)
        for q in range(nq):
            check_float_topk_ranked(gd[q], gi[q], od[q], oi[q])
    del codes_d
    torch.cuda.empty_cache()


def test_full_size_config4_sampled(ctx):
    """Config 4 as bench.py runs it: 10^9 uniform random 8-byte codes in 65 536 Zipf-sized lists (made on the GPU by
    the input generator), 10 000 queries in one call, nprobe 64, top-100.  Complete results of a sample of the queries
    against the oracle, which scans the lists the GPU probed (their codes are copied back; rows of the full array
    serve as ids); the probes themselves are checked for those queries as well."""
    nt, nlist, nq, nprobe, topk = 1_000_000_000, 65536, 10000, 64, 100
    mix = datagen.sift_like()
    coarse = mix.sample(nlist, datagen.SEED_DATA + 7)
    sizes = datagen.zipf_list_sizes(nt, nlist)
    offsets = datagen.offsets_from_sizes(sizes)
    codes_d = datagen.random_codes_device(nt, 8, datagen.SEED_CODES + 3)
    cb = datagen.sampled_codebooks(mix, 8, 256) * np.float32(0.25)
    queries = mix.sample(nq, datagen.SEED_QUERIES + 1)
    gd, gi, gp = ctx.ivf_adc_search(dev(coarse), dev(offsets), codes_d, None, dev(cb), binding.CODES_U8, dev(queries),
                                    nprobe, topk, return_probes=True)
    torch.cuda.synchronize()
    gd, gi, gp = gd.cpu().numpy(), gi.cpu().numpy(), gp.cpu().numpy()
    # the query that probes the longest list is part of the sample (its list is cut into the most chunks)
    longest = int(np.argmax(sizes))
    hits = np.flatnonzero((gp == longest).any(axis=1))
    sample = sorted(set([0, 1, 777, 4096, 5000, 9998, 9999] + hits[:2].tolist()))
    check_probes(queries[sample], coarse, gp[sample], nprobe)
    lists = np.unique(gp[sample])
    sub_sizes = sizes[lists].astype(np.int64)
    sub_off = datagen.offsets_from_sizes(sub_sizes)
    sub_codes = np.empty((int(sub_off[-1]), 8), np.uint8)
    sub_ids = np.empty(int(sub_off[-1]), np.int64)
    for j, l in enumerate(lists):
        a, b = int(offsets[l]), int(offsets[l + 1])
        sub_codes[sub_off[j]:sub_off[j + 1]] = codes_d[a:b].cpu().numpy()
        sub_ids[sub_off[j]:sub_off[j + 1]] = np.arange(a, b)
    remap = np.searchsorted(lists, gp[sample]).astype(np.int32)
    od, oi = orc.ivf_scan(queries[sample], coarse[lists], sub_off, sub_codes, sub_ids, cb, orc.CODES_U8, remap, topk)
    for r, q in enumerate(sample):
        check_float_topk_ranked(gd[q], gi[q], od[r], oi[r])
    # every query: ascending, rows valid and distinct, each result row inside one of the probed lists
    assert np.all(np.diff(gd, axis=1) >= 0) and gi.min() >= 0 and gi.max() < nt
    for q in range(0, nq, 97):
        assert len(set(gi[q].tolist())) == topk
        owner = np.searchsorted(offsets, gi[q], side="right") - 1
        assert np.isin(owner, gp[q]).all()
    del codes_d
    torch.cuda.empty_cache()


# ------------------------------------------------------------ Index step through approximate distances
# Calls of 512 and more tiles of 128 queries x 128 lists rank the lists by fp32 matrix-core distances first and
# measure nprobe + 16 of them exactly; the probed lists must be the oracle's all the same.
def _many_lists_problem(seed, nlist, nq, d, m=8, per_list=3):
    r = np.random.default_rng(seed)
    coarse = (r.random((nlist, d)) * 200 - 100).astype(np.float32)
    offsets = datagen.offsets_from_sizes(np.full(nlist, per_list))
    codes = r.integers(0, 256, (nlist * per_list, m), dtype=np.uint8)
    cb = (r.random((m, 256, d // m)) * 20).astype(np.float32)
    queries = (r.random((nq, d)) * 200 - 100).astype(np.float32)
    return coarse, offsets, codes, cb, queries


def _probes_only(ctx, coarse, offsets, codes, cb, queries, nprobe):
    _, _, p = ctx.ivf_adc_search(dev(coarse), dev(offsets), dev(codes), None, dev(cb), binding.CODES_U8, dev(queries), nprobe, 5,
                                 return_probes=True)
    torch.cuda.synchronize()
    return p.cpu().numpy()


# (with lists and queries enough nothing like a matrix is written: a sample of the lists gives every query a bound, and only
# the distances at or below it leave the kernel)
# (the last two cases have lists and queries enough for the form that writes no matrix; the last one with a ragged last
# tile of lists and sub-vectors that end inside a chunk of 32 dimensions)
@pytest.mark.parametrize("nlist,nq,d,nprobe", [(4096, 2100, 64, 16), (8192, 1100, 32, 64), (5000, 1700, 128, 3), (32768, 4100, 32, 20),
                                               (20000, 6700, 48, 10)])
def test_ivf_index_step_through_approximate_distances(ctx, opts, nlist, nq, d, nprobe):
    coarse, offsets, codes, cb, queries = _many_lists_problem(nlist + nq, nlist, nq, d)
    gp = _probes_only(ctx, coarse, offsets, codes, cb, queries, nprobe)
    ref, _ = orc.ivf_probe(queries, coarse, nprobe)
    assert np.array_equal(gp, ref)
    opts.set("ivf_coarse_f16", 0)   # the pass over all lists on the fp32 matrix cores instead of split fp16 operands
    assert np.array_equal(_probes_only(ctx, coarse, offsets, codes, cb, queries, nprobe), ref)
    opts.set("ivf_coarse_f32", 0)   # the exact Tables step for the Index step gives the same lists
    assert np.array_equal(_probes_only(ctx, coarse, offsets, codes, cb, queries, nprobe), ref)


def test_ivf_index_step_wide_dynamic_range(ctx):
    """Coordinates whose scales differ by factors of e^3 per dimension (a few dimensions carry nearly all of the norms, so
    the halves of the split operands lose most of the small ones' bits): the probed lists are still the oracle's."""
    nlist, nq, d, nprobe = 40000, 3400, 96, 100
    r = np.random.default_rng(103)
    spread = np.exp(r.standard_normal((1, d)) * 3)
    coarse = (r.standard_normal((nlist, d)) * spread).astype(np.float32)
    queries = (r.standard_normal((nq, d)) * spread).astype(np.float32)
    offsets = datagen.offsets_from_sizes(np.full(nlist, 2))
    codes = r.integers(0, 256, (nlist * 2, 8), dtype=np.uint8)
    cb = (r.random((8, 256, d // 8)) * 20).astype(np.float32)
    gp = _probes_only(ctx, coarse, offsets, codes, cb, queries, nprobe)
    ref, _ = orc.ivf_probe(queries, coarse, nprobe)
    assert np.array_equal(gp, ref)


@pytest.mark.parametrize("scale", [2.0 ** 50, 2.0 ** -50, 0.0])
def test_ivf_index_step_magnitudes_outside_the_split_operands(ctx, scale):
    """The split fp16 operands serve magnitudes of 2^-40 .. 2^40: beyond them (and for all-zero queries) the pass over all
    lists keeps nothing or its proof fails, and every query takes its exact row; the probed lists are the oracle's."""
    nlist, nq, d, nprobe = 32768, 1030, 32, 20
    coarse, offsets, codes, cb, queries = _many_lists_problem(5, nlist, nq, d)
    if scale == 0.0:
        queries = np.zeros_like(queries)
    else:
        coarse = (coarse * np.float32(scale)).astype(np.float32)
        queries = (queries * np.float32(scale)).astype(np.float32)
    gp = _probes_only(ctx, coarse, offsets, codes, cb, queries, nprobe)
    ref, _ = orc.ivf_probe(queries, coarse, nprobe)
    assert np.array_equal(gp, ref)


@pytest.mark.parametrize("nlist,nq,d", [(4096, 2100, 64), (32768, 4100, 32)])
def test_ivf_index_step_ties_beyond_the_exactly_measured_lists(ctx, nlist, nq, d):
    """100 copies of one centroid are the nearest lists of some queries: more equal distances than the nprobe + 16 lists
    measured exactly, so those queries take the exact rows; ties go by list number, as in the oracle."""
    nprobe = 16
    coarse, offsets, codes, cb, queries = _many_lists_problem(77, nlist, nq, d)
    r = np.random.default_rng(78)
    copies = r.choice(nlist, 100, replace=False)
    coarse[copies] = coarse[copies[0]]
    queries[::7] = coarse[copies[0]] + (r.random((len(queries[::7]), d)) * 2 - 1).astype(np.float32)   # near the copies
    gp = _probes_only(ctx, coarse, offsets, codes, cb, queries, nprobe)
    ref, _ = orc.ivf_probe(queries, coarse, nprobe)
    assert np.array_equal(gp, ref)
    assert np.array_equal(np.sort(ref[0]), np.sort(copies)[:nprobe])   # query 0 probes the copies with the smallest numbers


# ----------------------------------------------------------------------------- Quick ADC inside the inverted index
def make_index_u4(n, d, nlist, seed, ntrain=4000, sizes=None):
    """Packed 4-bit codes (m = 16, k = 16) of residuals, grouped by list; `sizes` replaces the assignment's list
    sizes by given ones (codes then uniformly random: list lengths and boundaries are what such a case is about)."""
    mix = datagen.Mixture(d, 16, (0.0, 128.0), (8.0, 32.0), (0.0, 255.0), seed=seed)
    base = mix.sample(max(n, ntrain), seed + 1)
    coarse = orc.kmeans(base[:ntrain], nlist, 3, np.arange(nlist, dtype=np.int64) * (ntrain // nlist))
    assign = ((base[:, None, :].astype(np.float32) - coarse[None]) ** 2).sum(-1).argmin(1)
    resid = base - coarse[assign]
    cb = orc.pq_train(resid[:ntrain], 16, 16, 3, datagen.kmeans_init_idx(ntrain, 16, 16, seed + 2))
    if sizes is None:
        order = np.argsort(assign[:n], kind="stable")
        packed = orc.pack_u4(orc.pq_encode(resid[:n][order], cb))
        offsets = datagen.offsets_from_sizes(np.bincount(assign[:n], minlength=nlist))
        return mix, coarse, cb, packed, order.astype(np.int64), offsets
    offsets = datagen.offsets_from_sizes(np.asarray(sizes))
    packed = np.random.default_rng(seed + 3).integers(0, 256, (int(offsets[-1]), 8), dtype=np.uint8)
    return mix, coarse, cb, packed, None, offsets


def run_ivf_quick(ctx, queries, coarse, offsets, packed, ids, cb, nprobe, init, kprime, topk):
    """Bit-exact: every float sum of the path is formed in double and rounded once on both sides, the rest is integer."""
    d, i, p = ctx.ivf_quick_adc_search(dev(coarse), dev(offsets), dev(packed), None if ids is None else dev(ids), dev(cb),
                                       dev(queries), nprobe, init, kprime, topk, return_probes=True)
    torch.cuda.synchronize()
    gd, gi, gp = d.cpu().numpy(), i.cpu().numpy(), p.cpu().numpy()
    check_probes(queries, coarse, gp, nprobe)
    od, oi = orc.ivf_quick_scan(queries, coarse, offsets, packed, ids, cb, orc.CODES_U4_PACKED, gp, init, kprime, topk)
    assert np.array_equal(gi, oi)
    assert np.array_equal(gd, od)
    return gd, gi


def test_ivf_quick_encoded_small(ctx):
    mix, coarse, cb, packed, order, offsets = make_index_u4(20000, 64, 40, seed=51)
    queries = mix.sample(13, 99)
    for nprobe, init, kprime, topk in ((1, 200, 40, 10), (8, 1000, 128, 100), (40, 4096, 100, 128), (5, 64, 1, 1),
                                       (8, 300, 20, 50)):
        run_ivf_quick(ctx, queries, coarse, offsets, packed, order, cb, nprobe, init, kprime, topk)
    run_ivf_quick(ctx, queries, coarse, offsets, packed, None, cb, 8, 500, 64, 50)


@pytest.mark.parametrize("chunk_rows", [None, 4096, 100_000])
def test_ivf_quick_long_lists_in_chunks_short_and_empty_lists(ctx, opts, chunk_rows):
    """Lists cut into chunks (the longest into 171 with 4096 rows per chunk: their candidates are merged per pair),
    lists shorter than kprime, empty lists, odd list boundaries."""
    if chunk_rows:
        opts.set("ivf_quick_chunk_rows", chunk_rows)
    sizes = [700_001, 90_003, 7, 0, 1, 33_333, 0, 129, 128, 127] + [1000 + 37 * i for i in range(14)]
    mix, coarse, cb, packed, _, offsets = make_index_u4(0, 32, 24, seed=53, sizes=sizes)
    queries = mix.sample(9, 97)
    run_ivf_quick(ctx, queries, coarse, offsets, packed, None, cb, 24, 2000, 128, 100)
    run_ivf_quick(ctx, queries, coarse, offsets, packed, None, cb, 6, 50, 30, 20)


def test_ivf_quick_ties_of_the_integer_sums(ctx):
    """Codes drawn from four distinct codes only: thousands of rows share every sum, the candidates are the smallest
    rows among them; and a first bound from one code (init = 1), which puts most sums into the last bin counted."""
    sizes = [5000, 3000, 40, 9000]
    mix, coarse, cb, packed, _, offsets = make_index_u4(0, 32, 4, seed=57, sizes=sizes)
    r = np.random.default_rng(5)
    few = r.integers(0, 256, (4, 8), dtype=np.uint8)
    packed = few[r.integers(0, 4, len(packed))]
    queries = mix.sample(7, 96)
    run_ivf_quick(ctx, queries, coarse, offsets, packed, None, cb, 4, 1000, 100, 60)
    run_ivf_quick(ctx, queries, coarse, offsets, packed, None, cb, 3, 1, 128, 128)
    mix, coarse, cb, packed, _, offsets = make_index_u4(0, 32, 4, seed=59, sizes=sizes)
    run_ivf_quick(ctx, queries, coarse, offsets, packed, None, cb, 4, 1, 77, 33)


def test_ivf_quick_many_queries_several_groups_per_list(ctx):
    """More than eight queries probe a list: several work items per list chunk."""
    mix, coarse, cb, packed, order, offsets = make_index_u4(30000, 64, 12, seed=61)
    queries = mix.sample(150, 95)
    run_ivf_quick(ctx, queries, coarse, offsets, packed, order, cb, 5, 800, 64, 40)


def test_ivf_quick_queries_served_in_several_batches(ctx, opts):
    """A 1 GiB workspace holds about 5000 queries of this shape: 12 000 queries take three batches."""
    opts.set("ivf_ws_gib", 1)
    r = np.random.default_rng(69)
    d, nlist, n, nq = 32, 16384, 200_000, 12_000
    sizes = datagen.zipf_list_sizes(n, nlist)
    offsets = datagen.offsets_from_sizes(sizes)
    packed = r.integers(0, 256, (n, 8), dtype=np.uint8)
    coarse = (r.random((nlist, d)) * 100).astype(np.float32)
    cb = (r.random((16, 16, d // 16)) * 20 - 10).astype(np.float32)
    queries = (r.random((nq, d)) * 100).astype(np.float32)
    run_ivf_quick(ctx, queries, coarse, offsets, packed, None, cb, 64, 500, 16, 20)


def test_ivf_quick_empty_index_and_fewer_candidates_than_topk(ctx):
    mix, coarse, cb, packed, _, offsets = make_index_u4(0, 32, 6, seed=65, sizes=[3, 0, 2, 1, 0, 40])
    queries = mix.sample(4, 93)
    gd, gi = run_ivf_quick(ctx, queries, coarse, offsets, packed, None, cb, 6, 100, 5, 20)
    assert np.all(gi[:, 11:] == -1) and np.all(np.isinf(gd[:, 11:]))      # 3 + 2 + 1 + min(5, 40) candidates
    empty = np.zeros_like(offsets)
    gd, gi = run_ivf_quick(ctx, queries, coarse, empty, packed[:0], None, cb, 3, 100, 5, 20)
    assert np.all(gi == -1) and np.all(np.isinf(gd))


def test_ivf_quick_rejects_what_is_not_covered(ctx):
    mix, coarse, cb, packed, order, offsets = make_index_u4(3000, 32, 6, seed=63)
    queries = mix.sample(3, 94)
    for kw in (dict(nprobe=7), dict(kprime=129), dict(topk=129), dict(init=4097), dict(init=0)):
        a = dict(nprobe=2, init=100, kprime=10, topk=5)
        a.update(kw)
        with pytest.raises(RuntimeError):
            ctx.ivf_quick_adc_search(dev(coarse), dev(offsets), dev(packed), None, dev(cb), dev(queries), a["nprobe"],
                                     a["init"], a["kprime"], a["topk"])


def test_ivf_quick_full_size_sampled(ctx):
    """The shape of config 4 with Quick ADC: 10^9 uniform random packed 4-bit codes (16 x 4, 8 bytes each) in 65 536
    Zipf-sized lists, 10 000 queries in one call, nprobe 64, init 1024, kprime 128, top-100.  Complete results of a
    sample of the queries against the oracle on the lists the GPU probed (their codes copied back, rows as ids)."""
    nt, nlist, nq, nprobe, init, kprime, topk = 1_000_000_000, 65536, 10000, 64, 1024, 128, 100
    mix = datagen.sift_like()
    coarse = mix.sample(nlist, datagen.SEED_DATA + 7)
    sizes = datagen.zipf_list_sizes(nt, nlist)
    offsets = datagen.offsets_from_sizes(sizes)
    codes_d = datagen.random_codes_device(nt, 8, datagen.SEED_CODES + 5)
    cb = datagen.sampled_codebooks(mix, 16, 16) * np.float32(0.25)
    queries = mix.sample(nq, datagen.SEED_QUERIES + 1)
    gd, gi, gp = ctx.ivf_quick_adc_search(dev(coarse), dev(offsets), codes_d, None, dev(cb), dev(queries), nprobe, init,
                                          kprime, topk, return_probes=True)
    torch.cuda.synchronize()
    gd, gi, gp = gd.cpu().numpy(), gi.cpu().numpy(), gp.cpu().numpy()
    longest = int(np.argmax(sizes))
    hits = np.flatnonzero((gp == longest).any(axis=1))
    sample = sorted(set([0, 1, 777, 4096, 9999] + hits[:1].tolist()))
    check_probes(queries[sample], coarse, gp[sample], nprobe)
    lists = np.unique(gp[sample])
    sub_off = datagen.offsets_from_sizes(sizes[lists].astype(np.int64))
    sub_codes = np.empty((int(sub_off[-1]), 8), np.uint8)
    sub_ids = np.empty(int(sub_off[-1]), np.int64)
    for j, l in enumerate(lists):
        a, b = int(offsets[l]), int(offsets[l + 1])
        sub_codes[sub_off[j]:sub_off[j + 1]] = codes_d[a:b].cpu().numpy()
        sub_ids[sub_off[j]:sub_off[j + 1]] = np.arange(a, b)
    remap = np.searchsorted(lists, gp[sample]).astype(np.int32)
    od, oi = orc.ivf_quick_scan(queries[sample], coarse[lists], sub_off, sub_codes, sub_ids, cb, orc.CODES_U4_PACKED,
                                remap, init, kprime, topk)
    assert np.array_equal(gi[sample], oi) and np.array_equal(gd[sample], od)
    assert np.all(np.diff(gd, axis=1) >= 0) and gi.min() >= 0 and gi.max() < nt
    for q in range(0, nq, 97):
        assert len(set(gi[q].tolist())) == topk
        owner = np.searchsorted(offsets, gi[q], side="right") - 1
        assert np.isin(owner, gp[q]).all()
    del codes_d
    torch.cuda.empty_cache()
