"""Parity of the HIP path (through the C ABI) against the CPU oracle, element by element.

Float distances: 1e-5 relative, top-k sets identical up to ties inside that band.
Integer sums, quantised tables and ids: bit-exact.
"""
import numpy as np
import pytest
import torch

from oracle import pq_oracle as orc
from paper_1712_02912_amd import binding, datagen
from util import RTOL, check_exact_topk, check_float_topk, sift_pq

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    c = binding.Context(0)
    yield c
    torch.cuda.synchronize()
    c.close()


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


# ----------------------------------------------------------------------------- Tables step
@pytest.mark.parametrize("m,k,d,nq", [(8, 256, 128, 16), (16, 16, 128, 37), (16, 256, 960, 21), (4, 7, 20, 3),
                                       (1, 256, 16, 1), (8, 1, 64, 5)])
def test_build_luts(ctx, m, k, d, nq):
    r = np.random.default_rng(m * 1000 + k)
    mix = datagen.sift_like() if d == 128 else None
    queries = mix.sample(nq, 5) if mix else (r.random((nq, d)).astype(np.float32))
    cb = datagen.sampled_codebooks(mix, m, k) if mix else r.random((m, k, d // m)).astype(np.float32)
    ref = orc.build_luts(queries, cb)
    got = host(ctx.pq_build_luts(dev(queries), dev(cb)))
    assert got.shape == ref.shape
    np.testing.assert_allclose(got, ref, rtol=4e-6, atol=1e-30)  # (dsub+1)*2^-24 at dsub=60 is 3.6e-6


def test_build_luts_exact_zero_distance(ctx):
    cb = np.arange(2 * 4 * 3, dtype=np.float32).reshape(2, 4, 3)
    queries = np.concatenate([cb[0, 2], cb[1, 1]])[None, :]
    got = host(ctx.pq_build_luts(dev(queries), dev(cb)))
    assert got[0, 0, 2] == 0.0 and got[0, 1, 1] == 0.0
    assert np.array_equal(got, orc.build_luts(queries, cb))  # small integers: exact in float


# Launches of 512 and more tiles of 128 x 128 entries take a kernel of their own (other tile, other
# block numbering, results written through LDS): ragged tiles on both sides, one and several chunks
# of 16 dimensions, a last chunk of 4 and of 12 dimensions, and rows of a length that rules out
# 16-byte stores.  Sub-vectors of 64 dimensions and more whose rows serve 8 tiles and more are converted to doubles
# by a pass of their own first (cases 3 and 7, the latter with rows padded from 68 to 80 dimensions).
@pytest.mark.parametrize("m,k,d,nq", [(32, 256, 256, 1100), (8, 300, 96, 4500), (1, 5000, 128, 1700), (4, 250, 80, 9000),
                                       (16, 256, 960, 2100), (2, 1100, 56, 8000), (2, 1100, 136, 4000)])
def test_build_luts_many_tiles(ctx, m, k, d, nq):
    r = np.random.default_rng(m * 1000 + k + nq)
    queries = (r.random((nq, d)) * 4 - 1).astype(np.float32)
    cb = (r.random((m, k, d // m)) * 4 - 1).astype(np.float32)
    # some queries lie exactly on centroids of their sub-spaces: these entries must be exact zeros
    ds = d // m
    hits = [(int(q), int(r.integers(0, m)), int(r.integers(0, k))) for q in r.integers(0, nq, 40)]
    for q, j, c in hits:
        queries[q, j * ds:(j + 1) * ds] = cb[j, c]
    ref = orc.build_luts(queries, cb)
    got = host(ctx.pq_build_luts(dev(queries), dev(cb)))
    assert got.shape == ref.shape
    np.testing.assert_allclose(got, ref, rtol=4e-6, atol=1e-30)
    for q, j, c in hits:
        assert got[q, j, c] == 0.0


# ----------------------------------------------------------------------------- quantiser
@pytest.mark.parametrize("m,k", [(16, 16), (8, 256), (3, 5)])
def test_quantize_luts_bit_exact(ctx, m, k):
    r = np.random.default_rng(11)
    nq = 33
    luts = (r.random((nq, m, k)) * 1000 + 3).astype(np.float32)
    qmax = (luts.min(axis=(1, 2)) + r.random(nq) * 2000).astype(np.float32)
    qmax[0] = luts[0].min()          # empty range
    qmax[1] = np.inf
    qmax[2] = luts[2].min() - 1.0    # negative range
    ref_q, ref_min, ref_scale = orc.quantize_luts(luts, qmax)
    q, qmin, scale = ctx.pq_quantize_luts(dev(luts), dev(qmax))
    assert np.array_equal(host(q), ref_q)
    assert np.array_equal(host(qmin), ref_min)
    assert np.array_equal(host(scale), ref_scale)


def test_qmax_prescan(ctx):
    _, queries, cb, codes16 = sift_pq(16, 16, 100000, 16)
    packed = orc.pack_u4(codes16)
    luts = ctx.pq_build_luts(dev(queries), dev(cb))
    luts_h = host(luts)
    for init, kq in ((200, 1), (1000, 1000), (4096, 1000), (3000, 77)):
        got = host(ctx.pq_qmax_prescan(dev(packed), binding.CODES_U4_PACKED, luts, init, kq))
        ref = orc.qmax_prescan(packed, orc.CODES_U4_PACKED, luts_h, init, kq)
        np.testing.assert_allclose(got, ref, rtol=2e-6)


# ----------------------------------------------------------------------------- float scan
def run_float_scan(ctx, codes, fmt, luts_h, topk):
    d, i = ctx.pq_adc_scan_topk(dev(codes) if len(codes) else torch.empty((0, codes.shape[1]), dtype=torch.uint8, device="cuda"),
                                fmt, dev(luts_h), topk)
    gd, gi = host(d), host(i)
    od, oi = orc.adc_scan_topk_f32(codes, fmt, luts_h, topk)
    for q in range(luts_h.shape[0]):
        check_float_topk(gd[q], gi[q], od[q], oi[q], codes, fmt, luts_h[q], len(codes))
    return gd, gi, od, oi


def test_scan_config0_pq8x8(ctx):
    """Config 0: d=128 mixture, 8x8 trained codebooks, N=100k encoded codes, 16 queries, top-100."""
    _, queries, cb, codes = sift_pq(8, 256, 100000, 16)
    luts_h = host(ctx.pq_build_luts(dev(queries), dev(cb)))
    gd, gi, od, oi = run_float_scan(ctx, codes, orc.CODES_U8, luts_h, 100)
    # encoded data holds many identical codes: their distances tie up to the rounding of the float
    # sum, so ids may swap inside the tolerance band, but the distance profile must match rank by rank
    np.testing.assert_allclose(gd, od, rtol=RTOL)


@pytest.mark.parametrize("n", [0, 1, 63, 127, 128, 129, 1023, 1025, 8191, 8193, 50001])
@pytest.mark.parametrize("nq,topk", [(1, 1), (3, 10), (5, 100), (8, 128)])
def test_scan_f32_ragged(ctx, n, nq, topk):
    r = np.random.default_rng(n * 7 + nq)
    codes = r.integers(0, 256, (n, 8), dtype=np.uint8)
    luts_h = (r.random((nq, 8, 256)) * 100).astype(np.float32)
    run_float_scan(ctx, codes, orc.CODES_U8, luts_h, topk)


@pytest.mark.parametrize("topk", [129, 500, 1024])
def test_scan_f32_large_topk(ctx, topk):
    r = np.random.default_rng(topk)
    n = 30011
    codes = r.integers(0, 256, (n, 8), dtype=np.uint8)
    luts_h = (r.random((6, 8, 256)) * 100).astype(np.float32)
    run_float_scan(ctx, codes, orc.CODES_U8, luts_h, topk)


def test_scan_f32_pq16x8(ctx):
    r = np.random.default_rng(3)
    n = 70007
    codes = r.integers(0, 256, (n, 16), dtype=np.uint8)
    luts_h = r.random((7, 16, 256)).astype(np.float32)
    run_float_scan(ctx, codes, orc.CODES_U8, luts_h, 100)


def test_scan_f32_many_chunks_and_groups(ctx):
    """Several chunks per query and several query groups: exercises the shared bounds and the merge."""
    r = np.random.default_rng(4)
    n = 1_000_003
    codes = r.integers(0, 256, (n, 8), dtype=np.uint8)
    luts_h = (r.random((13, 8, 256)) * 10).astype(np.float32)
    run_float_scan(ctx, codes, orc.CODES_U8, luts_h, 100)


def test_scan_f32_all_equal_and_ties(ctx):
    n = 20000
    codes = np.zeros((n, 8), np.uint8)
    luts_h = np.ones((2, 8, 256), np.float32)
    d, i = ctx.pq_adc_scan_topk(dev(codes), binding.CODES_U8, dev(luts_h), 50)
    assert np.array_equal(host(i), np.tile(np.arange(50), (2, 1)))  # equal values: smallest ids
    assert np.all(host(d) == 8.0)
    # few distinct values (exact in float, so ties are exact and the (value, id) order is unique)
    r = np.random.default_rng(5)
    codes = r.integers(0, 256, (n, 8), dtype=np.uint8)
    luts_h = r.integers(0, 3, (3, 8, 256)).astype(np.float32)
    d, i = ctx.pq_adc_scan_topk(dev(codes), binding.CODES_U8, dev(luts_h), 100)
    od, oi = orc.adc_scan_topk_f32(codes, orc.CODES_U8, luts_h, 100)
    assert np.array_equal(host(i), oi) and np.array_equal(host(d), od)


def test_scan_f32_descending_order_worst_case(ctx):
    """Distances strictly decreasing with position: every code beats the current bound."""
    n = 40000
    codes = np.zeros((n, 8), np.uint8)
    idx = np.arange(n)
    codes[:, 0] = idx % 256
    codes[:, 1] = idx // 256
    lut = np.zeros((1, 8, 256), np.float32)
    lut[0, 0] = 255 - np.arange(256)
    lut[0, 1] = (255 - np.arange(256)) * 256.0
    d, i = ctx.pq_adc_scan_topk(dev(codes), binding.CODES_U8, dev(lut), 100)
    od, oi = orc.adc_scan_topk_f32(codes, orc.CODES_U8, lut, 100)
    assert np.array_equal(host(i), oi) and np.array_equal(host(d), od)


@pytest.mark.parametrize("m,k,fmt", [(4, 16, orc.CODES_U8), (32, 16, orc.CODES_U4_PACKED), (2, 256, orc.CODES_U8),
                                     (16, 16, orc.CODES_U4_PACKED)])
def test_scan_f32_general_shapes(ctx, m, k, fmt):
    r = np.random.default_rng(m + k)
    n = 9001
    cb = m // 2 if fmt == orc.CODES_U4_PACKED else m
    hi = 256 if fmt == orc.CODES_U4_PACKED else k
    codes = r.integers(0, hi, (n, cb), dtype=np.uint8)
    luts_h = r.random((3, m, k)).astype(np.float32)
    run_float_scan(ctx, codes, fmt, luts_h, 20)


# ----------------------------------------------------------------------------- integer scan
# ------------------------------------------------------------- 8x8 float scan, pruned path
# Databases of 65536 codes and more take the scan that dismisses codes by 16-bit lower bounds
# before any float work; these cases aim at what is specific to it.
@pytest.mark.parametrize("n", [65535, 65536, 65537, 300_001])
def test_scan_f32_pruned_path_sizes(ctx, n):
    r = np.random.default_rng(n)
    codes = r.integers(0, 256, (n, 8), dtype=np.uint8)
    luts_h = (r.random((11, 8, 256)) * 50 + r.random((11, 8, 1)) * 200).astype(np.float32)
    run_float_scan(ctx, codes, orc.CODES_U8, luts_h, 100)


@pytest.mark.parametrize("topk", [1, 128, 129, 1000])
def test_scan_f32_pruned_topk_range(ctx, topk):
    r = np.random.default_rng(topk + 77)
    codes = r.integers(0, 256, (200_003, 8), dtype=np.uint8)
    luts_h = (r.random((5, 8, 256)) * 100).astype(np.float32)
    run_float_scan(ctx, codes, orc.CODES_U8, luts_h, topk)


def test_scan_f32_pruned_degenerate_tables(ctx):
    r = np.random.default_rng(21)
    n = 70_001
    # (a) every code is the per-table minimiser: the first bound equals the sum of the minima,
    #     which leaves no range for the 16-bit tables (nothing can be pruned)
    luts_h = (r.random((3, 8, 256)) * 10 + 1).astype(np.float32)
    codes = np.tile(luts_h[0].argmin(axis=1).astype(np.uint8), (n, 1))
    run_float_scan(ctx, codes, orc.CODES_U8, luts_h, 100)
    # (b) a large common offset with a tiny spread: too little fp32 resolution for a threshold
    codes = r.integers(0, 256, (n, 8), dtype=np.uint8)
    luts_h = (1.0e7 + r.random((2, 8, 256))).astype(np.float32)
    run_float_scan(ctx, codes, orc.CODES_U8, luts_h, 100)
    # (c) a huge dynamic range: most 16-bit entries clamp at their maximum
    luts_h = np.exp(r.random((4, 8, 256)) * 30 - 10).astype(np.float32)
    run_float_scan(ctx, codes, orc.CODES_U8, luts_h, 100)
    # (d) constant tables: all distances equal, the smallest ids win
    luts_h = np.full((2, 8, 256), 3.0, np.float32)
    d, i = ctx.pq_adc_scan_topk(dev(codes), binding.CODES_U8, dev(luts_h), 100)
    assert np.array_equal(host(i), np.tile(np.arange(100), (2, 1))) and np.all(host(d) == 24.0)
    # (e) few distinct table values: exact float sums, massive exact ties, unique (value, id) order
    luts_h = r.integers(0, 3, (9, 8, 256)).astype(np.float32)
    d, i = ctx.pq_adc_scan_topk(dev(codes), binding.CODES_U8, dev(luts_h), 100)
    od, oi = orc.adc_scan_topk_f32(codes, orc.CODES_U8, luts_h, 100)
    assert np.array_equal(host(i), oi) and np.array_equal(host(d), od)


def test_scan_f32_pruned_descending_order_worst_case(ctx):
    """Distances strictly decreasing with position over 2^17 codes: every code beats the bound."""
    n = 1 << 17
    codes = np.zeros((n, 8), np.uint8)
    idx = np.arange(n)
    codes[:, 0] = idx % 256
    codes[:, 1] = (idx // 256) % 256
    codes[:, 2] = idx // 65536
    lut = np.zeros((1, 8, 256), np.float32)
    lut[0, 0] = 255 - np.arange(256)
    lut[0, 1] = (255 - np.arange(256)) * 256.0
    lut[0, 2] = (255 - np.arange(256)) * 65536.0
    d, i = ctx.pq_adc_scan_topk(dev(codes), binding.CODES_U8, dev(lut), 100)
    od, oi = orc.adc_scan_topk_f32(codes, orc.CODES_U8, lut, 100)
    assert np.array_equal(host(i), oi) and np.array_equal(host(d), od)


@pytest.mark.parametrize("n,nq,topk", [(65536, 3, 100), (200_001, 9, 128), (131_072, 2, 1000)])
def test_scan_f32_pruned_16_tables(ctx, n, nq, topk):
    """16 x 256 float tables on the pruned path: random tables, then tables with exact ties."""
    r = np.random.default_rng(n + topk)
    codes = r.integers(0, 256, (n, 16), dtype=np.uint8)
    luts_h = (r.random((nq, 16, 256)) * 40 + r.random((nq, 16, 1)) * 300).astype(np.float32)
    run_float_scan(ctx, codes, orc.CODES_U8, luts_h, topk)
    luts_h = r.integers(0, 3, (nq, 16, 256)).astype(np.float32)
    d, i = ctx.pq_adc_scan_topk(dev(codes), binding.CODES_U8, dev(luts_h), topk)
    od, oi = orc.adc_scan_topk_f32(codes, orc.CODES_U8, luts_h, topk)
    assert np.array_equal(host(i), oi) and np.array_equal(host(d), od)


def test_scan_f32_pruned_encoded_duplicates(ctx):
    """Encoded mixture data (many identical codes), 37 queries: not a multiple of the group size."""
    _, queries, cb, codes = sift_pq(8, 256, 100000, 16)
    mix = datagen.sift_like()
    q2 = mix.sample(37, datagen.SEED_QUERIES + 5)
    luts_h = host(ctx.pq_build_luts(dev(q2), dev(cb)))
    gd, gi, od, oi = run_float_scan(ctx, codes, orc.CODES_U8, luts_h, 100)
    np.testing.assert_allclose(gd, od, rtol=RTOL)


def run_int_scan(ctx, codes, fmt, qluts_h, topk):
    s, i = ctx.pq_adc_scan_topk(dev(codes), fmt, dev(qluts_h), topk)
    os_, oi = orc.adc_scan_topk_u8(codes, fmt, qluts_h, topk)
    gs, gi = host(s), host(i)
    check_exact_topk(gs, gi, os_, oi)


@pytest.mark.parametrize("n", [1, 127, 129, 4097, 60001])
@pytest.mark.parametrize("nq,topk", [(1, 1), (7, 100), (9, 128), (3, 1000)])
def test_scan_u4_bit_exact(ctx, n, nq, topk):
    r = np.random.default_rng(n + nq)
    packed = r.integers(0, 256, (n, 8), dtype=np.uint8)
    qluts = r.integers(0, 256, (nq, 16, 16), dtype=np.uint8)
    run_int_scan(ctx, packed, orc.CODES_U4_PACKED, qluts, topk)


def test_scan_u4_heavy_ties_and_extremes(ctx):
    r = np.random.default_rng(6)
    n = 200_003
    packed = r.integers(0, 256, (n, 8), dtype=np.uint8)
    qluts = r.integers(0, 4, (10, 16, 16), dtype=np.uint8)      # sums in 0..48: thousands of ties
    qluts[1] = 255                                               # every sum = 4080
    qluts[2] = 0
    run_int_scan(ctx, packed, orc.CODES_U4_PACKED, qluts, 100)
    run_int_scan(ctx, packed, orc.CODES_U4_PACKED, qluts, 1000)


def test_scan_u8_general_shapes(ctx):
    r = np.random.default_rng(8)
    codes = r.integers(0, 256, (5003, 8), dtype=np.uint8)
    qluts = r.integers(0, 256, (4, 8, 256), dtype=np.uint8)
    run_int_scan(ctx, codes, orc.CODES_U8, qluts, 64)
    packed = r.integers(0, 256, (5003, 4), dtype=np.uint8)
    run_int_scan(ctx, packed, orc.CODES_U4_PACKED, r.integers(0, 256, (2, 8, 16), dtype=np.uint8), 10)


# ----------------------------------------------------------------------------- config 2 pipeline
def test_quick_adc_pipeline_config2_small(ctx):
    """16x4 codes: tables -> qmax pre-scan -> 8-bit tables -> integer scan top-1000 -> float rerank top-100.

    Stage-wise parity: each oracle stage is fed the GPU output of the previous stage, so that
    float rounding in the tables cannot move an integer decision.
    """
    _, queries, cb, codes16 = sift_pq(16, 16, 100000, 16)
    packed = orc.pack_u4(codes16)
    fmt = orc.CODES_U4_PACKED
    dpacked = dev(packed)
    luts = ctx.pq_build_luts(dev(queries), dev(cb))
    qmax = ctx.pq_qmax_prescan(dpacked, fmt, luts, 2000, 1000)
    qluts, qmin, scale = ctx.pq_quantize_luts(luts, qmax)
    sums, cand = ctx.pq_adc_scan_topk(dpacked, fmt, qluts, 1000)
    dist, ids = ctx.pq_rerank_f32(dpacked, fmt, luts, cand, 100)
    luts_h, qmax_h, qluts_h, cand_h = host(luts), host(qmax), host(qluts), host(cand)
    np.testing.assert_allclose(luts_h, orc.build_luts(queries, cb), rtol=4e-6)
    ref_q, ref_min, ref_scale = orc.quantize_luts(luts_h, qmax_h)
    assert np.array_equal(qluts_h, ref_q) and np.array_equal(host(qmin), ref_min) and np.array_equal(host(scale), ref_scale)
    os_, oi = orc.adc_scan_topk_u8(packed, fmt, qluts_h, 1000)
    check_exact_topk(host(sums), cand_h, os_, oi)
    od, oid = orc.rerank_f32(packed, fmt, luts_h, cand_h, 100)
    gd, gi = host(dist), host(ids)
    for q in range(len(queries)):
        np.testing.assert_allclose(gd[q], od[q], rtol=RTOL)
        exact = orc.adc_all_f32(packed[gi[q]], fmt, luts_h[q])
        np.testing.assert_allclose(gd[q], exact, rtol=RTOL)
        assert np.all(exact <= od[q][-1] * (1 + RTOL))
    # none of the top-1000 candidates has a clamped table entry (qmax = 1000-th distance of the pre-scan)
    un = np.stack([packed & 15, packed >> 4], axis=2).reshape(len(packed), 16)
    for q in range(len(queries)):
        assert np.all(qluts_h[q][np.arange(16)[None, :], un[cand_h[q, :100]]] < 255)


def test_rerank_matches_oracle(ctx):
    r = np.random.default_rng(10)
    n = 5000
    codes = r.integers(0, 256, (n, 8), dtype=np.uint8)
    luts_h = r.random((4, 8, 256)).astype(np.float32)
    cand = np.stack([r.choice(n, 300, replace=False) for _ in range(4)]).astype(np.int64)
    cand[2, 5:9] = -1
    d, i = ctx.pq_rerank_f32(dev(codes), binding.CODES_U8, dev(luts_h), dev(cand), 40)
    od, oi = orc.rerank_f32(codes, orc.CODES_U8, luts_h, cand, 40)
    assert np.array_equal(host(i), oi)
    np.testing.assert_allclose(host(d), od, rtol=RTOL)


# ----------------------------------------------------------------------------- error handling
def test_errors_are_reported_not_raised_in_kernels(ctx):
    codes = torch.zeros((10, 8), dtype=torch.uint8, device="cuda")
    luts = torch.zeros((1, 8, 256), dtype=torch.float32, device="cuda")
    with pytest.raises(binding.PqError) as e:
        ctx.pq_adc_scan_topk(codes, binding.CODES_U8, luts, 0)
    assert e.value.code == -1
    with pytest.raises(binding.PqError) as e:
        ctx.pq_adc_scan_topk(codes, binding.CODES_U8, luts, 5000)
    assert e.value.code == -3
    with pytest.raises(binding.PqError) as e:
        ctx.pq_build_luts(torch.zeros((1, 10), device="cuda"), torch.zeros((3, 4, 3), device="cuda"))
    assert e.value.code == -2
    with pytest.raises(binding.PqError) as e:
        ctx.pq_adc_scan_topk(codes[:, :4].contiguous(), binding.CODES_U4_PACKED, torch.zeros((1, 7, 16), device="cuda"), 5)
    assert e.value.code == -2
    # the context stays usable
    d, i = ctx.pq_adc_scan_topk(codes, binding.CODES_U8, luts, 3)
    assert host(i).tolist() == [[0, 1, 2]]


def test_scan_f32_plain_loop_on_a_large_database(ctx, opts):
    """The plain float loop (no pruning) normally serves small databases only; here it scans a large one."""
    opts.set("scan_prune", 0)
    r = np.random.default_rng(31)
    codes = r.integers(0, 256, (400_003, 8), dtype=np.uint8)
    luts_h = (r.random((9, 8, 256)) * 100).astype(np.float32)
    run_float_scan(ctx, codes, orc.CODES_U8, luts_h, 100)
    run_float_scan(ctx, codes, orc.CODES_U8, luts_h[:2], 700)


def test_switches_general_kernel_and_launch_shapes(ctx, opts):
    """The general kernel on the shapes the tuned kernels normally take, and unusual launch shapes."""
    r = np.random.default_rng(33)
    codes = r.integers(0, 256, (120_001, 8), dtype=np.uint8)
    luts_h = (r.random((6, 8, 256)) * 100).astype(np.float32)
    qluts = r.integers(0, 256, (5, 16, 16), dtype=np.uint8)
    opts.set("scan_force_general", 1)
    run_float_scan(ctx, codes, orc.CODES_U8, luts_h, 100)
    run_int_scan(ctx, codes, orc.CODES_U4_PACKED, qluts, 100)
    opts.set("scan_force_general", None)
    for blocks, items in ((3, 1), (1000, 7), (1, 1)):
        opts.set("scan_blocks", blocks)
        opts.set("scan_items_per_block", items)
        run_float_scan(ctx, codes, orc.CODES_U8, luts_h, 100)
        run_int_scan(ctx, codes, orc.CODES_U4_PACKED, qluts, 1000)


def test_build_luts_without_matrix_cores(ctx, opts):
    opts.set("lut_mfma", 0)
    r = np.random.default_rng(34)
    q = (r.random((19, 128)) * 255).astype(np.float32)
    cb = (r.random((8, 256, 16)) * 255).astype(np.float32)
    np.testing.assert_allclose(host(ctx.pq_build_luts(dev(q), dev(cb))), orc.build_luts(q, cb), rtol=4e-6, atol=0)


# ----------------------------------------------------------------------------- OPQ rotation
# the last two cases have 512 and more tiles of 128 x 128 outputs and take the kernel for large launches
@pytest.mark.parametrize("n,d", [(1000, 128), (77, 960), (4097, 20), (1, 8), (0, 16), (70001, 128), (9000, 960)])
def test_rotate_matches_oracle(ctx, n, d):
    r = np.random.default_rng(n + d)
    x = (r.random((n, d)) * 255).astype(np.float32)
    Q, _ = np.linalg.qr(r.standard_normal((d, d)))
    R = Q.astype(np.float32)
    got = host(ctx.pq_rotate(dev(x) if n else torch.empty((0, d), device="cuda"), dev(R)))
    ref = orc.rotate(x, R)
    # both sides add in double and round once; the orders differ, so the last float bit may
    np.testing.assert_allclose(got, ref, rtol=2e-7, atol=1e-30 + 2e-7 * np.abs(ref).max() if n else 0)
    if n:
        assert (got == ref).mean() > 0.99
        perm = r.permutation(d)
        P = np.zeros((d, d), np.float32)
        P[np.arange(d), perm] = 1.0
        assert np.array_equal(host(ctx.pq_rotate(dev(x), dev(P))), x[:, perm])


def test_opq_search_equals_search_on_rotated_data(ctx):
    """opq(x) = pq(R x): rotating database and queries, encoding and scanning on the GPU gives the
    oracle's results for the rotated data (rotation, encoder, tables and scan chained)."""
    mix = datagen.sift_like()
    r = np.random.default_rng(91)
    Q, _ = np.linalg.qr(r.standard_normal((128, 128)))
    R = Q.astype(np.float32)
    x = mix.sample(70_000, datagen.SEED_DATA + 5)
    y = mix.sample(9, datagen.SEED_QUERIES + 5)
    xr, yr = ctx.pq_rotate(dev(x), dev(R)), ctx.pq_rotate(dev(y), dev(R))
    cb = orc.rotate(mix.sample(256, 5), R).reshape(256, 8, 16).transpose(1, 0, 2).copy()   # centroids = rotated samples
    codes = ctx.pq_encode(xr, dev(cb))
    luts = ctx.pq_build_luts(yr, dev(cb))
    d, i = ctx.pq_adc_scan_topk(codes, binding.CODES_U8, luts, 100)
    xr_h, yr_h = host(xr), host(yr)
    codes_h = orc.pq_encode(xr_h, cb)
    assert np.array_equal(host(codes), codes_h)
    luts_h = host(luts)
    np.testing.assert_allclose(luts_h, orc.build_luts(yr_h, cb), rtol=4e-6)
    od, oi = orc.adc_scan_topk_f32(codes_h, orc.CODES_U8, luts_h, 100)
    gd, gi = host(d), host(i)
    for q in range(len(y)):
        check_float_topk(gd[q], gi[q], od[q], oi[q], codes_h, orc.CODES_U8, luts_h[q], len(codes_h))


# ----------------------------------------------------------------------------- encoder
@pytest.mark.parametrize("m,k,d,n,fmt", [(8, 256, 128, 100_000, orc.CODES_U8), (16, 16, 128, 33_333, orc.CODES_U4_PACKED),
                                         (16, 256, 960, 5_001, orc.CODES_U8), (4, 7, 20, 1_000, orc.CODES_U8),
                                         (2, 16, 6, 129, orc.CODES_U4_PACKED), (1, 200, 33, 63, orc.CODES_U8)])
def test_encode_bit_exact(ctx, m, k, d, n, fmt):
    """Codes of mixture data against trained-like codebooks equal the oracle's, index for index."""
    mix = datagen.sift_like() if d == 128 else (datagen.gist_like() if d == 960 else None)
    r = np.random.default_rng(m * 1000 + k)
    if mix is not None:
        x = mix.sample(n, datagen.SEED_DATA + 3)
        cb = datagen.sampled_codebooks(mix, m, k)
    else:
        x = (r.random((n, d)) * 10).astype(np.float32)
        cb = (r.random((m, k, d // m)) * 10).astype(np.float32)
    ref = orc.pq_encode(x, cb)
    if fmt == orc.CODES_U4_PACKED:
        ref = orc.pack_u4(ref)
    got = host(ctx.pq_encode(dev(x), dev(cb), fmt))
    assert np.array_equal(got, ref)


def test_encode_ties_and_exact_hits(ctx):
    """Duplicate centroids tie exactly (smallest index wins); vectors that are centroids encode to themselves."""
    r = np.random.default_rng(77)
    cb = (r.random((8, 256, 16)) * 255).astype(np.float32)
    cb[:, 200:] = cb[:, :56]                      # duplicates of centroids 0..55
    pick = r.integers(0, 256, (5000, 8))
    x = np.concatenate([cb[j][pick[:, j]] for j in range(8)], axis=1)
    got = host(ctx.pq_encode(dev(x), dev(cb)))
    assert np.array_equal(got, orc.pq_encode(x, cb))
    assert np.array_equal(got, np.where(pick >= 200, pick - 200, pick).astype(np.uint8))
    assert host(ctx.pq_encode(dev(x[:0]), dev(cb))).shape == (0, 8)


# ----------------------------------------------------------------------------- full size (bench configuration)
FULL_N, FULL_NQ = 25_000_000, 1000
SAMPLE_Q = [0, 1, 7, 8, 123, 500, 640, 777, 998, 999]


def test_full_size_config1_sampled(ctx):
    """Config 1 as bench.py runs it (25 M random codes, 1000 queries, top-100): complete results of a
    sample of the queries against the oracle."""
    mix = datagen.sift_like()
    queries = dev(mix.sample(FULL_NQ, datagen.SEED_QUERIES))
    cb = dev(datagen.sampled_codebooks(mix, 8, 256))
    codes_h = datagen.random_codes(FULL_N, 8)
    luts = ctx.pq_build_luts(queries, cb)
    d, i = ctx.pq_adc_scan_topk(dev(codes_h), binding.CODES_U8, luts, 100)
    gd, gi, luts_h = host(d), host(i), host(luts)
    od, oi = orc.adc_scan_topk_f32(codes_h, orc.CODES_U8, np.ascontiguousarray(luts_h[SAMPLE_Q]), 100)
    for r, q in enumerate(SAMPLE_Q):
        check_float_topk(gd[q], gi[q], od[r], oi[r], codes_h, orc.CODES_U8, luts_h[q], FULL_N)
    # properties that hold for every query: ascending, ids valid and distinct
    assert np.all(np.diff(gd, axis=1) >= 0) and gi.min() >= 0 and gi.max() < FULL_N
    assert all(len(set(row.tolist())) == 100 for row in gi[::50])


def test_full_size_config2_sampled(ctx):
    """Config 2 as bench.py runs it (25 M packed codes, 1000 queries, top-1000 by integer sums, rerank
    to top-100): stage-wise parity on a sample of the queries."""
    mix = datagen.sift_like()
    queries = dev(mix.sample(FULL_NQ, datagen.SEED_QUERIES))
    cb = dev(datagen.sampled_codebooks(mix, 16, 16))
    packed_h = datagen.random_codes(FULL_N, 8, seed=datagen.SEED_CODES + 1)
    fmt = orc.CODES_U4_PACKED
    dpacked = dev(packed_h)
    luts = ctx.pq_build_luts(queries, cb)
    qmax = ctx.pq_qmax_prescan(dpacked, fmt, luts, 2000, 1000)
    qluts, _, _ = ctx.pq_quantize_luts(luts, qmax)
    sums, cand = ctx.pq_adc_scan_topk(dpacked, fmt, qluts, 1000)
    dist, ids = ctx.pq_rerank_f32(dpacked, fmt, luts, cand, 100)
    luts_h, qmax_h, qluts_h, cand_h = host(luts), host(qmax), host(qluts), host(cand)
    ref_q, _, _ = orc.quantize_luts(np.ascontiguousarray(luts_h[SAMPLE_Q]), np.ascontiguousarray(qmax_h[SAMPLE_Q]))
    assert np.array_equal(qluts_h[SAMPLE_Q], ref_q)
    os_, oi = orc.adc_scan_topk_u8(packed_h, fmt, np.ascontiguousarray(qluts_h[SAMPLE_Q]), 1000)
    check_exact_topk(host(sums)[SAMPLE_Q], cand_h[SAMPLE_Q], os_, oi)
    od, oid = orc.rerank_f32(packed_h, fmt, np.ascontiguousarray(luts_h[SAMPLE_Q]), np.ascontiguousarray(cand_h[SAMPLE_Q]), 100)
    gd, gi = host(dist), host(ids)
    for r, q in enumerate(SAMPLE_Q):
        np.testing.assert_allclose(gd[q], od[r], rtol=RTOL)
        exact = orc.adc_all_f32(packed_h[gi[q]], fmt, luts_h[q])
        np.testing.assert_allclose(gd[q], exact, rtol=RTOL)
        assert np.all(exact <= od[r][-1] * (1 + RTOL))


def test_config3_gist_like_16x8_sampled(ctx):
    """Config 3 shape: d=960 mixture in [0,1], 16 x 256 codebooks (60 dims each), 1 M 16-byte codes, 1000
    queries, top-100.  Tables against the oracle for a sample of queries (the oracle's table build is slow),
    scan results for the same sample."""
    mix = datagen.gist_like()
    queries_h = mix.sample(FULL_NQ, datagen.SEED_QUERIES)
    cb_h = datagen.sampled_codebooks(mix, 16, 256)
    codes_h = datagen.random_codes(1_000_000, 16, seed=datagen.SEED_CODES + 4)
    luts = ctx.pq_build_luts(dev(queries_h), dev(cb_h))
    d, i = ctx.pq_adc_scan_topk(dev(codes_h), binding.CODES_U8, luts, 100)
    luts_h, gd, gi = host(luts), host(d), host(i)
    ref = orc.build_luts(np.ascontiguousarray(queries_h[SAMPLE_Q]), cb_h)
    np.testing.assert_allclose(luts_h[SAMPLE_Q], ref, rtol=4e-6, atol=0)
    od, oi = orc.adc_scan_topk_f32(codes_h, orc.CODES_U8, np.ascontiguousarray(luts_h[SAMPLE_Q]), 100)
    for r, q in enumerate(SAMPLE_Q):
        check_float_topk(gd[q], gi[q], od[r], oi[r], codes_h, orc.CODES_U8, luts_h[q], len(codes_h))



def test_scan_f32_few_queries_large_database_wide_first_bound(ctx):
    """Few query groups over a database large enough for the first bound to come from n / 64 codes
    (several seed slices): 8 x 256 tables, 3 and 17 queries, ragged size; top-100 and top-1."""
    r = np.random.default_rng(47)
    n = 9_000_011
    codes = r.integers(0, 256, (n, 8), dtype=np.uint8)
    codes[n // 2:n // 2 + 300] = codes[:300]          # exact ties across slices
    luts_h = (r.random((17, 8, 256)) * 100).astype(np.float32)
    run_float_scan(ctx, codes, orc.CODES_U8, luts_h[:3], 100)
    run_float_scan(ctx, codes, orc.CODES_U8, luts_h, 1)
    # distances descending with the row number for query 0: the first bound (from the front of the
    # database) is the loosest possible
    d0 = orc.adc_all_f32(codes[:2_000_000], orc.CODES_U8, luts_h[0])
    worst = np.ascontiguousarray(codes[:2_000_000][np.argsort(-d0, kind="stable")])
    big = np.concatenate([worst, codes[2_000_000:5_000_000]])
    run_float_scan(ctx, big, orc.CODES_U8, luts_h[:2], 100)


def test_scan_u4_few_queries_large_database_wide_first_bound(ctx):
    """The integer scan's first bound from n / 64 codes (several seed slices): bit-exact top-100 and top-1000."""
    r = np.random.default_rng(49)
    n = 9_000_011
    packed = r.integers(0, 256, (n, 8), dtype=np.uint8)
    qluts = r.integers(0, 256, (11, 16, 16), dtype=np.uint8)
    run_int_scan(ctx, packed, orc.CODES_U4_PACKED, qluts[:2], 100)
    run_int_scan(ctx, packed, orc.CODES_U4_PACKED, qluts, 1000)
    qluts[0, :, :] = 7                                  # every code has the same sum: ids decide
    run_int_scan(ctx, packed, orc.CODES_U4_PACKED, qluts[:1], 100)


# --------------------------------------------- 8x8 float scan, 8-bit lower bounds, 16 queries per pass
# 512 queries and more (enough groups of 16 to fill the GPU) take the loop on 8-bit lower bounds; these
# cases aim at what is specific to it: ragged last group, saturating entries, degenerate ranges, ties.
def many_queries(r, nq, spread=50.0, offset=200.0):
    return (r.random((nq, 8, 256)) * spread + r.random((nq, 8, 1)) * offset).astype(np.float32)


@pytest.mark.parametrize("n,nq,topk", [(65536, 512, 100), (70_001, 520, 1), (90_003, 777, 128), (66_000, 513, 1000),
                                       (75_001, 530, 129), (100_003, 512, 512), (80_001, 249, 100), (66_000, 250, 1000)])
def test_scan_f32_16_queries_per_pass_sizes(ctx, n, nq, topk):
    r = np.random.default_rng(n + nq)
    codes = r.integers(0, 256, (n, 8), dtype=np.uint8)
    run_float_scan(ctx, codes, orc.CODES_U8, many_queries(r, nq), topk)


def test_scan_f32_16_queries_per_pass_degenerate_tables(ctx, opts):
    r = np.random.default_rng(23)
    n, nq = 70_001, 515
    codes = r.integers(0, 256, (n, 8), dtype=np.uint8)
    # a huge dynamic range: most 8-bit entries saturate
    luts_h = np.exp(r.random((nq, 8, 256)) * 30 - 10).astype(np.float32)
    run_float_scan(ctx, codes, orc.CODES_U8, luts_h, 100)
    # a large common offset with a tiny spread: no fp32 resolution for a threshold (no pruning for those queries),
    # mixed with ordinary queries in the same groups
    luts_h = many_queries(r, nq)
    luts_h[::3] = (1.0e7 + r.random((len(luts_h[::3]), 8, 256))).astype(np.float32)
    run_float_scan(ctx, codes, orc.CODES_U8, luts_h, 100)
    # few distinct table values: exact sums, massive exact ties, unique (value, id) order
    luts_h = r.integers(0, 3, (nq, 8, 256)).astype(np.float32)
    d, i = ctx.pq_adc_scan_topk(dev(codes), binding.CODES_U8, dev(luts_h), 100)
    od, oi = orc.adc_scan_topk_f32(codes, orc.CODES_U8, luts_h, 100)
    assert np.array_equal(host(i), oi) and np.array_equal(host(d), od)
    # every code is the per-table minimiser of query 0: its first bound leaves no range
    luts_h = many_queries(r, nq)
    same = np.tile(luts_h[0].argmin(axis=1).astype(np.uint8), (n, 1))
    run_float_scan(ctx, same, orc.CODES_U8, luts_h, 100)
    # the 16-bit loop for the same inputs (switch), as a cross-check of the switch itself
    opts.set("scan_q8", 0)
    run_float_scan(ctx, codes, orc.CODES_U8, luts_h, 100)


def test_scan_f32_16_queries_per_pass_worst_case_order_and_duplicates(ctx):
    r = np.random.default_rng(29)
    n, nq = 80_000, 512
    codes = r.integers(0, 256, (n, 8), dtype=np.uint8)
    luts_h = many_queries(r, nq)
    d0 = orc.adc_all_f32(codes, orc.CODES_U8, luts_h[0])
    worst = np.ascontiguousarray(codes[np.argsort(-d0, kind="stable")])    # far to near for query 0
    worst[40_000:40_500] = worst[-500:]                                    # duplicates of the best codes
    run_float_scan(ctx, worst, orc.CODES_U8, luts_h, 100)


# ------------------------------------------------- integer scan of many queries (8-bit lower bounds, 16 per pass)
def quantized_like_tables(r, nq):
    """u8 tables shaped like quantised distance tables: a spread of small values per component and a few
    saturated entries."""
    base = r.integers(0, 40, (nq, 16, 1))
    t = base + (r.random((nq, 16, 16)) ** 2 * 60).astype(np.int64)
    t[r.random((nq, 16, 16)) < 0.05] = 255
    return np.clip(t, 0, 255).astype(np.uint8)


@pytest.mark.parametrize("n,nq,topk", [(65536, 512, 100), (70_001, 520, 1), (90_003, 777, 128), (66_001, 513, 1000),
                                       (75_001, 530, 129), (100_003, 512, 512), (80_001, 249, 100), (66_000, 250, 1000)])
def test_scan_u4_16_queries_per_pass_sizes(ctx, n, nq, topk):
    r = np.random.default_rng(n + nq)
    packed = r.integers(0, 256, (n, 8), dtype=np.uint8)
    run_int_scan(ctx, packed, orc.CODES_U4_PACKED, quantized_like_tables(r, nq), topk)


def test_scan_u4_16_queries_per_pass_degenerate_tables(ctx, opts):
    r = np.random.default_rng(31)
    n, nq = 70_001, 515
    packed = r.integers(0, 256, (n, 8), dtype=np.uint8)
    # uniform bytes: wide sums, the 8-bit entries saturate for most codes
    run_int_scan(ctx, packed, orc.CODES_U4_PACKED, r.integers(0, 256, (nq, 16, 16), dtype=np.uint8), 100)
    # sums in 0..48 (thousands of ties at the bound), constant tables (no range at all), all 255, all 0
    qluts = r.integers(0, 4, (nq, 16, 16), dtype=np.uint8)
    qluts[1] = 255
    qluts[2] = 0
    qluts[3] = 7
    qluts[20:40] = quantized_like_tables(r, 20)
    run_int_scan(ctx, packed, orc.CODES_U4_PACKED, qluts, 100)
    run_int_scan(ctx, packed, orc.CODES_U4_PACKED, qluts, 400)
    # every code is the minimiser of query 0: its first bound equals the sum of the minima
    qluts = quantized_like_tables(r, nq)
    best = qluts[0].argmin(axis=1)
    same = np.tile((best[0::2] | (best[1::2] << 4)).astype(np.uint8), (n, 1))
    run_int_scan(ctx, same, orc.CODES_U4_PACKED, qluts, 100)
    # the 16-bit loop for the same inputs (switch)
    opts.set("scan_q8", 0)
    run_int_scan(ctx, packed, orc.CODES_U4_PACKED, qluts, 100)


def test_scan_u4_16_queries_per_pass_worst_case_order_and_duplicates(ctx):
    r = np.random.default_rng(37)
    n, nq = 80_000, 512
    packed = r.integers(0, 256, (n, 8), dtype=np.uint8)
    qluts = quantized_like_tables(r, nq)
    d0 = orc.adc_all_u8(packed, orc.CODES_U4_PACKED, qluts[0]).astype(np.int64)
    worst = np.ascontiguousarray(packed[np.argsort(-d0, kind="stable")])   # far to near for query 0
    worst[40_000:40_500] = worst[-500:]                                    # duplicates of the best codes
    run_int_scan(ctx, worst, orc.CODES_U4_PACKED, qluts, 100)
    run_int_scan(ctx, worst, orc.CODES_U4_PACKED, qluts, 500)


def test_scan_16_queries_per_pass_first_round_of_short_items(ctx, opts):
    """Long result lists start with a round of short chunks (one per block) before the long ones: here forced onto a
    small database (one block tile per short chunk, few blocks), ragged end, float and integer scans."""
    opts.set("scan_head", 1)
    opts.set("scan_blocks", 20)   # one short chunk per group (513 queries), two (300 queries)
    r = np.random.default_rng(43)
    for n, nq, topk in [(100_003, 513, 1000), (140_001, 300, 300)]:
        codes = r.integers(0, 256, (n, 8), dtype=np.uint8)
        run_float_scan(ctx, codes, orc.CODES_U8, many_queries(r, nq), topk)
        run_int_scan(ctx, codes, orc.CODES_U4_PACKED, quantized_like_tables(r, nq), topk)


# ----------------------------------------------------------------------------- encoded data at full size
ENC_UNIQUE = 400_000   # vectors encoded by the oracle; the 25 M rows are drawn from them (so every code has ~60 exact copies)


def test_full_size_config1_encoded_sampled(ctx):
    """Config 1 on encoded data: mixture vectors encoded by the oracle against codebooks trained by the oracle's
    k-means, rows drawn from them to fill 25 M (clustered distances, heavy duplicates: what a pruning scan finds
    hardest), 1000 queries, top-100; complete results of a sample of the queries against the oracle."""
    _, _, cb, unique = sift_pq(8, 256, ENC_UNIQUE, 16)
    codes_h = datagen.tile_rows(unique, FULL_N)
    queries = dev(datagen.sift_like().sample(FULL_NQ, datagen.SEED_QUERIES))
    luts = ctx.pq_build_luts(queries, dev(cb))
    d, i = ctx.pq_adc_scan_topk(dev(codes_h), binding.CODES_U8, luts, 100)
    gd, gi, luts_h = host(d), host(i), host(luts)
    od, oi = orc.adc_scan_topk_f32(codes_h, orc.CODES_U8, np.ascontiguousarray(luts_h[SAMPLE_Q]), 100)
    for r, q in enumerate(SAMPLE_Q):
        check_float_topk(gd[q], gi[q], od[r], oi[r], codes_h, orc.CODES_U8, luts_h[q], FULL_N)
        np.testing.assert_allclose(gd[q], od[r], rtol=RTOL)
    assert np.all(np.diff(gd, axis=1) >= 0) and gi.min() >= 0 and gi.max() < FULL_N
    assert all(len(set(row.tolist())) == 100 for row in gi[::50])


def test_full_size_config2_encoded_sampled(ctx):
    """Config 2 on encoded data (16 x 4, packed; rows drawn from oracle-encoded vectors): 8-bit tables are coarse where
    the codes crowd, so thousands of codes tie at the 1000th integer sum and rows decide; stage-wise, bit-exact."""
    _, _, cb, unique = sift_pq(16, 16, ENC_UNIQUE, 16)
    fmt = orc.CODES_U4_PACKED
    packed_h = datagen.tile_rows(orc.pack_u4(unique), FULL_N)
    queries = dev(datagen.sift_like().sample(FULL_NQ, datagen.SEED_QUERIES))
    dpacked = dev(packed_h)
    luts = ctx.pq_build_luts(queries, dev(cb))
    qmax = ctx.pq_qmax_prescan(dpacked, fmt, luts, 2000, 1000)
    qluts, _, _ = ctx.pq_quantize_luts(luts, qmax)
    luts_h, qmax_h, qluts_h = host(luts), host(qmax), host(qluts)
    ref_q, _, _ = orc.quantize_luts(np.ascontiguousarray(luts_h[SAMPLE_Q]), np.ascontiguousarray(qmax_h[SAMPLE_Q]))
    assert np.array_equal(qluts_h[SAMPLE_Q], ref_q)
    for topk in (1000, 100):
        sums, cand = ctx.pq_adc_scan_topk(dpacked, fmt, qluts, topk)
        os_, oi = orc.adc_scan_topk_u8(packed_h, fmt, np.ascontiguousarray(qluts_h[SAMPLE_Q]), topk)
        check_exact_topk(host(sums)[SAMPLE_Q], host(cand)[SAMPLE_Q], os_, oi)
    # every query: sums ascending, rows valid, distinct, and ascending inside runs of equal sums
    gs, gc = host(sums).astype(np.int64), host(cand)
    assert np.all(np.diff(gs, axis=1) >= 0) and gc.min() >= 0 and gc.max() < FULL_N
    order_key = gs * (1 << 32) + gc
    assert np.all(np.diff(order_key, axis=1) > 0)


@pytest.mark.parametrize("nq", [20, 300])
def test_scan_u4_ties_at_the_kth_sum_far_beyond_k(ctx, nq):
    """Tables with entries 0 / 1 / 40: sums take a handful of values and tens of thousands of codes tie at the
    k-th; the result is the tied codes with the smallest rows.  Both integer loops, short and long lists."""
    r = np.random.default_rng(91 + nq)
    n = 400_003
    packed = r.integers(0, 256, (n, 8), dtype=np.uint8)
    qluts = r.choice(np.array([0, 1, 40], dtype=np.uint8), size=(nq, 16, 16), p=[0.5, 0.3, 0.2])
    qluts[1] = 0          # every code ties
    qluts[2, :, 1:] = 7   # one cheap entry per table: sums 0, 7, 14, ...
    qluts[2, :, 0] = 0
    for topk in (100, 1000, 1):
        run_int_scan(ctx, packed, orc.CODES_U4_PACKED, qluts, topk)


@pytest.mark.parametrize("m,nq", [(8, 5), (8, 300), (16, 5), (16, 40)])
def test_scan_f32_first_bound_equal_to_the_sum_of_the_table_minima(ctx, m, nq):
    """More than k codes are exact copies of a query's best possible code (every table entry at its minimum), as
    happens with encoded high-dimensional data: the first bound leaves no range for the lower-bound tables.
    Query 0: thousands of copies; query 1: k - 1 copies (the k-th result is an ordinary code); the others: none."""
    r = np.random.default_rng(300 + m + nq)
    n, topk = 200_003, 100
    codes = r.integers(0, 256, (n, m), dtype=np.uint8)
    luts_h = (r.random((nq, m, 256)) * 50 + r.random((nq, m, 1)) * 100).astype(np.float32)
    best0 = luts_h[0].argmin(axis=1).astype(np.uint8)
    best1 = luts_h[1].argmin(axis=1).astype(np.uint8)
    codes[r.choice(n, 5000, replace=False)] = best0
    rows1 = r.choice(n, topk - 1, replace=False)
    codes[rows1] = best1
    gd, gi, od, oi = run_float_scan(ctx, codes, orc.CODES_U8, luts_h, topk)
    assert np.all(gd[0] == gd[0][0])                       # a hundred copies of the best code
    np.testing.assert_allclose(gd, od, rtol=RTOL)
    run_float_scan(ctx, codes, orc.CODES_U8, luts_h, 1000 if nq <= 40 else 300)
