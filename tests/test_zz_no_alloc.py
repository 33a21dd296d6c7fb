"""The scan entry point that allocates nothing (fixed scratch array inside the library) against
pq_adc_scan_topk, through the C ABI: two calls in a row, the second on a smaller input."""
import numpy as np
import pytest
import torch

from paper_1712_02912_amd import binding

pytestmark = pytest.mark.gpu


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def both(ctx, codes, fmt, luts, topk):
    """Results of the allocating entry point and of the one that allocates nothing (outputs are the caller's)."""
    vdt = torch.int32 if luts.dtype == torch.uint8 else torch.float32
    nq = luts.shape[0]
    out = (torch.full((nq, topk), -7, dtype=vdt, device="cuda"), torch.full((nq, topk), -7, dtype=torch.int64, device="cuda"))
    ref_v, ref_i = ctx.pq_adc_scan_topk(codes, fmt, luts, topk)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    v, i = ctx.pq_adc_scan_topk(codes, fmt, luts, topk, out=out, noalloc=True)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    # once more with the driver's own count of free device memory around it: the call takes none
    free_before = torch.cuda.mem_get_info()[0]
    ctx.pq_adc_scan_topk(codes, fmt, luts, topk, out=out, noalloc=True)
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] == free_before
    return ref_v.cpu().numpy(), ref_i.cpu().numpy(), v.cpu().numpy(), i.cpu().numpy()


def check_float(rv, ri, v, i):
    """Same kernels on both sides: distances within 1e-5 (in fact equal), ids equal except inside ties."""
    np.testing.assert_allclose(v, rv, rtol=1e-5, atol=0)
    differ = ri != i
    if differ.any():   # an id may only differ where its distance ties with a neighbour's within the tolerance
        for q, r in zip(*np.nonzero(differ)):
            row = rv[q]
            assert np.isclose(row, row[r], rtol=1e-5, atol=0).sum() > 1, (q, r)
        assert all(len(set(i[q][i[q] >= 0].tolist())) == (i[q] >= 0).sum() for q in range(i.shape[0]))


def test_noalloc_scan_matches_allocating_scan_twice_in_a_row():
    ctx = binding.Context(0)
    r = np.random.default_rng(2024)
    # first call: pruned float scan over 300 003 codes, 40 queries (5 groups, ragged end), top-100;
    # second call: a smaller input (plain float loop, 20 001 codes, 7 queries, top-10) on the same scratch
    for n, nq, topk in ((300_003, 40, 100), (20_001, 7, 10)):
        codes = dev(r.integers(0, 256, (n, 8), dtype=np.uint8))
        luts = dev((r.random((nq, 8, 256)) * 100).astype(np.float32))
        check_float(*both(ctx, codes, binding.CODES_U8, luts, topk))
    # integer path, bit-exact: large then small
    for n, nq, topk in ((250_001, 33, 128), (9_000, 3, 50)):
        packed = dev(r.integers(0, 256, (n, 8), dtype=np.uint8))
        qluts = dev(r.integers(0, 256, (nq, 16, 16), dtype=np.uint8))
        rv, ri, v, i = both(ctx, packed, binding.CODES_U4_PACKED, qluts, topk)
        assert np.array_equal(rv, v) and np.array_equal(ri, i)
    # the general kernel (m = 4, k = 64) and fewer codes than results (padding)
    codes = dev(r.integers(0, 64, (5_000, 4), dtype=np.uint8))
    luts = dev((r.random((3, 4, 64)) * 10).astype(np.float32))
    check_float(*both(ctx, codes, binding.CODES_U8, luts, 20))
    rv, ri, v, i = both(ctx, codes[:5].contiguous(), binding.CODES_U8, luts, 20)
    assert np.array_equal(ri, i) and np.array_equal(rv, v) and np.all(i[:, 5:] == -1)
    torch.cuda.synchronize()
    ctx.close()


def test_noalloc_scan_rejects_what_does_not_fit():
    """1000 queries take 16 queries per pass and more scratch than the fixed array holds: a clear error, outputs untouched."""
    ctx = binding.Context(0)
    r = np.random.default_rng(7)
    codes = dev(r.integers(0, 256, (100_000, 8), dtype=np.uint8))
    luts = dev((r.random((1000, 8, 256)) * 100).astype(np.float32))
    out = (torch.full((1000, 100), -7.0, device="cuda"), torch.full((1000, 100), -7, dtype=torch.int64, device="cuda"))
    with pytest.raises(binding.PqError) as e:
        ctx.pq_adc_scan_topk(codes, binding.CODES_U8, luts, 100, out=out, noalloc=True)
    assert e.value.code == -5 and "fixed scratch" in str(e.value)
    torch.cuda.synchronize()
    assert bool((out[1] == -7).all())
    # the context still serves the allocating entry point and smaller no-alloc calls afterwards
    v, i = ctx.pq_adc_scan_topk(codes, binding.CODES_U8, luts[:5].contiguous(), 10, noalloc=True)
    rv, ri = ctx.pq_adc_scan_topk(codes, binding.CODES_U8, luts[:5].contiguous(), 10)
    torch.cuda.synchronize()
    assert torch.equal(i, ri) and torch.equal(v, rv)
    ctx.close()
