"""Helpers shared by the GPU parity tests (comparison rules and fixtures)."""
import functools

import numpy as np

from oracle import pq_oracle as orc
from paper_1712_02912_amd import datagen

RTOL = 1e-5  # float ADC distances: relative tolerance stated for this path


def check_float_topk(gpu_dist, gpu_ids, orc_dist, orc_ids, codes, code_fmt, lut, n):
    """Float top-k rule: distances within RTOL, sets identical up to ties inside RTOL.

    tau = oracle's k-th distance.  Every id the GPU returns must have an oracle distance
    <= tau*(1+RTOL); every oracle id with distance < tau*(1-RTOL) must be returned; for each
    returned id the GPU distance must match the oracle distance of that id within RTOL.
    """
    topk = len(orc_ids)
    got = min(topk, n)
    assert np.all(gpu_ids[got:] == -1) and np.all(np.isinf(gpu_dist[got:])), "padding"
    gi, gd = gpu_ids[:got], gpu_dist[:got]
    assert len(set(gi.tolist())) == got, "duplicate ids"
    assert np.all(gi >= 0) and np.all(gi < n)
    assert np.all(np.diff(gd) >= 0), "not ascending"
    if got == 0:
        return
    exact = orc.adc_all_f32(codes[gi], code_fmt, lut).astype(np.float64)
    np.testing.assert_allclose(gd, exact, rtol=RTOL, atol=0)
    tau = float(orc_dist[got - 1])
    assert np.all(exact <= tau * (1 + RTOL) + 1e-30), "an id outside the top-k tolerance band was returned"
    must = orc_ids[:got][orc_dist[:got] < tau * (1 - RTOL)]
    missing = set(must.tolist()) - set(gi.tolist())
    assert not missing, f"ids missing from the GPU result: {sorted(missing)[:5]}"


def check_exact_topk(gpu_val, gpu_ids, orc_val, orc_ids):
    """Integer path: sums and ids bit-exact, including the padding."""
    assert np.array_equal(gpu_ids, orc_ids)
    assert np.array_equal(gpu_val.astype(np.uint32), orc_val.astype(np.uint32))


@functools.lru_cache(maxsize=None)
def sift_pq(m, k, n, nq, ntrain=20000, iters=10):
    """Config-0 style fixture: mixture data, trained codebooks, encoded database, queries."""
    mix = datagen.sift_like()
    train = mix.sample(ntrain, datagen.SEED_KMEANS + 1)
    base = mix.sample(n, datagen.SEED_DATA + 1)
    queries = mix.sample(nq, datagen.SEED_QUERIES)
    cb = orc.pq_train(train, m, k, iters, datagen.kmeans_init_idx(ntrain, m, k))
    codes = orc.pq_encode(base, cb)
    return base, queries, cb, codes


def check_float_topk_ranked(gpu_dist, gpu_ids, orc_dist, orc_ids):
    """Float top-k rule when only the oracle's own top-k is at hand (IVF).

    Distances agree rank by rank within RTOL; an id may differ from the oracle's at a rank only
    where distances tie within RTOL (with another returned entry, or with the k-th at the boundary).
    """
    np.testing.assert_allclose(gpu_dist, orc_dist, rtol=RTOL, atol=0)
    valid = orc_ids >= 0
    assert np.array_equal(gpu_ids >= 0, valid), "padding differs"
    assert len(set(gpu_ids[valid].tolist())) == valid.sum(), "duplicate ids"
    where = {int(i): r for r, i in enumerate(orc_ids) if i >= 0}
    last = orc_dist[valid][-1] if valid.any() else 0.0
    for r in np.flatnonzero(valid & (gpu_ids != orc_ids)):
        j = where.get(int(gpu_ids[r]))
        if j is None:   # not in the oracle's list at all: only acceptable as a tie with the k-th
            assert abs(gpu_dist[r] - last) <= RTOL * abs(last) + 1e-30, f"rank {r}: id {gpu_ids[r]} is not a boundary tie"
        else:
            assert abs(orc_dist[j] - orc_dist[r]) <= 2 * RTOL * abs(orc_dist[r]) + 1e-30, f"rank {r}: ids differ without a tie"
