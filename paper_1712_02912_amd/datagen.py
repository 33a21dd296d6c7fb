"""Seeded synthetic inputs shared by the CPU oracle's tests and the GPU tests/bench.

Only input generation lives here -- no distance, table, quantisation, encoding
or selection arithmetic.  The inputs stand in for the descriptor datasets the
thesis measures on (128-dimensional non-negative byte-range local descriptors,
960-dimensional global descriptors in [0, 1], one 25 M-code inverted list, a
billion-code index with 2^16 cells); none of those datasets is reproduced.

All randomness comes from numpy's PCG64 with the seeds below, so that both sides
of every comparison see bit-identical inputs.  Inputs too large to be made on the host in
reasonable time (tens of millions of vectors, a billion codes) are drawn on the GPU from
torch's seeded generator by the ``*_device`` functions; they are copied to the host when
the CPU side needs them.
"""
import numpy as np

SEED_DATA = 1234
SEED_QUERIES = 4321
SEED_KMEANS = 7
SEED_CODES = 99
SEED_ZIPF = 2024


def _rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


class Mixture:
    """Gaussian mixture with isotropic components; samples are clipped to [lo, hi]."""

    def __init__(self, d, ncomp, mean_range, sigma_range, clip, seed=SEED_DATA):
        r = _rng(seed)
        self.d = d
        self.means = r.uniform(mean_range[0], mean_range[1], size=(ncomp, d))
        self.sigmas = r.uniform(sigma_range[0], sigma_range[1], size=ncomp)
        self.weights = r.dirichlet(np.ones(ncomp))
        self.clip = clip

    def sample(self, n, seed):
        r = _rng(seed)
        comp = r.choice(len(self.weights), size=n, p=self.weights)
        x = self.means[comp] + r.standard_normal((n, self.d)) * self.sigmas[comp][:, None]
        return np.clip(x, self.clip[0], self.clip[1]).astype(np.float32)


    def sample_device(self, n, seed, device="cuda"):
        """The same mixture drawn on the GPU (torch generator seeded with `seed`): [n][d] f32 device tensor."""
        import torch
        gen = torch.Generator(device=device).manual_seed(int(seed))
        w = torch.from_numpy(self.weights).to(device)
        comp = torch.multinomial(w, n, replacement=True, generator=gen)
        means = torch.from_numpy(self.means.astype(np.float32)).to(device)
        sig = torch.from_numpy(self.sigmas.astype(np.float32)).to(device)
        x = torch.randn((n, self.d), device=device, dtype=torch.float32, generator=gen)
        x.mul_(sig[comp][:, None]).add_(means[comp])
        return x.clamp_(self.clip[0], self.clip[1])


def random_codes_device(n, code_bytes, seed=SEED_CODES, device="cuda"):
    """[n][code_bytes] uniformly random bytes drawn on the GPU."""
    import torch
    gen = torch.Generator(device=device).manual_seed(int(seed))
    return torch.randint(0, 256, (n, code_bytes), dtype=torch.uint8, device=device, generator=gen)


def tile_rows(unique, n, seed=SEED_CODES + 17):
    """n rows drawn with replacement (seeded) from the rows of `unique`: a large database with the value
    distribution of a smaller encoded one (and many exact duplicates)."""
    idx = _rng(seed).integers(0, unique.shape[0], size=n)
    return np.ascontiguousarray(unique[idx])


def sift_like():
    """d=128, 64 components, values in [0, 255] (stand-in for byte-range local descriptors)."""
    return Mixture(128, 64, (0.0, 128.0), (8.0, 32.0), (0.0, 255.0))


def gist_like():
    """d=960, 128 components, values in [0, 1] (stand-in for global descriptors)."""
    return Mixture(960, 128, (0.2, 0.8), (0.02, 0.1), (0.0, 1.0))


def kmeans_init_idx(n_train, m, k, seed=SEED_KMEANS):
    """For each of the m sub-spaces, k distinct training-row indexes used as initial centroids."""
    r = _rng(seed)
    return np.stack([r.choice(n_train, size=k, replace=False) for _ in range(m)]).astype(np.int64)


def sampled_codebooks(mix, m, k, seed=SEED_KMEANS):
    """Codebooks [m][k][d/m] whose centroids are sub-vectors of k mixture samples.

    A stand-in for trained codebooks where only the value distribution of the
    lookup tables matters (throughput runs): no training arithmetic involved.
    """
    x = mix.sample(k, seed)
    dsub = mix.d // m
    return np.ascontiguousarray(x.reshape(k, m, dsub).transpose(1, 0, 2))


def clustered_codebooks(mix, m, k, kbar=256, spread=6.0, seed=SEED_KMEANS + 11):
    """Stand-in for jointly trained codebooks of a 16-bit product quantizer and its derived 8-bit
    quantizer (throughput runs and parity inputs): kbar cluster centres per sub-space taken from
    mixture samples, centroid i scattered around centre i % kbar, so the low bits of an index
    name its cluster; the derived centroid of a cluster is the mean of its members.
    Returns (codebooks [m][k][d/m], derived [m][kbar][d/m])."""
    centres = sampled_codebooks(mix, m, kbar, seed)                      # [m][kbar][dsub]
    r = _rng(seed + 1)
    cb = centres[:, np.arange(k) % kbar, :] + r.normal(0.0, spread, size=(m, k, centres.shape[2])).astype(np.float32)
    cb = np.ascontiguousarray(cb, dtype=np.float32)
    derived = cb.astype(np.float64).reshape(m, k // kbar, kbar, -1).mean(axis=1).astype(np.float32)
    return cb, derived


def random_codes(n, code_bytes, seed=SEED_CODES, chunk=1 << 24):
    """[n][code_bytes] uniformly random bytes, generated in chunks of rows."""
    out = np.empty((n, code_bytes), np.uint8)
    r = _rng(seed)
    for start in range(0, n, chunk):
        stop = min(n, start + chunk)
        out[start:stop] = r.integers(0, 256, size=(stop - start, code_bytes), dtype=np.uint8)
    return out


def zipf_list_sizes(ntotal, nlist, s=1.0, seed=SEED_ZIPF):
    """List sizes proportional to rank^-s, ranks randomly permuted over list ids; sums to ntotal."""
    w = 1.0 / np.arange(1, nlist + 1, dtype=np.float64) ** s
    sizes = np.floor(w / w.sum() * ntotal).astype(np.int64)
    sizes[0] += ntotal - sizes.sum()
    r = _rng(seed)
    return sizes[r.permutation(nlist)]


def offsets_from_sizes(sizes):
    off = np.zeros(len(sizes) + 1, np.int64)
    np.cumsum(sizes, out=off[1:])
    return off
