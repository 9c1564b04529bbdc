"""Seeded synthetic inputs shaped like the paper's workloads.

This module serves BOTH the CPU oracle's tests and the HIP path's tests and
bench, and therefore holds none of the search method itself: it only draws
numbers.  Every array handed to the two sides comes from here as the same
bytes.

The paper evaluates on BIGANN (128-d SIFT descriptors), Deep1B (96-d) and
Contriever embeddings (768-d, inner product), 10k queries each (Sec. 2
"datasets").  None of those files is used; the recipes below only borrow
their shapes and value structure (non-negative integer descriptors,
unit-norm embeddings).

Index parameters are also inputs here: coarse centroids are database rows
picked by a seeded permutation, and every sub-codebook is a set of K residual
sub-vectors of rows picked by a second seeded permutation (the residual is
taken against the row's closest centroid in float64; this is a recipe for
producing plausible codebook numbers, not the library's assignment step).
"""
import numpy as np

# name -> parameters; sizes can be overridden for scaled-down test cases.
CONFIGS = {
    # tiny IVF-PQ, L2
    "C1": dict(kind="gauss", nb=10_000, nq=100, d=32, nlist=16, M=8, nbits=8, metric=0,
               k=10, nprobe=4, seed=1001),
    # flat exact L2 k-NN, SIFT-like
    "C2": dict(kind="sift", nb=1_000_000, nq=10_000, d=128, ncomp=1000, sigma=20.0, metric=0,
               k=100, seed=1002),
    # IVF4096,PQ16x8, L2, SIFT-like (same data recipe as C2)
    "C3": dict(kind="sift", nb=1_000_000, nq=10_000, d=128, ncomp=1000, sigma=20.0, nlist=4096,
               M=16, nbits=8, metric=0, k=10, nprobe=16, seed=1002),
    # IVF65536,PQ32x8, L2, Deep-like unit-norm
    "C4": dict(kind="unit", nb=100_000_000, nq=10_000, d=96, ncomp=10_000, sigma=0.3,
               nlist=65536, M=32, nbits=8, metric=0, k=100, nprobe=64, seed=1004),
    # IVF16384,PQ64x4, inner product, embedding-like unit-norm; queries are
    # perturbed database rows
    "C5": dict(kind="unit", nb=10_000_000, nq=10_000, d=768, ncomp=5000, sigma=0.3,
               nlist=16384, M=64, nbits=4, metric=1, k=10, nprobe=32, seed=1005,
               query_noise=0.05),
}


def config(name, **overrides):
    c = dict(CONFIGS[name])
    c.update(overrides)
    return c


def _normalise(a):
    n = np.sqrt((a.astype(np.float64) ** 2).sum(axis=1, keepdims=True))
    n[n == 0] = 1.0
    return (a / n).astype(np.float32)


def gauss(n, d, rng):
    return rng.standard_normal((n, d), dtype=np.float32)


def sift_like(n, d, centres, sigma, rng, chunk=65536):
    """Non-negative integer-valued descriptors: a mixture of isotropic
    Gaussians clipped to [0, 255] and rounded, stored as fp32."""
    out = np.empty((n, d), dtype=np.float32)
    for s in range(0, n, chunk):
        e = min(n, s + chunk)
        comp = rng.integers(0, centres.shape[0], size=e - s)
        v = centres[comp] + sigma * rng.standard_normal((e - s, d), dtype=np.float32)
        out[s:e] = np.rint(np.clip(v, 0.0, 255.0))
    return out


def unit_mixture(n, d, centres, sigma, rng, chunk=65536):
    """Unit-norm embedding-like vectors from a mixture of Gaussians."""
    out = np.empty((n, d), dtype=np.float32)
    for s in range(0, n, chunk):
        e = min(n, s + chunk)
        comp = rng.integers(0, centres.shape[0], size=e - s)
        v = centres[comp] + sigma * rng.standard_normal((e - s, d), dtype=np.float32)
        out[s:e] = _normalise(v)
    return out


def make_data(cfg):
    """Returns (x [nb, d], q [nq, d]) fp32, C-contiguous."""
    rng = np.random.default_rng(cfg["seed"])
    nb, nq, d = cfg["nb"], cfg["nq"], cfg["d"]
    kind = cfg["kind"]
    if kind == "gauss":
        x = gauss(nb, d, rng)
        q = gauss(nq, d, rng)
    elif kind == "sift":
        centres = rng.uniform(0.0, 255.0, size=(cfg["ncomp"], d)).astype(np.float32)
        x = sift_like(nb, d, centres, cfg["sigma"], rng)
        q = sift_like(nq, d, centres, cfg["sigma"], rng)
    elif kind == "unit":
        centres = rng.standard_normal((cfg["ncomp"], d), dtype=np.float32)
        x = unit_mixture(nb, d, centres, cfg["sigma"], rng)
        if "query_noise" in cfg:
            pick = rng.integers(0, nb, size=nq)
            q = _normalise(x[pick] + cfg["query_noise"] * rng.standard_normal((nq, d), dtype=np.float32))
        else:
            q = unit_mixture(nq, d, centres, cfg["sigma"], rng)
    else:
        raise ValueError(kind)
    return np.ascontiguousarray(x), np.ascontiguousarray(q)


def make_centroids(x, nlist, seed):
    """Coarse centroids = the first nlist rows of a seeded shuffle of x."""
    rng = np.random.default_rng(seed + 7919)
    perm = rng.permutation(x.shape[0])[:nlist]
    return np.ascontiguousarray(x[perm])


def make_codebooks(x, centroids, M, nbits, seed):
    """Sub-codebook m = m-th slices of the residuals of K seeded sample rows.
    Returns [M, K, dsub] fp32."""
    K = 1 << nbits
    d = x.shape[1]
    dsub = d // M
    rng = np.random.default_rng(seed + 104729)
    rows = x[rng.permutation(x.shape[0])[:K]].astype(np.float64)
    if rows.shape[0] < K:  # fewer database rows than codewords: recycle
        rows = np.resize(rows, (K, d))
    c64 = centroids.astype(np.float64)
    d2 = (rows ** 2).sum(1)[:, None] - 2.0 * rows @ c64.T + (c64 ** 2).sum(1)[None, :]
    near = d2.argmin(axis=1)
    res = (rows - c64[near]).astype(np.float32)          # [K, d]
    cb = res.reshape(K, M, dsub).transpose(1, 0, 2)       # [M, K, dsub]
    return np.ascontiguousarray(cb)


def make_index_params(cfg, x):
    cent = make_centroids(x, cfg["nlist"], cfg["seed"])
    cb = make_codebooks(x, cent, cfg["M"], cfg["nbits"], cfg["seed"])
    return cent, cb


# ---- on-device generation for the configurations too large for host memory ------
# Same recipes as above, drawn with torch's generator ON THE DEVICE in chunks; the bytes that
# reach the oracle are copied back from these tensors (CPU and GPU random streams are not
# interchangeable, so the data are generated once and shared).

def make_data_device(cfg, device="cuda", chunk=4_000_000):
    """Returns (x [nb, d], q [nq, d]) fp32 torch tensors on `device` (kind 'unit' only)."""
    import torch
    assert cfg["kind"] == "unit"
    g = torch.Generator(device=device)
    g.manual_seed(cfg["seed"])
    nb, nq, d = cfg["nb"], cfg["nq"], cfg["d"]
    centres = torch.randn((cfg["ncomp"], d), generator=g, device=device, dtype=torch.float32)

    def draw(n):
        out = torch.empty((n, d), device=device, dtype=torch.float32)
        for s in range(0, n, chunk):
            e = min(n, s + chunk)
            comp = torch.randint(0, cfg["ncomp"], (e - s,), generator=g, device=device)
            v = centres[comp]
            v += cfg["sigma"] * torch.randn((e - s, d), generator=g, device=device, dtype=torch.float32)
            v /= v.norm(dim=1, keepdim=True).clamp_min(1e-30)
            out[s:e] = v
        return out

    x = draw(nb)
    if "query_noise" in cfg:
        pick = torch.randint(0, nb, (nq,), generator=g, device=device)
        q = x[pick] + cfg["query_noise"] * torch.randn((nq, d), generator=g, device=device, dtype=torch.float32)
        q /= q.norm(dim=1, keepdim=True).clamp_min(1e-30)
    else:
        q = draw(nq)
    return x, q


def make_index_params_device(cfg, x):
    """Centroids / codebooks for a device-resident x: the sampled rows are copied to the
    host and go through the same numpy recipe.  Returns numpy arrays."""
    import torch
    rng = np.random.default_rng(cfg["seed"] + 7919)
    rows = np.sort(rng.choice(cfg["nb"], cfg["nlist"], replace=False))
    cent = x[torch.from_numpy(rows).to(x.device)].cpu().numpy()
    K = 1 << cfg["nbits"]
    rng2 = np.random.default_rng(cfg["seed"] + 104729)
    rows2 = np.sort(rng2.choice(cfg["nb"], K, replace=False))
    sample = x[torch.from_numpy(rows2).to(x.device)].cpu().numpy()
    d, M = cfg["d"], cfg["M"]
    c64 = cent.astype(np.float64)
    s64 = sample.astype(np.float64)
    d2 = (s64 ** 2).sum(1)[:, None] - 2.0 * s64 @ c64.T + (c64 ** 2).sum(1)[None, :]
    res = (s64 - c64[d2.argmin(axis=1)]).astype(np.float32)
    cb = np.ascontiguousarray(res.reshape(K, M, d // M).transpose(1, 0, 2))
    return np.ascontiguousarray(cent), cb
