"""Seeded synthetic vector generators (stand-ins for SIFT1M / GIST1M / SIFT1B of Sec. 5).

The real benchmark sets are not available; these generators reproduce their
shapes, value ranges and clustered structure (many empty bins, skewed bin
occupancy, low intrinsic dimension inside a cluster).  Nothing here depends
on the quantisation method.

`sift_like` is counter based: element (id, dim) is a pure function of
(seed, id, dim) computed with 32/64-bit integer arithmetic only, so any chunk
of the database can be regenerated anywhere (CPU or GPU) bit-identically.
"""
import numpy as np

_U32 = np.uint64(0xFFFFFFFF)


# --------------------------------------------------------------------------
# Tiny: Gaussian mixture
# --------------------------------------------------------------------------
def tiny_mixture(n, d=32, components=64, sigma=0.05, seed=0, centre_seed=0):
    """n fp32 vectors from a `components`-component isotropic Gaussian mixture with
    centres uniform in [0,1]^d and standard deviation sigma, uniform weights.
    The centres depend on centre_seed only, so database (seed 0) and queries
    (seed 1) come from the same mixture."""
    crng = np.random.default_rng([centre_seed, 0xC3])
    centres = crng.random((components, d))
    rng = np.random.default_rng([seed, 0xDA7A])
    comp = rng.integers(0, components, size=n)
    x = centres[comp] + sigma * rng.standard_normal((n, d))
    return np.ascontiguousarray(x, dtype=np.float32)


# --------------------------------------------------------------------------
# SIFT-shaped: integer valued 0..255, clustered, heavy tailed, counter based
# --------------------------------------------------------------------------
def _mix32(x):
    """Avalanche a uint64 array holding 32-bit values (multiply-xorshift integer hash)."""
    x = x & _U32
    x ^= x >> np.uint64(16)
    x = (x * np.uint64(0x7FEB352D)) & _U32
    x ^= x >> np.uint64(15)
    x = (x * np.uint64(0x846CA68B)) & _U32
    x ^= x >> np.uint64(16)
    return x


def _stream(seed, ids, lane):
    """32-bit hash of (seed, id, lane); ids uint64 array (< 2**40), lane int or array."""
    s = np.uint64((int(seed) * 0x9E3779B1 + 0x7F4A7C15) & 0xFFFFFFFF)
    h = _mix32(ids ^ s)
    h = _mix32(h + (ids >> np.uint64(32)) * np.uint64(0x85EBCA6B) + np.uint64(0x165667B1))
    lane = np.asarray(lane, dtype=np.uint64)
    return _mix32(h ^ (lane * np.uint64(0x9E3779B1) & _U32))


N_CLUSTERS = 1000
N_LATENT = 24


def sift_like_tables(d=128, table_seed=0):
    """Small tables shared by database and queries: integer cluster centres with
    heavy-tailed per-dimension magnitudes (most mass near 0, long tail, clipped at 255),
    an integer latent basis, and the cumulative Zipf-like cluster weights as uint32
    thresholds."""
    rng = np.random.default_rng([table_seed, 0x51F7, d])
    dim_scale = rng.lognormal(mean=0.0, sigma=0.6, size=(1, d))
    centres = rng.exponential(scale=28.0, size=(N_CLUSTERS, d)) * dim_scale
    centres *= rng.random((N_CLUSTERS, d)) < 0.8          # SIFT histograms have many zeros
    centres = np.clip(np.floor(centres), 0, 255).astype(np.int64)
    basis = rng.integers(-48, 49, size=(N_LATENT, d)).astype(np.int64)
    basis *= rng.random((N_LATENT, d)) < 0.5
    wts = 1.0 / (np.arange(N_CLUSTERS) + 10.0) ** 0.9      # Zipf-like: skewed bin occupancy
    cdf = np.cumsum(wts / wts.sum())
    thresholds = np.minimum(np.floor(cdf * 2.0 ** 32), 2.0 ** 32 - 1).astype(np.uint64)
    thresholds[-1] = np.uint64(0xFFFFFFFF)
    return {"centres": centres, "basis": basis, "thresholds": thresholds}


def sift_like(start, count, d=128, seed=0, tables=None, chunk=65536):
    """Vectors start..start+count-1 of the SIFT-shaped stream `seed`: fp32 array
    (count, d) of integers in 0..255.

    x[id][j] = clip( (centre[c][j]*gain >> 7) + sum_f (z_f*basis[f][j] >> 8) + noise[id][j], 0, 255 )
    with cluster c, gain in [104,168), 24 latents z_f (triangular in -255..255) and
    noise (triangular in -15..15) all integer hashes of (seed, id, lane).  The latent
    spread makes the nearest-neighbour distance about 0.4 of the distance between
    random pairs, as in SIFT descriptors, so bins are filled far more evenly than a
    tight mixture would fill them."""
    if tables is None:
        tables = sift_like_tables(d)
    centres, basis, thr = tables["centres"], tables["basis"], tables["thresholds"]
    out = np.empty((count, d), dtype=np.float32)
    dims = np.arange(d, dtype=np.uint64)[None, :]
    for c0 in range(0, count, chunk):
        n = min(chunk, count - c0)
        ids = np.arange(start + c0, start + c0 + n, dtype=np.uint64)
        cl = np.searchsorted(thr, _stream(seed, ids, 0), side="left")
        cl = np.minimum(cl, N_CLUSTERS - 1)
        gain = (104 + (_stream(seed, ids, 1) & np.uint64(63))).astype(np.int64)
        x = (centres[cl] * gain[:, None]) >> 7
        for f in range(N_LATENT):
            h = _stream(seed, ids, 2 + f)
            z = ((h & np.uint64(0xFF)) + ((h >> np.uint64(8)) & np.uint64(0xFF))).astype(np.int64) - 255
            x += (z[:, None] * basis[f][None, :]) >> 8
        h = _stream(seed, ids[:, None], 64 + dims)
        noise = ((h & np.uint64(31)).astype(np.int64) - ((h >> np.uint64(5)) & np.uint64(31)).astype(np.int64)) >> 1
        x += noise
        out[c0:c0 + n] = np.clip(x, 0, 255)
    return out


# --------------------------------------------------------------------------
# GIST-shaped: fp32 in [0,1], clustered, unit L2 norm
# --------------------------------------------------------------------------
def gist_like(start, count, d=960, seed=0, table_seed=0, chunk=16384):
    """Vectors start..start+count-1 of the GIST-shaped stream: values in [0,1] from a
    1000-cluster mixture with an 8-dimensional latent offset and small isotropic noise,
    each vector scaled to unit L2 norm.  Generated in fixed chunks of `chunk` ids with a
    per-chunk seed, so any aligned range is reproducible (CPU only)."""
    trng = np.random.default_rng([table_seed, 0x6157, d])
    centres = trng.random((N_CLUSTERS, d)) * (trng.random((N_CLUSTERS, d)) < 0.7)
    basis = trng.standard_normal((N_LATENT, d)) * 0.08
    wts = 1.0 / (np.arange(N_CLUSTERS) + 10.0) ** 0.9
    cdf = np.cumsum(wts / wts.sum())
    out = np.empty((count, d), dtype=np.float32)
    first = start // chunk
    last = (start + count - 1) // chunk if count > 0 else first - 1
    for ci in range(first, last + 1):
        rng = np.random.default_rng([seed, 0x6157DA7A, ci])
        cl = np.minimum(np.searchsorted(cdf, rng.random(chunk)), N_CLUSTERS - 1)
        z = rng.standard_normal((chunk, N_LATENT))
        x = centres[cl] + z @ basis + 0.02 * rng.standard_normal((chunk, d))
        np.clip(x, 0.0, 1.0, out=x)
        x /= np.maximum(np.linalg.norm(x, axis=1, keepdims=True), 1e-12)
        lo = max(start, ci * chunk)
        hi = min(start + count, (ci + 1) * chunk)
        out[lo - start:hi - start] = x[lo - ci * chunk:hi - ci * chunk]
    return out


# --------------------------------------------------------------------------
# small-integer vectors: every squared norm and dot product stays far below 2**24,
# so any fp32 evaluation order of a squared distance is exact
# --------------------------------------------------------------------------
def small_integer_vectors(n, d, lo=0, hi=8, seed=0, clusters=0):
    """n fp32 vectors of integers in [lo, hi).  With clusters>0 the vectors are
    integer cluster centres plus integer noise in {-1,0,1}, clipped to [lo, hi)."""
    rng = np.random.default_rng([seed, 0x1D7])
    if clusters <= 0:
        x = rng.integers(lo, hi, size=(n, d))
    else:
        crng = np.random.default_rng([0x1D7C, d, clusters, lo, hi])
        cen = crng.integers(lo, hi, size=(clusters, d))
        x = cen[rng.integers(0, clusters, size=n)] + rng.integers(-1, 2, size=(n, d))
        x = np.clip(x, lo, hi - 1)
    return np.ascontiguousarray(x, dtype=np.float32)


# --------------------------------------------------------------------------
# the same SIFT-shaped stream computed with torch integer ops (any device)
# --------------------------------------------------------------------------
def sift_like_torch(start, count, d=128, seed=0, tables=None, device="cpu", chunk=1 << 20):
    """Bit-identical to sift_like(): int64 tensors hold the 32-bit hash state (products wrap
    modulo 2**64, the low 32 bits are what the uint64 NumPy version keeps)."""
    import torch
    if tables is None:
        tables = sift_like_tables(d)
    dev = torch.device(device)
    centres = torch.from_numpy(tables["centres"]).to(dev)
    basis = torch.from_numpy(tables["basis"]).to(dev)
    thr = torch.from_numpy(tables["thresholds"].astype(np.int64)).to(dev)
    mask = 0xFFFFFFFF

    def mix32(x):
        x = x & mask
        x = x ^ (x >> 16)
        x = (x * 0x7FEB352D) & mask
        x = x ^ (x >> 15)
        x = (x * 0x846CA68B) & mask
        x = x ^ (x >> 16)
        return x

    s = (int(seed) * 0x9E3779B1 + 0x7F4A7C15) & mask

    def stream(ids, lane):
        h = mix32(ids ^ s)
        h = mix32(h + (ids >> 32) * 0x85EBCA6B + 0x165667B1)
        return mix32(h ^ ((lane * 0x9E3779B1) & mask))

    out = torch.empty((count, d), dtype=torch.float32, device=dev)
    dims = torch.arange(d, dtype=torch.int64, device=dev)[None, :]
    for c0 in range(0, count, chunk):
        n = min(chunk, count - c0)
        ids = torch.arange(start + c0, start + c0 + n, dtype=torch.int64, device=dev)
        zero = torch.zeros((), dtype=torch.int64, device=dev)
        cl = torch.searchsorted(thr, stream(ids, zero), right=False).clamp_(max=N_CLUSTERS - 1)
        gain = 104 + (stream(ids, zero + 1) & 63)
        x = (centres[cl] * gain[:, None]) >> 7
        for f in range(N_LATENT):
            h = stream(ids, zero + 2 + f)
            z = (h & 0xFF) + ((h >> 8) & 0xFF) - 255
            x += (z[:, None] * basis[f][None, :]) >> 8
        h = stream(ids[:, None], 64 + dims)
        x += ((h & 31) - ((h >> 5) & 31)) >> 1
        out[c0:c0 + n] = x.clamp_(0, 255).to(torch.float32)
    return out


def gist_like_torch(start, count, d=960, seed=0, table_seed=0, device="cpu", chunk=65536):
    """The GIST-shaped recipe of gist_like() drawn with torch's generator on `device` (same
    cluster centres, latent basis and weights; the per-chunk random streams are torch's, so the
    values differ from the NumPy version and are reproducible per device type).  Any range is
    assembled from fixed chunks of `chunk` ids, each with its own seed."""
    import torch
    dev = torch.device(device)
    trng = np.random.default_rng([table_seed, 0x6157, d])
    centres = trng.random((N_CLUSTERS, d)) * (trng.random((N_CLUSTERS, d)) < 0.7)
    basis = trng.standard_normal((N_LATENT, d)) * 0.08
    wts = 1.0 / (np.arange(N_CLUSTERS) + 10.0) ** 0.9
    cdf = torch.from_numpy(np.cumsum(wts / wts.sum())).to(dev)
    centres = torch.from_numpy(centres.astype(np.float32)).to(dev)
    basis = torch.from_numpy(basis.astype(np.float32)).to(dev)
    out = torch.empty((count, d), dtype=torch.float32, device=dev)
    first = start // chunk
    last = (start + count - 1) // chunk if count > 0 else first - 1
    gen = torch.Generator(device=dev)
    for ci in range(first, last + 1):
        gen.manual_seed((int(seed) * 0x9E3779B1 + ci * 0x85EBCA6B + 0x6157DA7A) & 0x7FFFFFFFFFFFFFFF)
        u = torch.rand(chunk, generator=gen, device=dev, dtype=torch.float64)
        cl = torch.searchsorted(cdf, u).clamp_(max=N_CLUSTERS - 1)
        z = torch.randn((chunk, N_LATENT), generator=gen, device=dev)
        x = centres[cl] + z @ basis + 0.02 * torch.randn((chunk, d), generator=gen, device=dev)
        x.clamp_(0.0, 1.0)
        x /= x.norm(dim=1, keepdim=True).clamp_min(1e-12)
        lo = max(start, ci * chunk)
        hi = min(start + count, (ci + 1) * chunk)
        out[lo - start:hi - start] = x[lo - ci * chunk:hi - ci * chunk]
    return out
