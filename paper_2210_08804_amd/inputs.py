"""Seeded synthetic inputs: key streams and the backing-store row generator.

This module serves the tests' CPU side and the GPU side alike.  It holds none of the cache's
own arithmetic (no set mapping, no probing, no replacement): only how keys are drawn and what
row a lower storage tier would return for a key.

The key streams stand in for the paper's click-through workloads (Sec. 7.1: 26 categorical
features per sample, rows of 128 fp32, key popularity close to a power law, Sec. 2.2); none
of those datasets is reproduced here.
"""
import numpy as np

_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_GOLDEN = np.uint64(0x9E3779B97F4A7C15)


def _mix(x: np.ndarray) -> np.ndarray:
    """64-bit finaliser of splitmix64 on a uint64 array (wrapping arithmetic)."""
    x = x ^ (x >> np.uint64(30))
    x = x * _M1
    x = x ^ (x >> np.uint64(27))
    x = x * _M2
    x = x ^ (x >> np.uint64(31))
    return x


def backing_rows(keys, dim: int, version: int = 0) -> np.ndarray:
    """Row a lower tier returns for each key: float32 [n, dim], element j of key k is

        z = mix(k XOR mix(((version << 32) | j) + GOLDEN));  value = (int(z >> 40) - 2^23) * 2^-23

    i.e. a 24-bit integer scaled by a power of two: exactly representable, in [-1, 1).
    `version` may be a scalar or an array of one version per key.
    """
    keys = np.ascontiguousarray(keys, dtype=np.int64).view(np.uint64)
    n = keys.shape[0]
    ver = np.broadcast_to(np.asarray(version, dtype=np.uint64), (n,))
    j = np.arange(dim, dtype=np.uint64)
    with np.errstate(over="ignore"):
        inner = _mix(((ver[:, None] << np.uint64(32)) | j[None, :]) + _GOLDEN)
        z = _mix(keys[:, None] ^ inner)
    q = (z >> np.uint64(40)).astype(np.int64) - (1 << 23)
    return (q.astype(np.float32) * np.float32(2.0 ** -23)).astype(np.float32)


def uniform_keys(n: int, key_space: int, seed: int) -> np.ndarray:
    """n int64 keys uniform over [0, key_space)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    return rng.integers(0, key_space, size=n, dtype=np.int64)


def zipf_keys(n: int, key_space: int, alpha: float, seed: int) -> np.ndarray:
    """n int64 keys with rank r in [1, key_space] drawn with p(r) roughly proportional to
    r^-alpha (inverse CDF of the continuous power law on [1, key_space], floored); key = r - 1,
    so the hottest key is 0.  Positions are in draw order, i.e. already shuffled.
    """
    if alpha == 1.0:
        raise ValueError("alpha must differ from 1")
    rng = np.random.Generator(np.random.PCG64(seed))
    u = rng.random(n)
    a = 1.0 - alpha
    r = np.floor((1.0 + u * (float(key_space) ** a - 1.0)) ** (1.0 / a))
    r = np.clip(r, 1.0, float(key_space)).astype(np.int64)
    return r - 1


def log_uniform_vocab(n_tables: int, lo: float, hi: float, seed: int) -> np.ndarray:
    """Vocabulary sizes of n_tables tables, log-uniform over [lo, hi]."""
    rng = np.random.Generator(np.random.PCG64(seed))
    e = rng.uniform(np.log(lo), np.log(hi), size=n_tables)
    return np.clip(np.round(np.exp(e)), lo, hi).astype(np.int64)
