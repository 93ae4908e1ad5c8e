"""Counter-based seeded random numbers for the synthetic workloads.

Every tensor the workloads need (images, weights, normalisation statistics)
is a pure function of (seed, stream ids, element index), so any subset can be
regenerated in any order.  Definition (all arithmetic modulo 2**64):

    mix(z):   z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9
              z = (z ^ (z >> 27)) * 0x94D049BB133111EB
              return z ^ (z >> 31)                      (SplitMix64 finaliser)
    key(seed, a, b, c) = mix(mix(mix(mix(seed) + a) + b) + c)
    bits(key, i)       = mix(key + (i + 1) * 0x9E3779B97F4A7C15)
    uniform(key, i)    = ((bits >> 11) + 0.5) * 2**-53          in (0, 1)
    normal(key, i)     = sqrt(-2 ln uniform(key, 2i)) * cos(2 pi uniform(key, 2i+1))

This module holds no arithmetic of the ensemble method itself; it only makes
inputs that both the CPU oracle and the GPU library are fed.
"""
import numpy as np

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)

KIND_IMAGE = 1
KIND_WEIGHT = 2
KIND_BIAS = 3
KIND_BN_MEAN = 4
KIND_BN_VAR = 5


def mix(z):
    z = np.asarray(z, dtype=np.uint64)
    with np.errstate(over="ignore"):
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        return z ^ (z >> np.uint64(31))


def stream_key(seed, a, b, c):
    with np.errstate(over="ignore"):
        k = mix(np.uint64(seed & 0xFFFFFFFFFFFFFFFF))
        k = mix(k + np.uint64(a))
        k = mix(k + np.uint64(b))
        k = mix(k + np.uint64(c))
    return np.uint64(k)


def bits(key, idx):
    idx = np.asarray(idx, dtype=np.uint64)
    with np.errstate(over="ignore"):
        return mix(np.uint64(key) + (idx + np.uint64(1)) * _GOLDEN)


def uniform(key, idx):
    b = bits(key, idx)
    return ((b >> np.uint64(11)).astype(np.float64) + 0.5) * (2.0 ** -53)


def normal(key, count, start=0):
    """`count` standard normals, elements start .. start+count-1 of the stream."""
    i = np.arange(start, start + count, dtype=np.uint64)
    u1 = uniform(key, i * np.uint64(2))
    u2 = uniform(key, i * np.uint64(2) + np.uint64(1))
    return np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)


def uniform_range(key, count, lo, hi, start=0):
    i = np.arange(start, start + count, dtype=np.uint64)
    return lo + (hi - lo) * uniform(key, i)
