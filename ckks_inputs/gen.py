"""Seeded random draws: residues, secrets, errors, slot values, rotation steps.

All randomness comes from numpy's Philox counter-based generator keyed by an explicit
seed, so the same call returns the same array on every machine.
"""
import numpy as np


def _rng(seed):
    return np.random.Generator(np.random.Philox(key=int(seed) & 0xFFFFFFFFFFFFFFFF))


def uniform_residues(seed, moduli, shape_prefix, N):
    """uint64 array shape_prefix + (len(moduli), N); limb i uniform in [0, moduli[i])."""
    rng = _rng(seed)
    out = np.empty(tuple(shape_prefix) + (len(moduli), N), dtype=np.uint64)
    for i, m in enumerate(moduli):
        out[..., i, :] = rng.integers(0, m, size=tuple(shape_prefix) + (N,), dtype=np.uint64)
    return out


def ternary_secret(seed, N, hamming_weight):
    """int64[N] with exactly `hamming_weight` entries in {-1,+1} (equiprobable), rest 0."""
    rng = _rng(seed)
    s = np.zeros(N, dtype=np.int64)
    pos = rng.choice(N, size=hamming_weight, replace=False)
    s[pos] = rng.integers(0, 2, size=hamming_weight) * 2 - 1
    return s


def gaussian_error(seed, shape, sigma=3.2):
    """int64 rounded N(0, sigma^2), clipped at 6 sigma."""
    rng = _rng(seed)
    e = np.rint(rng.normal(0.0, sigma, size=shape))
    lim = np.floor(6 * sigma)
    return np.clip(e, -lim, lim).astype(np.int64)


def uniform_slots(seed, nslots, lo=-1.0, hi=1.0):
    return _rng(seed).uniform(lo, hi, size=nslots)


def normal_slots(seed, nslots, scale=1.0):
    return _rng(seed).normal(0.0, 1.0, size=nslots) * scale


def seeded_rotation_steps(seed, count, lo, hi):
    """`count` rotation steps uniform in [lo, hi]."""
    return [int(x) for x in _rng(seed).integers(lo, hi + 1, size=count)]


def galois_element(step, logN):
    """Galois element 5^step mod 2N for a left rotation of the slot vector by `step`."""
    return pow(5, int(step), 2 << logN)
