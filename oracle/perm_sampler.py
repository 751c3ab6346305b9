"""Oracle of the on-device permutation sampler (test infrastructure only; numpy, no code shared with
the HIP library).

Sec. 3.3: sigma ~ Uniform(S_n), sampled independently per layer (and, when asked, per head and batch
element).  The sampler is "sort by random key": slot p of slice (pb, ph) of layer `layer` gets the
64-bit key

    stream = mix(mix(seed) + GAMMA * ((layer << 32) | slice)),   slice = pb * perm_H + ph
    r(p)   = mix(stream + GAMMA * (p + 1))

i.e. the (p+1)-th output of the SplitMix64 generator (Steele, Lea, Flood 2014) started at `stream`.
The sort key is r(p) with its low 20 bits replaced by p (n <= 2^20): 44 i.i.d. uniform bits, ties
broken by the slot index, all keys distinct.  perm = the argsort of the keys: perm[k] = the p whose
key has rank k.  The result is uniform over S_n up to collisions of the 44 random bits
(probability < n^2 / 2^45 per slice).
"""
import numpy as np

GAMMA = np.uint64(0x9E3779B97F4A7C15)
_C1 = np.uint64(0xBF58476D1CE4E5B9)
_C2 = np.uint64(0x94D049BB133111EB)


def mix(z):
    """SplitMix64 output function on uint64 (arrays or scalars), arithmetic modulo 2^64."""
    z = np.asarray(z, dtype=np.uint64)
    with np.errstate(over="ignore"):
        z = (z ^ (z >> np.uint64(30))) * _C1
        z = (z ^ (z >> np.uint64(27))) * _C2
    return z ^ (z >> np.uint64(31))


def keys(stream, n):
    with np.errstate(over="ignore"):
        return mix(np.uint64(stream) + GAMMA * np.arange(1, n + 1, dtype=np.uint64))


INDEX_MASK = np.uint64(0xFFFFF)


def sort_keys(stream, n):
    assert n <= 1 << 20
    return (keys(stream, n) & ~INDEX_MASK) | np.arange(n, dtype=np.uint64)


def stream_of(seed, layer, slice_index):
    with np.errstate(over="ignore"):
        tag = np.uint64((int(layer) << 32) | int(slice_index))
        return mix(mix(np.uint64(seed)) + GAMMA * tag)


def sample_perm(seed, layer, perm_B, perm_H, n):
    """int32 [perm_B, perm_H, n]; entry p of a slice = original index of the token placed at slot p."""
    out = np.empty((perm_B, perm_H, n), np.int32)
    for pb in range(perm_B):
        for ph in range(perm_H):
            k = sort_keys(stream_of(seed, layer, pb * perm_H + ph), n)
            out[pb, ph] = np.argsort(k).astype(np.int32)
    return out
