"""Counter-based random numbers for the stochastic choices of the method.

The paper draws the bonus token t ~ p' (Algorithm 1, last lines) and the beams of
stochastic beam sampling (Section 2.1, Eq. 2) without saying how.  Reading used here: a
keyed hash of (seed, stream, absolute token position, index) gives a uniform number per
candidate; a draw from a categorical distribution is argmax(log-weight + Gumbel noise),
which does not depend on the order candidates are visited in.

Hash: the 64-bit finaliser of SplitMix64 (Steele, Lea, Flood 2014).
"""
import numpy as np

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)

STREAM_BONUS = 0   # bonus token drawn from the target row
STREAM_BEAM = 1    # stochastic beam sampling on the draft model
STREAM_ACCEPT = 2  # token-wise accept draws of vanilla speculative decoding
STREAMS_PER_SEQ = 4


def mix64(z):
    with np.errstate(over="ignore"):
        z = np.asarray(z, dtype=np.uint64)
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        return z ^ (z >> np.uint64(31))


def stream_id(seq_index: int, kind: int) -> int:
    return seq_index * STREAMS_PER_SEQ + kind


def hash_u64(seed: int, stream: int, position: int, idx):
    """64-bit hash per candidate index (idx may be an array)."""
    with np.errstate(over="ignore"):
        k0 = mix64(np.uint64(seed) ^ (_GOLDEN * np.uint64(stream + 1)))
        k1 = mix64(k0 + np.uint64(position))
        return mix64(k1 ^ (_GOLDEN * (np.asarray(idx, dtype=np.uint64) + np.uint64(1))))


def uniform(seed: int, stream: int, position: int, idx):
    """Uniform in (0, 1): the top 23 bits of the hash, centred: (k + 1/2) / 2^23.
    Every value is exactly representable in float32."""
    k = hash_u64(seed, stream, position, idx) >> np.uint64(41)
    return (k.astype(np.float64) + 0.5) * (2.0 ** -23)


def gumbel(seed: int, stream: int, position: int, idx):
    """Standard Gumbel noise g = -log(-log(u))."""
    u = uniform(seed, stream, position, idx)
    return -np.log(-np.log(u))
