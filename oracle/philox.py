"""Philox4x32-10 counter-based generator (Salmon, Moraes, Dror, Shaw, SC'11), numpy.

TEST INFRASTRUCTURE (part of the CPU oracle; shares no code with the HIP path).

The paper's Algorithm 2 draws u_m ~ Uniform(0,1) for every accept test and samples draft and
residual tokens; it does not say how.  So that the oracle and the GPU path take the *same*
random decisions, both implement this published generator independently and key it the same
way:

    key     = (seed low 32 bits, seed high 32 bits)
    counter = (position, step, sequence, stream)

and use output word 0 only.  ``stream`` separates the draws of a speculative round:
0 = draft-token sample, 1 = accept-test uniform, 2 = residual sample, 3 = re-corruption of a
low-confidence position (Algorithm 2, "Re-corrupt").

A 32-bit word w becomes the uniform  u = ((w >> 9) + 1/2) * 2**-23 : 2**23 equally spaced
values strictly inside (0,1), each exactly representable in fp32 as well as fp64 (odd
integer below 2**24 times 2**-24), so both sides compare against the identical number.

Pinned in tests against the generator's published known-answer vectors.
"""
import numpy as np

_M0 = np.uint64(0xD2511F53)
_M1 = np.uint64(0xCD9E8D57)
_W0 = np.uint32(0x9E3779B9)
_W1 = np.uint32(0xBB67AE85)
_MASK32 = np.uint64(0xFFFFFFFF)
_SHIFT32 = np.uint64(32)

STREAM_DRAFT = 0
STREAM_ACCEPT = 1
STREAM_RESIDUAL = 2
STREAM_RECORRUPT = 3


def philox4x32_10(counter, key):
    """Ten Philox rounds.

    counter: integer array [..., 4]; key: integer array [..., 2] (broadcastable).
    Returns uint32 array [..., 4].
    """
    counter = np.asarray(counter, dtype=np.uint64) & _MASK32
    key = np.asarray(key, dtype=np.uint64) & _MASK32
    shape = np.broadcast_shapes(counter.shape[:-1], key.shape[:-1])
    c0, c1, c2, c3 = (np.broadcast_to(counter[..., i], shape).copy() for i in range(4))
    k0 = np.broadcast_to(key[..., 0], shape).astype(np.uint32)
    k1 = np.broadcast_to(key[..., 1], shape).astype(np.uint32)
    for rnd in range(10):
        if rnd > 0:
            with np.errstate(over="ignore"):
                k0 = (k0 + _W0).astype(np.uint32)
                k1 = (k1 + _W1).astype(np.uint32)
        p0 = _M0 * c0  # 32x32 -> 64 bit product, no overflow in uint64
        p1 = _M1 * c2
        hi0, lo0 = p0 >> _SHIFT32, p0 & _MASK32
        hi1, lo1 = p1 >> _SHIFT32, p1 & _MASK32
        n0 = hi1 ^ c1 ^ k0.astype(np.uint64)
        n2 = hi0 ^ c3 ^ k1.astype(np.uint64)
        c0, c1, c2, c3 = n0, lo1, n2, lo0
    return np.stack([c0, c1, c2, c3], axis=-1).astype(np.uint32)


def word_to_uniform(w):
    """Top 23 bits of a 32-bit word -> u in (0,1), exact in fp32 and fp64."""
    w = np.asarray(w, dtype=np.uint32)
    return ((w >> np.uint32(9)).astype(np.float64) + 0.5) * (2.0 ** -23)


def uniform(seed, position, step, sequence, stream):
    """u(seed; position, step, sequence, stream) with numpy broadcasting over the counter
    fields.  Returns float64."""
    seed = int(seed) & 0xFFFFFFFFFFFFFFFF
    key = np.array([seed & 0xFFFFFFFF, seed >> 32], dtype=np.uint64)
    position, step, sequence, stream = np.broadcast_arrays(
        np.asarray(position, dtype=np.uint64), np.asarray(step, dtype=np.uint64),
        np.asarray(sequence, dtype=np.uint64), np.asarray(stream, dtype=np.uint64))
    ctr = np.stack([position, step, sequence, stream], axis=-1)
    return word_to_uniform(philox4x32_10(ctr, key)[..., 0])
