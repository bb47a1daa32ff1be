"""Counter-based uniforms for the oracle (test infrastructure).

The paper fixes no random number generator; the accept test (Sec. 3.1, Eq. 1)
needs one uniform per draft position and the residual draw (Eq. 2) one more.
This build uses Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random
numbers: as easy as 1, 2, 3", SC'11): a 10-round bijection of a 128-bit
counter under a 64-bit key.  Written here from the published round function,
in numpy, independently of the HIP implementation.

Counter convention of the verification step (word 0 of the output is used):
    key     = (seed & 0xffffffff, seed >> 32)
    counter = (t, b, rng_counter & 0xffffffff,
               (stream << 24) | ((rng_counter >> 32) & 0xffffff))
with t the block-local position, b the batch index, stream 0 for the accept
uniform and 1 for the sampler word.
"""
import numpy as np

_M0 = np.uint64(0xD2511F53)
_M1 = np.uint64(0xCD9E8D57)
_W0 = 0x9E3779B9
_W1 = 0xBB67AE85
_MASK = np.uint64(0xFFFFFFFF)
_S32 = np.uint64(32)

STREAM_ACCEPT = 0
STREAM_SAMPLE = 1
STREAM_SEQUENTIAL = 2   # sequential re-sampling (Alg. 1 Step 6)


def philox4x32(c0, c1, c2, c3, k0, k1, rounds=10):
    """Philox-4x32 with `rounds` rounds on arrays of counters.

    c0..c3: integer arrays (broadcastable), each word < 2**32.
    k0, k1: python ints (key words).  Returns four uint32 arrays.
    One round: (hi0, lo0) = M0 * c0, (hi1, lo1) = M1 * c2 as 64-bit products;
    new counter = (hi1 ^ c1 ^ k0, lo1, hi0 ^ c3 ^ k1, lo0); the key words are
    advanced by the Weyl constants between rounds.
    """
    c0, c1, c2, c3 = np.broadcast_arrays(
        *[np.asarray(c).astype(np.uint64) & _MASK for c in (c0, c1, c2, c3)])
    k0 = int(k0) & 0xFFFFFFFF
    k1 = int(k1) & 0xFFFFFFFF
    for r in range(rounds):
        p0 = _M0 * c0
        p1 = _M1 * c2
        hi0, lo0 = p0 >> _S32, p0 & _MASK
        hi1, lo1 = p1 >> _S32, p1 & _MASK
        c0, c1, c2, c3 = (hi1 ^ c1 ^ np.uint64(k0), lo1,
                          hi0 ^ c3 ^ np.uint64(k1), lo0)
        k0 = (k0 + _W0) & 0xFFFFFFFF
        k1 = (k1 + _W1) & 0xFFFFFFFF
    return tuple(c.astype(np.uint32) for c in (c0, c1, c2, c3))


def step_words(seed, rng_counter, stream, B, L):
    """Word 0 for every (b, t) of a verification step: uint32 [B, L]."""
    t = np.arange(L, dtype=np.uint64)[None, :]
    b = np.arange(B, dtype=np.uint64)[:, None]
    c2 = int(rng_counter) & 0xFFFFFFFF
    c3 = ((int(stream) & 0xFF) << 24) | ((int(rng_counter) >> 32) & 0xFFFFFF)
    w0, _, _, _ = philox4x32(t, b, c2, c3, int(seed) & 0xFFFFFFFF, (int(seed) >> 32) & 0xFFFFFFFF)
    return np.ascontiguousarray(np.broadcast_to(w0, (B, L)))


def uniform24(words):
    """u = (word >> 8) * 2**-24 in [0, 1): exactly representable in float32."""
    return ((np.asarray(words, dtype=np.uint32) >> np.uint32(8)).astype(np.float32)
            * np.float32(2.0 ** -24))
