"""Counter-based Philox generators (test infrastructure: CPU oracle side).

This file belongs to the slow, plain CPU oracle.  It is test infrastructure:
only tests, the smoke check and the CPU-baseline leg of the benchmark may use
it; the HIP product path has its own, independently written generator and
shares no code with this one.

The generator is Philox-4xW-R of Salmon, Moraes, Dror and Shaw, "Parallel
random numbers: as easy as 1, 2, 3" (SC'11): a 4-word counter and a 2-word key
go through R rounds; each round multiplies counter words 0 and 2 by two fixed
odd multipliers, keeps high and low halves of the products, XORs the high
halves with the other counter words and the round key, and permutes; the key
is bumped by two Weyl constants between rounds.  The constants are the
published ones.

Two implementations live here on purpose:

* ``philox4_generic`` - plain Python integers, any word width W in {32, 64}.
  Instantiated at W=64 it is pinned against NumPy's own Philox bit generator
  (an independent implementation of Philox-4x64-10), which fixes the round
  structure, the key schedule and the word order.  Instantiated at W=32 it is
  pinned against the known-answer vectors distributed with the authors'
  reference implementation (tests/golden/philox4x32_10_kat.txt).
* ``philox4x32_10`` - a NumPy-vectorised W=32 version used by the oracle for
  speed, pinned against the generic one.

The paper whose method the oracle implements says nothing about random number
generation; the counter layout used for speculative-sampling uniforms
(``sv_uniforms``) is this repository's convention.
"""
from __future__ import annotations

import numpy as np

# Published constants (Salmon et al. 2011).
_CONST = {
    32: dict(M0=0xD2511F53, M1=0xCD9E8D57, W0=0x9E3779B9, W1=0xBB67AE85),
    64: dict(M0=0xD2E7470EE14C6C93, M1=0xCA5A826395121157,
             W0=0x9E3779B97F4A7C15, W1=0xBB67AE8584CAA73B),
}


def philox4_generic(counter, key, width=32, rounds=10):
    """Philox-4xW-R on Python integers.

    counter: 4 ints, key: 2 ints, each < 2**width.  Returns 4 ints.
    """
    k = _CONST[width]
    mask = (1 << width) - 1
    c0, c1, c2, c3 = (int(c) & mask for c in counter)
    k0, k1 = (int(x) & mask for x in key)
    for r in range(rounds):
        if r > 0:
            k0 = (k0 + k["W0"]) & mask
            k1 = (k1 + k["W1"]) & mask
        p0 = k["M0"] * c0
        p1 = k["M1"] * c2
        hi0, lo0 = p0 >> width, p0 & mask
        hi1, lo1 = p1 >> width, p1 & mask
        c0, c1, c2, c3 = (hi1 ^ c1 ^ k0) & mask, lo1, (hi0 ^ c3 ^ k1) & mask, lo0
    return c0, c1, c2, c3


def philox4x32_10(c0, c1, c2, c3, k0, k1):
    """Vectorised Philox-4x32-10.

    All arguments broadcast against each other; they are taken modulo 2**32.
    Returns four uint32 arrays (output words 0..3).
    """
    m32 = np.uint64(0xFFFFFFFF)
    sh = np.uint64(32)
    c0, c1, c2, c3, k0, k1 = np.broadcast_arrays(
        *[np.asarray(a).astype(np.uint64) & m32 for a in (c0, c1, c2, c3, k0, k1)])
    M0 = np.uint64(_CONST[32]["M0"])
    M1 = np.uint64(_CONST[32]["M1"])
    W0 = np.uint64(_CONST[32]["W0"])
    W1 = np.uint64(_CONST[32]["W1"])
    for r in range(10):
        if r > 0:
            k0 = (k0 + W0) & m32
            k1 = (k1 + W1) & m32
        p0 = M0 * c0          # < 2**64, no overflow: both factors < 2**32
        p1 = M1 * c2
        hi0, lo0 = p0 >> sh, p0 & m32
        hi1, lo1 = p1 >> sh, p1 & m32
        c0, c1, c2, c3 = hi1 ^ c1 ^ k0, lo1, hi0 ^ c3 ^ k1, lo0
    return tuple(a.astype(np.uint32) for a in (c0, c1, c2, c3))


def u32_to_unit(w):
    """Map a 32-bit word to the open interval (0,1): ((w >> 8) + 1/2) * 2**-24.

    With n = w >> 8 < 2**24 the value (2n + 1) * 2**-25 has up to 25
    significant bits: exact in float64, not always in float32.  Both sides of
    the parity check therefore carry uniforms in float64.
    """
    n = (np.asarray(w).astype(np.uint64) >> np.uint64(8)).astype(np.float64)
    return (n + 0.5) * (2.0 ** -24)


def sv_uniforms(seed, step, b, i, stream=0):
    """Uniforms for sequence b, position i of decode step `step`.

    Counter = (i, b, stream, step), key = (seed low 32 bits, seed high 32
    bits).  Output word 0 -> accept uniform u, word 1 -> sampling uniform u'.
    Because uniforms are addressed, never consumed in sequence, positions that
    are not verified simply leave their counters unused.
    Returns (u, u_prime) as float64 arrays broadcast over b and i.
    """
    seed = int(seed)
    w = philox4x32_10(i, b, stream, step, seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF)
    return u32_to_unit(w[0]), u32_to_unit(w[1])
