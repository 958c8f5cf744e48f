"""Counter-based uniforms for the sampling calls (test infrastructure only, like the rest of oracle/).

The method draws at T > 0 (section 2.1: stochastic acceptance and the residual-distribution redraw; the
paper's T = 1 columns of Table 2) but does not say where its random numbers come from.  Reading used
here and by the library: the published Philox4x32-10 counter-based generator (Salmon, Moraes, Dror,
Shaw, "Parallel random numbers: as easy as 1, 2, 3", SC'11), written out from its definition:

  one round on counter (c0, c1, c2, c3) with round key (k0, k1):
      hi0:lo0 = 0xD2511F53 * c0        hi1:lo1 = 0xCD9E8D57 * c2        (32 x 32 -> 64 bit products)
      (c0, c1, c2, c3) <- (hi1 ^ c1 ^ k0,  lo1,  hi0 ^ c3 ^ k1,  lo0)
  ten rounds; before every round but the first the key is bumped by (0x9E3779B9, 0xBB67AE85) mod 2^32.

A uniform is the top 24 bits of output word 0 times 2^-24 (exactly representable in float32, in [0, 1)).
Which counter a draw uses is fixed by `draw_counter`: word 0 = index of the number inside its array,
word 1 = purpose of the array, words 2-3 = the low / high half of the context's count of drawing calls.
"""
import numpy as np

M0, M1 = 0xD2511F53, 0xCD9E8D57
W0, W1 = 0x9E3779B9, 0xBB67AE85
MASK = 0xFFFFFFFF

# purposes (counter word 1)
FIRST_TOKEN, DRAFT, ACCEPT, RESAMPLE, TREE = 0, 1, 2, 3, 4


def philox4x32_10(counter, key):
    """counter: 4 words, key: 2 words (python ints below 2^32).  Returns the 4 output words."""
    c0, c1, c2, c3 = (int(x) & MASK for x in counter)
    k0, k1 = (int(x) & MASK for x in key)
    for rnd in range(10):
        if rnd > 0:
            k0 = (k0 + W0) & MASK
            k1 = (k1 + W1) & MASK
        p0 = M0 * c0
        p1 = M1 * c2
        hi0, lo0 = p0 >> 32, p0 & MASK
        hi1, lo1 = p1 >> 32, p1 & MASK
        c0, c1, c2, c3 = hi1 ^ c1 ^ k0, lo1, hi0 ^ c3 ^ k1, lo0
    return c0, c1, c2, c3


def seed_key(seed):
    """64-bit seed -> the two key words (low half, high half)."""
    seed = int(seed) & 0xFFFFFFFFFFFFFFFF
    return seed & MASK, seed >> 32


def draw_counter(index, purpose, call):
    call = int(call) & 0xFFFFFFFFFFFFFFFF
    return int(index) & MASK, int(purpose) & MASK, call & MASK, call >> 32


def uniform(seed, call, purpose, index):
    """The float32 uniform in [0, 1) that drawing call number `call` of a context seeded with `seed` uses as number
    `index` of the array with the given purpose."""
    word0 = philox4x32_10(draw_counter(index, purpose, call), seed_key(seed))[0]
    return np.float32((word0 >> 8) * 2.0 ** -24)


def uniforms(seed, call, purpose, n):
    return np.array([uniform(seed, call, purpose, i) for i in range(n)], np.float32)
