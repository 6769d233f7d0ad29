"""Philox4x32-10 counter-based random number generator.

Definition: J. Salmon, M. Moraes, R. Dror, D. Shaw, "Parallel random numbers:
as easy as 1, 2, 3", SC'11, Sec. 3.3 (Philox) with the 4x32 constants of
their Table 2 and ten rounds.  The paper under test does not fix a generator;
this one is the reading taken for the Bernoulli(p) and cut-point draws of
Sec. 3.1 and Sec. 4.

Test infrastructure: not used by the product path.
"""
import numpy as np

MASK32 = 0xFFFFFFFF
MUL_A = 0xD2511F53   # multiplier applied to counter word 0
MUL_B = 0xCD9E8D57   # multiplier applied to counter word 2
WEYL_A = 0x9E3779B9  # key word 0 increment per round (golden ratio)
WEYL_B = 0xBB67AE85  # key word 1 increment per round (sqrt(3)-1)
ROUNDS = 10


def philox4x32_10(counter, key):
    """One 128-bit block.  counter: 4 ints < 2**32, key: 2 ints < 2**32.

    Pure Python integers, one round per loop iteration: the S-box multiplies
    words 0 and 2 into 64-bit products, and the permutation places
    (hi(B)^c1^k0, lo(B), hi(A)^c3^k1, lo(A)).
    """
    c0, c1, c2, c3 = (int(x) & MASK32 for x in counter)
    k0, k1 = (int(x) & MASK32 for x in key)
    for rnd in range(ROUNDS):
        if rnd > 0:
            k0 = (k0 + WEYL_A) & MASK32
            k1 = (k1 + WEYL_B) & MASK32
        prod_a = MUL_A * c0
        prod_b = MUL_B * c2
        c0, c1, c2, c3 = ((prod_b >> 32) ^ c1 ^ k0,
                          prod_b & MASK32,
                          (prod_a >> 32) ^ c3 ^ k1,
                          prod_a & MASK32)
    return (c0, c1, c2, c3)


def philox4x32_10_array(c0, c1, c2, c3, k0, k1):
    """Vectorised form of philox4x32_10 over numpy arrays (broadcast).

    All arithmetic is in uint64 so the 32x32->64 products are exact.
    Returns a tuple of four uint32 arrays.
    """
    c0, c1, c2, c3 = np.broadcast_arrays(*(np.asarray(x, dtype=np.uint64) & np.uint64(MASK32)
                                           for x in (c0, c1, c2, c3)))
    k0 = np.uint64(int(k0) & MASK32)
    k1 = np.uint64(int(k1) & MASK32)
    m32 = np.uint64(MASK32)
    sh = np.uint64(32)
    for rnd in range(ROUNDS):
        if rnd > 0:
            k0 = (k0 + np.uint64(WEYL_A)) & m32
            k1 = (k1 + np.uint64(WEYL_B)) & m32
        prod_a = np.uint64(MUL_A) * c0
        prod_b = np.uint64(MUL_B) * c2
        c0, c1, c2, c3 = ((prod_b >> sh) ^ c1 ^ k0,
                          prod_b & m32,
                          (prod_a >> sh) ^ c3 ^ k1,
                          prod_a & m32)
    return tuple(x.astype(np.uint32) for x in (c0, c1, c2, c3))
