"""Second, independent statement of the build's mask rule in pure Python integers.

Written from the mathematical definition of Philox4x32-10 (Salmon, Moraes, Dror, Shaw,
SC'11) with arbitrary-precision ints; shares nothing with oracle/ or the GPU code.
Used to extend the reach of the known-answer vectors to the counter/key mapping.
"""
MASK32 = (1 << 32) - 1


def philox4x32_10(ctr, key):
    c = [int(v) & MASK32 for v in ctr]
    k = [int(v) & MASK32 for v in key]
    for _ in range(10):
        prod_a = 0xD2511F53 * c[0]
        prod_b = 0xCD9E8D57 * c[2]
        c = [((prod_b >> 32) ^ c[1] ^ k[0]) & MASK32, prod_b & MASK32,
             ((prod_a >> 32) ^ c[3] ^ k[1]) & MASK32, prod_a & MASK32]
        k = [(k[0] + 0x9E3779B9) & MASK32, (k[1] + 0xBB67AE85) & MASK32]
    return tuple(c)


def coord_bits(seed, rnd, j):
    blk = j >> 2
    out = philox4x32_10((blk & MASK32, blk >> 32, rnd & MASK32, rnd >> 32), (seed & MASK32, seed >> 32))
    return out[j & 3]


def keep(seed, rnd, j, c):
    """Bernoulli(1/c) decision for integer-valued c."""
    return coord_bits(seed, rnd, j) < (1 << 32) // int(c)
