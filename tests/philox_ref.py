"""Pure-Python-integer Philox4x32-10, written from the published algorithm
(Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as 1, 2, 3", SC'11).
Third, independent implementation used to cross-check the C oracle and the HIP kernels."""

MASK = 0xFFFFFFFF
MULT = (0xD2511F53, 0xCD9E8D57)
WEYL = (0x9E3779B9, 0xBB67AE85)


def philox4x32_10(ctr, key):
    c = [int(x) & MASK for x in ctr]
    k = [int(x) & MASK for x in key]
    for rnd in range(10):
        prod0 = MULT[0] * c[0]
        prod1 = MULT[1] * c[2]
        c = [((prod1 >> 32) ^ c[1] ^ k[0]) & MASK, prod1 & MASK,
             ((prod0 >> 32) ^ c[3] ^ k[1]) & MASK, prod0 & MASK]
        k = [(k[0] + WEYL[0]) & MASK, (k[1] + WEYL[1]) & MASK]
    return c


def accept_words(seed, seq, rnd, pos):
    out = philox4x32_10([0, pos, rnd, seq], [seed & MASK, (seed >> 32) & MASK])
    return out[0], out[1]


def gumbel_word(seed, seq, rnd, pos, v):
    out = philox4x32_10([v >> 2, pos | (1 << 16), rnd, seq], [seed & MASK, (seed >> 32) & MASK])
    return out[v & 3]
