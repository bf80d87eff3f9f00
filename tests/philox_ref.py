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


def philox4x32_10_np(c0, c1, c2, c3, key):
    """The same generator over numpy arrays of counter words (uint64 arithmetic, masked to 32 bits):
    used to search a whole vocabulary row for equal words.  Returns an array [..., 4] of uint32."""
    import numpy as np
    m = np.uint64(MASK)
    c0 = np.asarray(c0, dtype=np.uint64)
    c1 = np.zeros_like(c0) + np.uint64(c1)
    c2 = np.zeros_like(c0) + np.uint64(c2)
    c3 = np.zeros_like(c0) + np.uint64(c3)
    k0, k1 = np.uint64(int(key[0]) & MASK), np.uint64(int(key[1]) & MASK)
    for _ in range(10):
        prod0 = np.uint64(MULT[0]) * c0
        prod1 = np.uint64(MULT[1]) * c2
        c0, c1, c2, c3 = (((prod1 >> np.uint64(32)) ^ c1 ^ k0) & m, prod1 & m,
                          ((prod0 >> np.uint64(32)) ^ c3 ^ k1) & m, prod0 & m)
        k0, k1 = (k0 + np.uint64(WEYL[0])) & m, (k1 + np.uint64(WEYL[1])) & m
    return np.stack([c0, c1, c2, c3], axis=-1).astype(np.uint32)


def noise_words_of_row(seed, seq, rnd, pos, stream, V):
    """Word of every vocabulary element of one Gumbel draw: counter (v >> 2, pos | stream << 16, round,
    sequence), word v & 3 (stream 1: correction / bonus token, stream 2: drafted token)."""
    import numpy as np
    blocks = np.arange((V + 3) // 4, dtype=np.uint64)
    w = philox4x32_10_np(blocks, pos | (stream << 16), rnd, seq, (seed & MASK, (seed >> 32) & MASK))
    return w.reshape(-1)[:V]


def equal_word_pairs(words):
    """Index pairs (i < j) of a row of noise words that hold the same 32-bit word."""
    import numpy as np
    order = np.argsort(words, kind="stable")
    s = words[order]
    hits = np.flatnonzero(s[1:] == s[:-1])
    return sorted((int(min(order[h], order[h + 1])), int(max(order[h], order[h + 1]))) for h in hits)
