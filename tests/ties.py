"""Finite exact ties: pairs of tokens of one race whose generator words coincide.

32-bit words collide within one row of a large vocabulary (about V^2 / 2^33 pairs: 7.6 at V = 256000), and two such
tokens with the same logit have exactly equal scores on every side and at every precision, so they are the case in
which the lowest-index rule decides.  The generator here is a vectorised numpy restatement of Philox4x32 (Salmon et
al. 2011), written for this search only: it shares no code with the library or with the oracle, and
`words_of_context` is checked against the oracle's generator where it is used.
"""
import numpy as np

M0, M1 = np.uint64(0xD2511F53), np.uint64(0xCD9E8D57)
W0, W1 = 0x9E3779B9, 0xBB67AE85
MASK = np.uint64(0xFFFFFFFF)
SHIFT = np.uint64(32)


def words_of_context(V, seed, c1, c2, c3, rounds):
    """Word of every token i < V of the race with counter (i >> 2, c1, c2, c3) and key (seed low, seed high)."""
    n = (V + 3) // 4
    c = [np.arange(n, dtype=np.uint64), np.full(n, c1, dtype=np.uint64), np.full(n, c2, dtype=np.uint64),
         np.full(n, c3, dtype=np.uint64)]
    k0, k1 = seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF
    for r in range(rounds):
        a, b = M0 * c[0], M1 * c[2]           # below 2^64: both factors are below 2^32
        c = [(b >> SHIFT) ^ c[1] ^ np.uint64(k0), b & MASK, (a >> SHIFT) ^ c[3] ^ np.uint64(k1), a & MASK]
        k0, k1 = (k0 + W0) & 0xFFFFFFFF, (k1 + W1) & 0xFFFFFFFF
    return np.stack(c, axis=1).reshape(-1)[:V].astype(np.uint32)


def colliding_pairs(V, seed, c1, c2, c3, rounds):
    """[(i, j)] with i < j and equal words, sorted; words that occur three times give their first two tokens."""
    w = words_of_context(V, seed, c1, c2, c3, rounds)
    order = np.argsort(w, kind="stable")
    same = np.nonzero(w[order][1:] == w[order][:-1])[0]
    pairs = sorted({(int(min(order[t], order[t + 1])), int(max(order[t], order[t + 1]))) for t in same})
    return pairs, w


def find_context_with_pairs(V, rounds, min_pairs=2, c1=0, c2=0, c3=0, seeds=range(64)):
    """The first seed whose race (c1, c2, c3) holds at least `min_pairs` colliding pairs -> (seed, pairs, words)."""
    for seed in seeds:
        pairs, w = colliding_pairs(V, seed, c1, c2, c3, rounds)
        if len(pairs) >= min_pairs:
            return seed, pairs, w
    raise AssertionError("no seed with enough colliding words (expected about V^2 / 2^33 pairs per race)")
