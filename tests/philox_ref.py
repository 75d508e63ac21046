"""Philox4x32-10 written out with Python integers, straight from the description in
Salmon, Moraes, Dror, Shaw, "Parallel random numbers: as easy as 1, 2, 3" (SC'11), Section 3.3 and
the 4x32 parameter table: a test-side check for the oracle's and the library's generators.

One round maps the counter (c0, c1, c2, c3) under round key (k0, k1) to
    (hi(B*c2) ^ c1 ^ k0,  lo(B*c2),  hi(A*c0) ^ c3 ^ k1,  lo(A*c0))
and the round key advances by the Weyl constants between rounds.
"""

MASK = 0xFFFFFFFF
A = 0xD2511F53
B = 0xCD9E8D57
WEYL = (0x9E3779B9, 0xBB67AE85)


def philox4x32_10(ctr, key, rounds=10):
    c0, c1, c2, c3 = (int(x) & MASK for x in ctr)
    k0, k1 = (int(x) & MASK for x in key)
    for r in range(rounds):
        pa = A * c0
        pb = B * c2
        c0, c1, c2, c3 = ((pb >> 32) ^ c1 ^ k0) & MASK, pb & MASK, ((pa >> 32) ^ c3 ^ k1) & MASK, pa & MASK
        k0 = (k0 + WEYL[0]) & MASK
        k1 = (k1 + WEYL[1]) & MASK
    return [c0, c1, c2, c3]


def stream_u32(seed, hop_id, word_index, j):
    """j-th 32-bit word of the stream of (seed, hop id, packed-word index)."""
    out = philox4x32_10([j >> 2, hop_id, word_index & MASK, word_index >> 32],
                        [seed & MASK, (seed >> 32) & MASK])
    return out[j & 3]
