"""Philox4x32-10 with Python integers: a second, independent writing of the
generator that oracle/zo_oracle_rng.c implements in C.

TEST INFRASTRUCTURE ONLY.  It exists so that the C generator can be pinned
against something other than itself: both must reproduce the known-answer
vectors published with the generator (Salmon et al., SC'11) and agree with each
other on the (seed, tensor id, element) counter layout used for the random
direction z of the ZO-SGD step (DistZO2, Preliminaries Eq. 1-2; App. A Alg. 1:
the generator is re-seeded so that all passes of a step draw the same z).
"""

MASK = 0xFFFFFFFF
MUL_A, MUL_B = 0xD2511F53, 0xCD9E8D57      # multipliers for counter words 0 and 2
WEYL_A, WEYL_B = 0x9E3779B9, 0xBB67AE85    # per-round key increments


def philox4x32(counter, key, rounds=10):
    c = [int(x) & MASK for x in counter]
    k = [int(x) & MASK for x in key]
    for rnd in range(rounds):
        prod_a = MUL_A * c[0]
        prod_b = MUL_B * c[2]
        c = [
            ((prod_b >> 32) ^ c[1] ^ k[0]) & MASK,
            prod_b & MASK,
            ((prod_a >> 32) ^ c[3] ^ k[1]) & MASK,
            prod_a & MASK,
        ]
        k = [(k[0] + WEYL_A) & MASK, (k[1] + WEYL_B) & MASK]
    return tuple(c)


def words_for(seed, tensor_id, block_index, stream_tag=0):
    """The four 32-bit words that serve elements 4*block_index .. 4*block_index+3."""
    counter = (block_index & MASK, (block_index >> 32) & MASK, tensor_id, stream_tag)
    key = (seed & MASK, (seed >> 32) & MASK)
    return philox4x32(counter, key)
