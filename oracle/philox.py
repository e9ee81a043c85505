"""Philox4x32-10 counter-based generator and the uniform / Gumbel maps.

TEST INFRASTRUCTURE (CPU oracle) -- not part of the product path.

The paper only asks for i.i.d. standard Gumbel noise per (row, vocabulary
entry) (Sec. 3.2.1, Eq. (6); Alg. 4) and for U ~ Uniform[0,1] per verified
draft token (Alg. 6).  To let a parallel GPU kernel and this sequential
oracle draw the *same* numbers, randomness is a pure function of position:

    key     = (seed & 0xffffffff, seed >> 32)
    counter = (vocab_index >> 2, node_row, seq, stream_tag | (step << 4))
    word    = output word number (vocab_index & 3) of the Philox block

The generator is Philox4x32 with 10 rounds as published by Salmon, Moraes,
Dror and Shaw, "Parallel random numbers: as easy as 1, 2, 3" (SC'11): per
round two 32x32->64 bit products with the multipliers M0, M1; the high halves
are xored with the neighbouring counter words and the round key; the key is
bumped by the Weyl constants W0, W1 between rounds.

Uniform map:  u = (2*(word >> 9) + 1) * 2**-24   (odd multiples of 2**-24,
strictly inside (0,1), exactly representable in fp32 and fp64).
Gumbel map:   G = -log(-log(u)).
"""
import numpy as np

M0 = 0xD2511F53
M1 = 0xCD9E8D57
W0 = 0x9E3779B9
W1 = 0xBB67AE85
_MASK = np.uint64(0xFFFFFFFF)

# stream tags (low 4 bits of counter word 3)
TAG_DRAFT_GUMBEL = 0   # Gumbel noise of the drafting samplers
TAG_ACCEPT_UNIFORM = 1  # uniform of one accept/reject test
TAG_LAST_GUMBEL = 2    # Gumbel noise of the final-token sample


def philox4x32_10(c0, c1, c2, c3, k0, k1):
    """Ten Philox4x32 rounds.  All arguments broadcastable integer arrays
    holding 32-bit values; returns four uint32 arrays (the output block)."""
    c0, c1, c2, c3, k0, k1 = (np.asarray(a, dtype=np.uint64) & _MASK
                              for a in (c0, c1, c2, c3, k0, k1))
    c0, c1, c2, c3, k0, k1 = np.broadcast_arrays(c0, c1, c2, c3, k0, k1)
    m0 = np.uint64(M0)
    m1 = np.uint64(M1)
    for _ in range(10):
        p0 = m0 * c0            # < 2**64, no overflow
        p1 = m1 * c2
        hi0, lo0 = p0 >> np.uint64(32), p0 & _MASK
        hi1, lo1 = p1 >> np.uint64(32), p1 & _MASK
        c0, c1, c2, c3 = hi1 ^ c1 ^ k0, lo1, hi0 ^ c3 ^ k1, lo0
        k0 = (k0 + np.uint64(W0)) & _MASK
        k1 = (k1 + np.uint64(W1)) & _MASK
    return (c0.astype(np.uint32), c1.astype(np.uint32),
            c2.astype(np.uint32), c3.astype(np.uint32))


def words(seed, step, tag, seq, node_row, vocab_index):
    """32-bit random word for each (seq, node_row, vocab_index) triple
    (broadcast against each other) under (seed, step, tag)."""
    seed = int(seed)
    vi = np.asarray(vocab_index, dtype=np.uint64)
    c3 = (int(tag) & 0xF) | ((int(step) << 4) & 0xFFFFFFFF)
    out = philox4x32_10(vi >> np.uint64(2), node_row, seq, c3,
                        seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF)
    out = np.broadcast_arrays(*out)
    sel = (np.broadcast_to(vi, out[0].shape) & np.uint64(3)).astype(np.int64)
    return np.choose(sel, out)


def uniform_from_word(w):
    """Open-interval uniform on the odd 24-bit grid, as float64."""
    w = np.asarray(w, dtype=np.uint64)
    return (2.0 * (w >> np.uint64(9)).astype(np.float64) + 1.0) * 2.0 ** -24


def gumbel_from_word(w):
    """Standard Gumbel variate -log(-log u)."""
    return -np.log(-np.log(uniform_from_word(w)))


def gumbel_row(seed, step, tag, seq, node_row, vocab_size):
    """Gumbel noise for vocabulary entries 0..vocab_size-1 of one row."""
    x = np.arange(vocab_size, dtype=np.uint64)
    return gumbel_from_word(words(seed, step, tag, seq, node_row, x))


def accept_uniform(seed, step, seq, node):
    """Uniform used by the accept/reject test of draft node `node`."""
    return float(uniform_from_word(
        words(seed, step, TAG_ACCEPT_UNIFORM, seq, node, 0)))
