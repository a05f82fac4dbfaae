"""Philox4x32-10 and the layout of the uniform stream the sampling path draws from.

TEST INFRASTRUCTURE ONLY.  Written independently of the device generator.

Philox4x32-10 is the counter-based generator of Salmon, Moraes, Dror and Shaw
(SC'11): ten rounds of  (c0,c1,c2,c3) <- (hi(M1*c2)^c1^k0, lo(M1*c2), hi(M0*c0)^c3^k1,
lo(M0*c0)),  the key advancing by the Weyl constants after each round.

Stream layout (a reading; the paper only says sampling follows the cited speculative
decoding works): key = (seed low word, seed high word); counter = (round, global
sequence id, position i, 0); of the four output words, word 0 -> u_draft(i) (inverse-CDF
draw of draft token i, i = 1..k), word 1 -> u_accept(i) (acceptance test of draft token
i), word 2 -> u_resample(i) (residual / bonus draw when n = i, i = 0..k).  A word w maps
to the uniform (w >> 8) * 2^-24 in [0, 1).
"""
from __future__ import annotations

import numpy as np

M0 = 0xD2511F53
M1 = 0xCD9E8D57
W0 = 0x9E3779B9
W1 = 0xBB67AE85
MASK = 0xFFFFFFFF


def philox4x32_10(ctr, key):
    c0, c1, c2, c3 = (int(x) & MASK for x in ctr)
    k0, k1 = (int(x) & MASK for x in key)
    for _ in range(10):
        p0 = M0 * c0
        p1 = M1 * c2
        c0, c1, c2, c3 = ((p1 >> 32) ^ c1 ^ k0) & MASK, p1 & MASK, ((p0 >> 32) ^ c3 ^ k1) & MASK, p0 & MASK
        k0 = (k0 + W0) & MASK
        k1 = (k1 + W1) & MASK
    return c0, c1, c2, c3


def word_to_uniform(w: int) -> float:
    return float((w >> 8) * 2.0 ** -24)


def round_uniforms(seed: int, rnd: int, seq: int, k: int):
    """(u_draft[0..k], u_accept[0..k], u_resample[0..k]) for one sequence in one round;
    index i is the position; u_draft[0] and u_accept[0] are unused by the method."""
    ud, ua, ur = np.zeros(k + 1), np.zeros(k + 1), np.zeros(k + 1)
    for i in range(k + 1):
        w = philox4x32_10((rnd, seq, i, 0), (seed & MASK, (seed >> 32) & MASK))
        ud[i], ua[i], ur[i] = word_to_uniform(w[0]), word_to_uniform(w[1]), word_to_uniform(w[2])
    return ud, ua, ur
