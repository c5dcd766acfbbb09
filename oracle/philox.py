"""Philox4x32-10 counter-based generator (Salmon, Moraes, Dror, Shaw, SC'11) in
NumPy integer arithmetic, and the slot map that turns it into the uniforms the
sampler consumes.  TEST INFRASTRUCTURE (oracle side); the HIP library carries its
own implementation of the same published algorithm.

Slot map: for position b, draft s and slot t, the 128-bit counter is
(t // 4, b, s, offset) and the 64-bit key is (seed low word, seed high word);
slot t takes output word t % 4 and maps it to u = (word >> 8) * 2^-24, which is
exact in fp32 and lies in [0, 1).  Drafting uses s = 0 .. S-1; the verification step
(its acceptance tests in slots 0..n-1, its final draw in slot n) uses s = 2^32 - 1.
"""
from __future__ import annotations

import numpy as np

_M0 = np.uint64(0xD2511F53)
_M1 = np.uint64(0xCD9E8D57)
_W0 = np.uint64(0x9E3779B9)
_W1 = np.uint64(0xBB67AE85)
_MASK = np.uint64(0xFFFFFFFF)
_SH = np.uint64(32)


def philox4x32_10(counter, key):
    """counter: 4 arrays (or ints) of 32-bit words, key: 2 words.  Returns the four
    output words as uint64 arrays holding 32-bit values."""
    c = [np.asarray(x, dtype=np.uint64) & _MASK for x in counter]
    k0 = np.asarray(key[0], dtype=np.uint64) & _MASK
    k1 = np.asarray(key[1], dtype=np.uint64) & _MASK
    for rnd in range(10):
        if rnd > 0:
            k0 = (k0 + _W0) & _MASK
            k1 = (k1 + _W1) & _MASK
        p0 = _M0 * c[0]
        p1 = _M1 * c[2]
        hi0, lo0 = p0 >> _SH, p0 & _MASK
        hi1, lo1 = p1 >> _SH, p1 & _MASK
        c = [hi1 ^ c[1] ^ k0, lo1, hi0 ^ c[3] ^ k1, lo0]
    return c


VERIFY_DRAFT_INDEX = 0xFFFFFFFF


def verify_uniforms(B: int, slots: int, seed: int, offset: int = 0) -> np.ndarray:
    """u[b,t] of the verification step: the same generator and slot map with the draft index
    fixed at 2^32 - 1, a value no drafting call reaches (its S is a 32-bit signed count), so that
    equal (seed, offset) never hand a test the uniform that drew the token it tests."""
    return uniforms(B, 1, slots, seed, offset, first_draft=VERIFY_DRAFT_INDEX)[:, 0]


def uniforms(B: int, S: int, slots: int, seed: int, offset: int = 0, first_draft: int = 0) -> np.ndarray:
    """u[b,s,t] for t < slots, float64 holding values exact in fp32 (draft indices
    first_draft .. first_draft + S - 1)."""
    b = np.arange(B, dtype=np.uint64)[:, None, None]
    s = (np.arange(S, dtype=np.uint64) + np.uint64(first_draft))[None, :, None]
    t = np.arange(slots, dtype=np.uint64)[None, None, :]
    b, s, t = np.broadcast_arrays(b, s, t)
    key = (np.uint64(seed & 0xFFFFFFFF), np.uint64((seed >> 32) & 0xFFFFFFFF))
    words = philox4x32_10((t // np.uint64(4), b, s, np.uint64(offset & 0xFFFFFFFF) + 0 * t), key)
    sel = (t % np.uint64(4)).astype(np.int64)
    w = np.choose(sel, words)
    return (w >> np.uint64(8)).astype(np.float64) * (2.0 ** -24)
