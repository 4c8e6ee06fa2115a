"""Dropout keep-masks from a counter-based generator, as the layer oracle's dropout variant uses them.

TEST INFRASTRUCTURE, NOT PRODUCT CODE.  Only tests, the smoke check and the benchmark's
CPU-baseline leg may call this module; it shares no code with the HIP path and never imports it.

The paper has no dropout (it prints no layer equations at all); a GPT block trained with the
systems it builds on (section 3, "NVIDIA Megatron-LM") drops attention probabilities and the
output of each half before the residual addition.  This variant is defined here so that both
sides can draw the same random numbers independently of how they tile the work:

  generator   Philox4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw: "Parallel random numbers:
              as easy as 1, 2, 3", SC 2011): counter (c0, c1, c2, c3) and key (k0, k1) of 32-bit
              words; one round maps the counter to
                  (hi(M1*c2) ^ c1 ^ k0,  lo(M1*c2),  hi(M0*c0) ^ c3 ^ k1,  lo(M0*c0))
              with M0 = 0xD2511F53, M1 = 0xCD9E8D57, and between rounds the key advances by
              (0x9E3779B9, 0xBB67AE85).
  key         (seed mod 2^32, seed div 2^32) of a 64-bit seed.
  bytes       the 4 output words in order, each least-significant byte first: 16 random bytes,
              which serve 16 consecutive elements along a tensor's last index.
  keep rule   with the drop probability given in 1/256ths, t in 0..255: an element is DROPPED
              iff its byte < t; kept elements are multiplied by 256 / (256 - t).
  counters    attention probability P[b, head, i, j] (head = the global head index):
                  (i, j div 16, b * heads + head, 1), byte j mod 16
              output of the attention half, element (token, column c) of [T, H]:
                  (token, c div 16, 0, 2), byte c mod 16
              output of the feed-forward half: (token, c div 16, 0, 3), byte c mod 16

Pins (tests/test_oracle_dropout.py): the generator's published known-answer vectors, the byte
order on a hand-expanded word, mask frequencies against the binomial bound, the t = 0 identity.
"""
from __future__ import annotations

import numpy as np

_M0, _M1 = np.uint64(0xD2511F53), np.uint64(0xCD9E8D57)
_W0, _W1 = np.uint64(0x9E3779B9), np.uint64(0xBB67AE85)
_LOW = np.uint64(0xFFFFFFFF)
_32 = np.uint64(32)

STREAM_ATTN_PROBS, STREAM_ATTN_OUT, STREAM_MLP_OUT = 1, 2, 3


def philox4x32_10(c0, c1, c2, c3, k0, k1):
    """Philox4x32-10 on arrays of counters (broadcast together) with one key.  Returns four
    uint32 arrays."""
    c = [np.asarray(a, dtype=np.uint64) & _LOW for a in np.broadcast_arrays(c0, c1, c2, c3)]
    k0, k1 = np.uint64(int(k0) & 0xFFFFFFFF), np.uint64(int(k1) & 0xFFFFFFFF)
    for _ in range(10):
        p0 = _M0 * c[0]                         # 32 x 32 -> 64 bit products, exact in uint64
        p1 = _M1 * c[2]
        c = [(p1 >> _32) ^ c[1] ^ k0, p1 & _LOW, (p0 >> _32) ^ c[3] ^ k1, p0 & _LOW]
        k0, k1 = (k0 + _W0) & _LOW, (k1 + _W1) & _LOW
    return tuple(a.astype(np.uint32) for a in c)


def random_bytes(c0, c1, c2, c3, seed):
    """16 random bytes per counter: array of shape broadcast(c*) + (16,), dtype uint8."""
    seed = int(seed)
    words = philox4x32_10(c0, c1, c2, c3, seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF)
    out = np.empty(words[0].shape + (16,), dtype=np.uint8)
    for w in range(4):
        for byte in range(4):
            out[..., 4 * w + byte] = (words[w] >> np.uint32(8 * byte)) & np.uint32(0xFF)
    return out


def _check_t(t):
    t = int(t)
    if not 0 <= t <= 255:
        raise ValueError("drop probability is given in 1/256ths, 0..255")
    return t


def scale_of(t):
    return 256.0 / (256.0 - _check_t(t))


def keep_attention(seed, t, seq, sample, head, heads):
    """Keep mask [seq, seq] (True = kept) of the attention probabilities of one sample and one
    global head.  Entries above the diagonal are generated too; causality zeroes them anyway."""
    t = _check_t(t)
    groups = (seq + 15) // 16
    i = np.arange(seq, dtype=np.uint64)[:, None]
    jg = np.arange(groups, dtype=np.uint64)[None, :]
    b = random_bytes(i, jg, sample * heads + head, STREAM_ATTN_PROBS, seed)      # [seq, groups, 16]
    return b.reshape(seq, groups * 16)[:, :seq] >= t


def keep_hidden(seed, t, tokens, hidden, stream):
    """Keep mask [tokens, hidden] of a half's output (stream STREAM_ATTN_OUT or STREAM_MLP_OUT)."""
    t = _check_t(t)
    groups = (hidden + 15) // 16
    r = np.arange(tokens, dtype=np.uint64)[:, None]
    cg = np.arange(groups, dtype=np.uint64)[None, :]
    b = random_bytes(r, cg, 0, stream, seed)
    return b.reshape(tokens, groups * 16)[:, :hidden] >= t
