"""Second, independent implementation of the sampling path in pure Python.

Written from the published definitions with Python big integers, ``fractions`` and ``math``
only (no numpy arithmetic, no ctypes), so that it cannot share a mistake with the C oracle:
Philox4x32-10 (Salmon et al., SC'11), the open-interval uniform, g = -log(-log u)
(Alg. 1 of the paper), and the streaming strict-> argmax (appendix Alg. "Gumbel-Max sampling
(standalone logits)").  Only usable on tiny inputs.
"""
import math
import struct
from fractions import Fraction

M32 = (1 << 32) - 1


def philox4x32_10(ctr, key):
    c = [int(v) & M32 for v in ctr]
    k = [int(v) & M32 for v in key]
    for _ in range(10):
        p0 = 0xD2511F53 * c[0]
        p1 = 0xCD9E8D57 * c[2]
        c = [((p1 >> 32) ^ c[1] ^ k[0]) & M32, p1 & M32, ((p0 >> 32) ^ c[3] ^ k[1]) & M32, p0 & M32]
        k = [(k[0] + 0x9E3779B9) & M32, (k[1] + 0xBB67AE85) & M32]
    return c


def random_word(seed, row, vocab_id):
    out = philox4x32_10([vocab_id >> 2, row, 0, 0], [seed & M32, (seed >> 32) & M32])
    return out[vocab_id & 3]


def _round_to_f32(q: Fraction) -> float:
    """Round an exact rational to the nearest float32 (ties to even) via struct."""
    # float(q) is correctly rounded to fp64; fp64 -> fp32 by struct is round-to-nearest-even.
    # Double rounding cannot bite here: the inputs below have at most 34 significant bits.
    return struct.unpack("f", struct.pack("f", float(q)))[0]


def uniform_x(r: int) -> float:
    """x = min(fl32(fl32(r) * 2^-32 + 2^-33), 1 - 2^-24)."""
    rf = _round_to_f32(Fraction(r))                       # (float) r
    x = _round_to_f32(Fraction(rf) / (1 << 32) + Fraction(1, 1 << 33))   # one rounding, as fma
    cap = 1.0 - 2.0 ** -24
    return min(x, cap)


def gumbel_from_word(r: int) -> float:
    x = uniform_x(r)
    return -math.log(-math.log1p(-x))


def bf16_to_float(bits: int) -> float:
    return struct.unpack("f", struct.pack("I", (int(bits) & 0xFFFF) << 16))[0]


def logit(Hrow, Wrow) -> float:
    """Exact dot product of two bf16 rows (rational arithmetic), rounded once to fp64."""
    acc = Fraction(0)
    for h, w in zip(Hrow, Wrow):
        acc += Fraction(bf16_to_float(h)) * Fraction(bf16_to_float(w))
    return float(acc)


def sample_row(Hrow, W, tau, seed, row, vocab_offset=0):
    best, best_i = -math.inf, -1
    scores = []
    for i, Wrow in enumerate(W):
        vid = vocab_offset + i
        s = logit(Hrow, Wrow) / tau + gumbel_from_word(random_word(seed, row, vid))
        scores.append(s)
        if s > best:
            best, best_i = s, vid
    return best_i, best, scores
