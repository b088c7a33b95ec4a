"""Seeded synthetic vocabularies shaped like byte-level BPE vocabularies.

ids 0..255 are the single bytes; the rest are byte strings whose class is drawn
once per token (so long all-letter / all-digit / all-punctuation tokens exist)
and whose bytes are then uniform within the class.  Duplicates are kept.
"""
import numpy as np
from .rng import stream

PUNCT = b'{}[]:," \t\n\r'          # JSON punctuation + whitespace
DIGIT = b'0123456789-+.eE'
LETTER = bytes(range(65, 91)) + bytes(range(97, 123))


def _utf8(cp: int) -> bytes:
    if cp < 0x800:
        return bytes([0xC0 | (cp >> 6), 0x80 | (cp & 0x3F)])
    return bytes([0xE0 | (cp >> 12), 0x80 | ((cp >> 6) & 0x3F), 0x80 | (cp & 0x3F)])


def _non_ascii(rs, n: int) -> bytes:
    out = b""
    while len(out) < n:
        while True:
            cp = 0x80 + rs.below(0x10000 - 0x80)
            if not (0xD800 <= cp <= 0xDFFF):
                break
        out += _utf8(cp)
    return out[:n]            # the last code point may be cut (byte-fallback style fragment)


def make_vocab(seed: int, size: int, *, uniform_2_8: bool = False, non_ascii: bool = True):
    """Return a list of `size` byte strings.

    uniform_2_8: lengths uniform on 2..8 (the 2,048-token configuration); otherwise
    geometric with mean 4 truncated to 1..16.  Class mix 40/30/30 (P/D/L), or
    36/27/27/10 with the non-ASCII class.
    """
    rs = stream(seed, "vocab")
    toks = [bytes([b]) for b in range(256)][:size]
    while len(toks) < size:
        if uniform_2_8:
            n = 2 + rs.below(7)
        else:
            n = 1
            while n < 16 and rs.below(4) != 0:
                n += 1
        r = rs.below(100)
        if non_ascii:
            cls = PUNCT if r < 36 else DIGIT if r < 63 else LETTER if r < 90 else None
        else:
            cls = PUNCT if r < 40 else DIGIT if r < 70 else LETTER
        if cls is None:
            toks.append(_non_ascii(rs, n))
        else:
            toks.append(bytes(cls[rs.below(len(cls))] for _ in range(n)))
    return toks


def vocab_csr(tokens):
    """(off int64[V+1], bytes uint8[total]) in the layout the C boundary takes."""
    off = np.zeros(len(tokens) + 1, dtype=np.int64)
    np.cumsum([len(t) for t in tokens], out=off[1:])
    data = np.frombuffer(b"".join(tokens), dtype=np.uint8).copy() if off[-1] else np.zeros(0, np.uint8)
    return off, data
