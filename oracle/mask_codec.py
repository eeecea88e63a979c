"""Stored activation masks: the packed bit mask and the sparse (difference-coded) form -- TEST INFRASTRUCTURE ONLY.

The paper names the memory that stored activation masks take as a hardware limitation and asks, as future
work, for a light-weight mask compression such as a sparse encoding; it defines no format.  The formats
below are this build's own (stated in full here, in include/clada.h and in the design notes); this file is
their plain definition, in pure Python loops, sharing nothing with the HIP library and never importing it.

Bit mask      : ceil(d_ff/32) words of 32 bits, bit j%32 of word j/32 set iff neuron j is kept; bits past
                d_ff are zero.
Sparse form   : the ascending positions j_0 < j_1 < ... at which a mask differs from a reference mask of the
                same layer (no reference = the all-zero mask, so the positions are the kept neurons), as the
                gaps g_i = j_i - j_{i-1} - 1 (j_{-1} = -1), each gap written as a little-endian base-128
                number: 7 value bits per byte, low group first, high bit set on every byte but the last.
                A mask that stays close to its reference (the prefix-static mask of the layer, or the previous
                token's mask) costs about one byte per changed neuron.
"""
from __future__ import annotations


def mask_words(d_ff: int) -> int:
    return (d_ff + 31) // 32


def pack(active_idx, d_ff: int) -> list[int]:
    """Ascending (or any) list of kept neurons -> bit-mask words."""
    words = [0] * mask_words(d_ff)
    for j in active_idx:
        j = int(j)
        assert 0 <= j < d_ff
        words[j // 32] |= 1 << (j % 32)
    return words


def unpack(words, d_ff: int) -> list[int]:
    """Bit-mask words -> ascending list of kept neurons (bits past d_ff are ignored)."""
    out = []
    for j in range(d_ff):
        if (int(words[j // 32]) >> (j % 32)) & 1:
            out.append(j)
    return out


def sparse_encode(words, ref_words, d_ff: int) -> tuple[bytes, int]:
    """(byte stream, number of coded positions) of the mask `words` against `ref_words` (None = all zero)."""
    out = bytearray()
    prev = -1
    n = 0
    for j in range(d_ff):
        bit = (int(words[j // 32]) >> (j % 32)) & 1
        ref = (int(ref_words[j // 32]) >> (j % 32)) & 1 if ref_words is not None else 0
        if bit != ref:
            gap = j - prev - 1
            while gap >= 128:
                out.append((gap & 127) | 128)
                gap >>= 7
            out.append(gap)
            prev = j
            n += 1
    return bytes(out), n


def sparse_decode(stream: bytes, ref_words, d_ff: int) -> list[int]:
    """Byte stream -> bit-mask words (the reference with the coded positions flipped)."""
    words = [int(w) for w in ref_words] if ref_words is not None else [0] * mask_words(d_ff)
    if d_ff % 32:                               # bits past d_ff are zero in the result
        words[-1] &= (1 << (d_ff % 32)) - 1
    pos = -1
    gap = 0
    shift = 0
    for byte in stream:
        gap |= (byte & 127) << shift
        if byte & 128:
            shift += 7
            continue
        pos += gap + 1
        assert pos < d_ff, "stream runs past d_ff"
        words[pos // 32] ^= 1 << (pos % 32)
        gap = 0
        shift = 0
    assert shift == 0, "stream ends inside a number"
    return words


def sparse_max_bytes(d_ff: int) -> int:
    """Upper bound of a stream's length: one byte per position, one more per gap >= 128, another per gap >= 16384
    (such gaps consume that many positions of the d_ff available)."""
    return d_ff + d_ff // 128 + d_ff // 16384
