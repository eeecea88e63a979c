"""Pins of oracle/mask_codec.py (stored masks: bit mask and sparse difference form)."""
import os

import numpy as np
import pytest

from oracle import mask_codec as mc

GOLD = os.path.join(os.path.dirname(__file__), "golden", "mask_codec_hand_case.txt")


def _gold():
    out = {}
    for ln in open(GOLD):
        if ln.startswith("#") or not ln.strip():
            continue
        k, *v = ln.split()
        out[k] = v
    return out


def test_hand_worked_example():
    g = _gold()
    kept = [0, 1, 5, 31, 32, 63, 64, 200, 299]
    words = [int(v, 16) for v in g["mask_words"]]
    ref = [int(v, 16) for v in g["ref_words"]]
    assert mc.pack(kept, 300) == words and mc.unpack(words, 300) == kept
    assert mc.unpack(ref, 300) == [0, 1, 5, 31, 33, 63, 64, 299]
    plain = bytes(int(v, 16) for v in g["sparse_plain"])
    vs_ref = bytes(int(v, 16) for v in g["sparse_vs_ref"])
    assert mc.sparse_encode(words, None, 300) == (plain, 9)
    assert mc.sparse_encode(words, ref, 300) == (vs_ref, 3)
    assert mc.sparse_decode(plain, None, 300) == words
    assert mc.sparse_decode(vs_ref, ref, 300) == words
    far = mc.pack([20000], 20001)
    assert mc.sparse_encode(far, None, 20001) == (bytes(int(v, 16) for v in g["gap_20000"]), 1)


@pytest.mark.parametrize("d_ff,density", [(1, 1.0), (31, 0.5), (32, 0.5), (33, 0.5), (1376, 0.6), (11008, 0.55),
                                          (14336, 0.02), (40000, 0.001), (5000, 0.0), (262144, 0.0001)])
def test_bit_mask_is_numpy_packbits_and_round_trips(d_ff, density):
    r = np.random.default_rng(d_ff)
    m = r.random(d_ff) < density
    idx = np.flatnonzero(m)
    words = mc.pack(idx, d_ff)
    pad = np.zeros(mc.mask_words(d_ff) * 32, bool)
    pad[:d_ff] = m
    assert np.array_equal(np.array(words, np.uint32), np.packbits(pad, bitorder="little").view(np.uint32))
    assert mc.unpack(words, d_ff) == idx.tolist()
    # bits past d_ff are ignored by unpack
    dirty = list(words)
    if d_ff % 32:
        dirty[-1] |= 1 << 31
        assert mc.unpack(dirty, d_ff) == idx.tolist()


def _leb128(n):
    """Independent statement of the number format (unsigned LEB128)."""
    out = []
    while True:
        b = n % 128
        n //= 128
        out.append(b + (128 if n else 0))
        if not n:
            return out


@pytest.mark.parametrize("d_ff,density,flip", [(300, 0.5, 0.02), (11008, 0.55, 0.01), (14336, 0.45, 0.0),
                                               (262144, 0.3, 0.0002), (40000, 0.0, 0.0), (33, 1.0, 1.0)])
def test_sparse_form_round_trips_and_matches_its_definition(d_ff, density, flip):
    r = np.random.default_rng(d_ff + 1)
    ref_m = r.random(d_ff) < density
    m = ref_m ^ (r.random(d_ff) < flip)
    words, ref = mc.pack(np.flatnonzero(m), d_ff), mc.pack(np.flatnonzero(ref_m), d_ff)
    for reference, positions in ((ref, np.flatnonzero(m ^ ref_m)), (None, np.flatnonzero(m))):
        stream, n = mc.sparse_encode(words, reference, d_ff)
        assert n == positions.size and len(stream) <= mc.sparse_max_bytes(d_ff)
        gaps = np.diff(np.concatenate(([-1], positions))) - 1
        assert list(stream) == [b for g in gaps for b in _leb128(int(g))]
        assert mc.sparse_decode(stream, reference, d_ff) == words
    # one byte per changed neuron while gaps stay below 128
    stream, n = mc.sparse_encode(words, ref, d_ff)
    gaps = np.diff(np.concatenate(([-1], np.flatnonzero(m ^ ref_m)))) - 1
    assert len(stream) == n + int((gaps >= 128).sum()) + int((gaps >= 16384).sum())


def test_worst_case_length_bound_is_attained_only_by_wide_gaps():
    d_ff = 262144
    assert len(mc.sparse_encode(mc.pack(range(d_ff), d_ff), None, d_ff)[0]) == d_ff          # every gap 0
    every129 = list(range(128, d_ff, 129))                                                     # every gap 128: 2 bytes
    assert len(mc.sparse_encode(mc.pack(every129, d_ff), None, d_ff)[0]) == 2 * len(every129) <= mc.sparse_max_bytes(d_ff)


def test_malformed_streams_are_rejected():
    with pytest.raises(AssertionError):
        mc.sparse_decode(bytes([0x80]), None, 64)            # ends inside a number
    with pytest.raises(AssertionError):
        mc.sparse_decode(bytes([64]), None, 64)              # position 64 of 64
