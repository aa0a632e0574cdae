"""Pins for the oracle's packed layout: round trips, structural invariants, hand-assembled bytes.

The byte layout is this build's own (Section 2.2 only requires that the N:M metadata be well
defined), so nothing printed in the paper can pin it; the fixtures under tests/golden were
assembled by hand from the layout rules.
"""
import os

import numpy as np
import pytest

import oracle

PATTERNS = [(2, 4), (1, 4), (2, 8), (6, 8), (4, 8), (1, 2), (3, 4), (8, 8), (4, 4), (1, 8), (7, 8)]
GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "pack_2of4_row128.txt")
GOLDEN_OTHER = os.path.join(os.path.dirname(__file__), "golden", "pack_other_patterns_row128.txt")


def gaussian(shape, seed, sigma=0.02):
    return (np.random.default_rng(seed).standard_normal(shape) * sigma).astype(np.float32)


def read_golden(path=GOLDEN):
    out = {}
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        tag, *hexbytes = line.split()
        out[tag] = np.array([int(h, 16) for h in hexbytes], dtype=np.uint8)
    return out


def test_golden_case_a():
    W = np.tile(np.array([1.0, -1.0, 0.0, 0.0], np.float32), (1, 32))
    packed, gamma = oracle.quantize_mask_pack(W, 2, 4)
    assert gamma == np.float32(0.5)
    assert np.array_equal(packed, read_golden()["A"])


def test_golden_case_b():
    W = np.zeros((1, 128), np.float32)
    W[0, 22] = -1.0
    W[0, 23] = 0.001
    packed, _ = oracle.quantize_mask_pack(W, 2, 4)
    assert np.array_equal(packed, read_golden()["B"])


@pytest.mark.parametrize("N,M", PATTERNS)
@pytest.mark.parametrize("d_in", [128, 256, 136, 8])
def test_round_trip_and_size(N, M, d_in):
    W = gaussian((24, d_in), 300 + N * 16 + M)
    Weff, mask, _ = oracle.quantize_mask(W, N, M)
    packed = oracle.pack(Weff, mask, N, M)
    bits = 0 if N == M else {2: 1, 4: 2, 8: 3}[M]
    slots = 128 * N // M
    assert oracle.chunk_bytes(N, M) == slots * bits // 8 + slots // 4
    assert packed.size == 24 * ((d_in + 127) // 128) * oracle.chunk_bytes(N, M) == oracle.packed_bytes(24, d_in, N, M)
    Weff2, mask2 = oracle.unpack(packed, 24, d_in, N, M)
    assert np.array_equal(Weff, Weff2) and np.array_equal(mask, mask2)
    # pack(unpack(p)) == p
    assert np.array_equal(oracle.pack(Weff2, mask2, N, M), packed)


def test_bits_per_weight():
    assert oracle.packed_bytes(2560, 2560, 2, 4) == 2560 * 2560 // 4          # 2 bits per weight
    assert oracle.packed_bytes(6912, 2560, 2, 4) == 4423680
    assert oracle.packed_bytes(6912, 2560, 1, 4) == 4423680 // 2             # 1 bit per weight
    assert oracle.packed_bytes(6912, 2560, 2, 8) == 6912 * 2560 * 5 // 32    # 1.25 bits per weight
    assert oracle.packed_bytes(16, 130, 2, 4) == -1                          # d_in not a multiple of M
    assert oracle.packed_bytes(16, 128, 5, 4) == -1 and oracle.packed_bytes(16, 128, 1, 3) == -1


def independent_decode_2of4(packed, d_out, d_in):
    """Second reading of the 2:4 layout, written from the rules with numpy bit operations."""
    nch = (d_in + 127) // 128
    p = packed.reshape(d_out, nch, 32)
    idx_words = p[..., :16].copy().view("<u4")      # [d_out, nch, 4]
    code_words = p[..., 16:].copy().view("<u4")
    W = np.zeros((d_out, nch * 128), np.int8)
    M_ = np.zeros((d_out, nch * 128), np.uint8)
    rows = np.arange(d_out)[:, None]
    for c in range(nch):
        for j in range(4):
            for t in range(8):
                nib = (idx_words[:, c, j] >> (4 * t)) & 0xF
                for half, idx in ((0, nib & 3), (1, nib >> 2)):
                    v = 2 * t + half
                    code = (code_words[:, c, j] >> (8 * (v % 4) + 2 * (v // 4))) & 3
                    col = c * 128 + 32 * j + 4 * t + idx
                    val = np.where(code == 1, 1, np.where(code == 3, -1, 0)).astype(np.int8)
                    W[rows[:, 0], col] = val
                    M_[rows[:, 0], col] = 1
                    assert (code != 2).all()
    return W[:, :d_in], M_[:, :d_in]


def test_2of4_layout_second_reading_and_invariants():
    W = gaussian((40, 384), 7)
    Weff, mask, _ = oracle.quantize_mask(W, 2, 4)
    packed = oracle.pack(Weff, mask, 2, 4)
    W2, M2 = independent_decode_2of4(packed, 40, 384)
    assert np.array_equal(W2, Weff) and np.array_equal(M2, mask)
    # index nibbles strictly ascending: idx0 < idx1 in every group
    idx = packed.reshape(40, 3, 32)[..., :16]
    lo, hi = idx & 0xF, idx >> 4
    for nib in (lo, hi):
        assert ((nib & 3) < (nib >> 2)).all()


def test_pack_rejects_bad_masks():
    Weff = np.zeros((2, 128), np.int8)
    mask = np.zeros((2, 128), np.uint8)
    mask[:, 0::4] = 1                                   # only one kept per group
    with pytest.raises(ValueError):
        oracle.pack(Weff, mask, 2, 4)
    with pytest.raises(ValueError):
        oracle.unpack(np.zeros(10, np.uint8), 2, 128, 2, 4)


# ----------------------------------------------------------------------------- other patterns: fixtures
_VALUE_BY_3 = (1, -1, 0)           # value of slot s by s % 3 (cases Q and S of the fixture file)
_VALUE_BY_5 = (1, -1, 0, -1, 1)    # value of slot s by s % 5 (cases E and D)


def _row_from_kept(kept_of_group, M, values):
    """One row of 128 weights: group g keeps the ascending positions kept_of_group(g); the s-th kept weight of
    the row (slot s) has value values[s % len(values)]."""
    Weff = np.zeros((1, 128), np.int8)
    mask = np.zeros((1, 128), np.uint8)
    s = 0
    for g in range(128 // M):
        for p in kept_of_group(g):
            mask[0, g * M + p] = 1
            Weff[0, g * M + p] = values[s % len(values)]
            s += 1
    return Weff, mask


FIXTURES = {
    "Q": (1, 4, lambda g: (g % 4,), _VALUE_BY_3),
    "E": (2, 8, lambda g: (g % 7, 7), _VALUE_BY_5),
    "S": (6, 8, lambda g: ((2, 3, 4, 5, 6, 7), (0, 1, 2, 3, 4, 5), (1, 2, 3, 4, 5, 6), (0, 1, 2, 5, 6, 7))[g % 4], _VALUE_BY_3),
    "D": (8, 8, lambda g: tuple(range(8)), _VALUE_BY_5),
}


@pytest.mark.parametrize("case", sorted(FIXTURES))
def test_golden_other_patterns(case):
    # hand-assembled bytes for the other index widths: 2 bits (1:4), 3 bits (2:8, 6:8) and none (8:8)
    N, M, kept, values = FIXTURES[case]
    Weff, mask = _row_from_kept(kept, M, values)
    want = read_golden(GOLDEN_OTHER)[case]
    assert want.size == oracle.chunk_bytes(N, M)
    assert np.array_equal(oracle.pack(Weff, mask, N, M), want)
    W2, M2 = oracle.unpack(want, 1, 128, N, M)
    assert np.array_equal(W2, Weff) and np.array_equal(M2, mask)


def independent_decode(packed, d_out, d_in, N, M):
    """Second reading of the layout for any pattern, written from the rules with numpy on whole bit planes:
    the index field as one little-endian bit string cut into b-bit numbers, the code field as bit pairs
    gathered by their position 8*(v%4) + 2*(v/4) inside each 32-bit word."""
    b = 0 if N == M else {2: 1, 4: 2, 8: 3}[M]
    S = 128 * N // M
    nch = (d_in + 127) // 128
    idx_bytes, code_bytes = S * b // 8, S // 4
    chunks = packed.reshape(d_out * nch, idx_bytes + code_bytes)
    if b:
        bits = np.unpackbits(chunks[:, :idx_bytes], axis=1, bitorder="little").reshape(-1, S, b)
        pos = (bits.astype(np.int64) << np.arange(b)).sum(axis=2)                  # [chunks, S]
    else:
        pos = np.tile(np.arange(S) % M, (chunks.shape[0], 1))
    cbits = np.unpackbits(chunks[:, idx_bytes:], axis=1, bitorder="little").reshape(-1, S // 16, 32)
    v = np.arange(16)
    at = 8 * (v % 4) + 2 * (v // 4)
    code = (cbits[:, :, at] + 2 * cbits[:, :, at + 1]).reshape(-1, S)                 # [chunks, S]
    assert (code != 2).all()
    val = np.select([code == 1, code == 3], [1, -1], 0).astype(np.int8)
    col = (np.arange(S) // N) * M + pos                                               # column inside the chunk
    W = np.zeros((d_out * nch, 128), np.int8)
    K = np.zeros((d_out * nch, 128), np.uint8)
    r = np.arange(d_out * nch)[:, None]
    W[r, col] = val
    K[r, col] = 1
    # slots of a group ascend strictly: no two slots land on one weight
    assert (K.reshape(d_out * nch, 128 // M, M).sum(axis=2) == N).all()
    return W.reshape(d_out, nch * 128)[:, :d_in], K.reshape(d_out, nch * 128)[:, :d_in]


@pytest.mark.parametrize("N,M", PATTERNS)
def test_layout_second_reading_all_patterns(N, M):
    W = gaussian((40, 392), 700 + 10 * N + M)             # ragged last chunk
    Weff, mask, _ = oracle.quantize_mask(W, N, M)
    packed = oracle.pack(Weff, mask, N, M)
    W2, M2 = independent_decode(packed, 40, 392, N, M)
    assert np.array_equal(W2, Weff) and np.array_equal(M2, mask)
    for case, (n, m, kept, values) in FIXTURES.items():
        if (n, m) == (N, M):
            We, Mk = _row_from_kept(kept, m, values)
            Wd, Md = independent_decode(read_golden(GOLDEN_OTHER)[case], 1, 128, N, M)
            assert np.array_equal(Wd, We) and np.array_equal(Md, Mk)
