"""Pins of the oracle's observation codec (Section 4.1: observations are stored compressed, losslessly):
a hand-worked row, closed-form sizes, a second derivation of mask and counts with numpy, and the round trip
on rows of every mixture.  None of them calls the encoder to obtain its expected values."""
import os

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "codec_hand_row.txt")


def read_golden():
    out = {}
    for line in open(GOLDEN):
        line = line.split("#")[0].strip()
        if line:
            k, v = line.split(":")
            out[k.strip()] = v.split()
    return out


def hand_row():
    row = np.empty(256, np.uint8)
    row[0:64] = 0x07
    row[64:128] = np.arange(64)
    row[128:192] = 0xFF
    row[192:255] = 0x2A
    row[255] = 0x2B
    return row


def test_hand_worked_row():
    g = read_golden()
    row = hand_row()
    enc, used = oracle.codec_encode(row[None])
    assert enc.shape == (1, int(g["stride"][0])) and oracle.codec_row_bytes(int(g["raw_bytes"][0])) == int(g["stride"][0])
    assert int(used[0]) == int(g["used"][0])
    hexs = lambda b: [("%02x" % x) for x in b]
    assert hexs(enc[0, 0:16]) == g["mask"]
    assert hexs(enc[0, 16:32]) == g["flat"]
    image = enc[0, 32:]
    assert np.array_equal(image[64:128], row[64:128]) and np.array_equal(image[192:256], row[192:256])
    assert not image[0:64].any() and not image[128:192].any()
    assert np.array_equal(oracle.codec_decode(enc, 256)[0], row)


@pytest.mark.parametrize("raw_bytes,stride", [(64, 96), (4096, 16 + 64 + 4096), (4160, 16 + 80 + 4160),
                                              (28224, 64 + 448 + 28224), (256, 288)])
def test_stride_closed_form(raw_bytes, stride):
    assert oracle.codec_row_bytes(raw_bytes) == stride


@pytest.mark.parametrize("bad", [0, 1, 63, 100, 28225])
def test_sizes_that_are_refused(bad):
    assert oracle.codec_row_bytes(bad) == 0


def frame_like(rng, n, raw_bytes, flat_share):
    """Rows whose blocks are flat with probability flat_share, else random bytes."""
    nb = raw_bytes // 64
    rows = rng.integers(0, 256, (n, nb, 64), dtype=np.uint8)
    flat = rng.random((n, nb)) < flat_share
    rows[flat] = rng.integers(0, 256, (int(flat.sum()), 1), dtype=np.uint8)
    return rows.reshape(n, raw_bytes)


@pytest.mark.parametrize("raw_bytes", [64, 128, 4096, 4160, 28224])
@pytest.mark.parametrize("flat_share", [0.0, 0.3, 0.9, 1.0])
def test_round_trip_and_second_derivation(raw_bytes, flat_share):
    rng = np.random.default_rng(raw_bytes + int(flat_share * 10))
    rows = frame_like(rng, 6, raw_bytes, flat_share)
    enc, used = oracle.codec_encode(rows)
    assert np.array_equal(oracle.codec_decode(enc, raw_bytes), rows)        # lossless
    # the same mask, bytes and image from array operations
    nb = raw_bytes // 64
    blocks = rows.reshape(6, nb, 64)
    not_flat = (blocks != blocks[:, :, :1]).any(axis=2)
    n_kept = not_flat.sum(axis=1)
    M = (8 * ((nb + 63) // 64) + 15) // 16 * 16
    V = (nb + 15) // 16 * 16
    bits = np.unpackbits(enc[:, :M], axis=1, bitorder="little")
    assert np.array_equal(bits[:, :nb].astype(bool), not_flat) and not bits[:, nb:].any()
    assert np.array_equal(used, M + (nb - n_kept) + 64 * n_kept)
    flat_bytes = enc[:, M:M + nb]
    assert np.array_equal(flat_bytes[~not_flat], blocks[~not_flat][:, 0])
    image = enc[:, M + V:].reshape(6, nb, 64)
    assert np.array_equal(image[not_flat], blocks[not_flat])


def test_every_part_of_the_encoding_matters():
    """A changed mask bit, byte of a flat block or stored block changes what is decoded."""
    rng = np.random.default_rng(5)
    rows = frame_like(rng, 1, 4160, 0.5)
    enc, _ = oracle.codec_encode(rows)
    blocks = rows.reshape(65, 64)
    not_flat = (blocks != blocks[:, :1]).any(axis=1)
    first_flat, first_kept = int(np.argmin(not_flat)), int(np.argmax(not_flat))
    M, V = 16, 80
    for off in (0, M + first_flat, M + V + 64 * first_kept + 5):
        bad = enc.copy()
        bad[0, off] ^= 1
        assert not np.array_equal(oracle.codec_decode(bad, 4160), rows)
