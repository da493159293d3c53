"""Pins for the data-flow oracle (encode / decode): each checks it against something other than itself.

The paper prints no worked numeric example for these algorithms, so the pins are what integer arithmetic fixes:
numbers worked out by hand (tests/golden/dataflow_worked.txt), the byte view of a little-endian machine word (a numpy
routine), Python's own int.to_bytes / int.from_bytes, capacity bounds, the round trip, and digit extraction by
shifts.  The last test shows why the loss-less algorithm is not taken as printed.
"""
import os

import numpy as np
import pytest

from oracle import dataflow_oracle as D
from paper_2105_00619_amd import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "dataflow_worked.txt")


def _cases():
    """Hand-worked examples: `kind | pixels of image 0, 1, ... at one position | expected numbers`."""
    out = []
    for line in open(GOLDEN):
        line = line.split("#")[0].strip()
        if not line:
            continue
        kind, pix, exp = [f.strip() for f in line.split("|")]
        out.append((kind, [int(v) for v in pix.split()], [int(v, 0) for v in exp.split()]))
    return out


def _rand(Z, P, seed):
    return np.random.default_rng(seed).integers(0, 256, size=(Z, P), dtype=np.uint8)


def test_hand_worked_examples():
    n = 0
    for kind, pix, exp in _cases():
        X = np.array(pix, dtype=np.uint8).reshape(len(pix), 1)
        if kind == "encode":
            assert int(D.encode(X)[0]) == exp[0]
            assert list(D.decode(np.array([exp[0]], dtype=object), len(pix))[:, 0]) == pix
        elif kind == "lossless":
            A, O = D.encode_lossless(X)
            assert int(A[0]) == exp[0]
            assert int(D.pack_offsets(O)[0]) == exp[1]
            assert list(D.decode_lossless(np.array([exp[0]], dtype=object), D.unpack_offsets(np.array([exp[1]]), len(pix)))[:, 0]) == pix
        elif kind == "words":
            got = D.to_words(np.array([exp[0]], dtype=object), len(exp) - 1)[0]
            assert [int(v) for v in got] == exp[1:]
            assert int(D.from_words(got[None, :])[0]) == exp[0]
        else:
            raise AssertionError(kind)
        n += 1
    assert n >= 8


def test_a_single_image_encodes_to_itself():
    # exponent 0 for the first image (the algorithm's counter starts at 0)
    X = _rand(1, 50, 1)
    assert np.array_equal(D.encode(X).astype(np.int64), X[0].astype(np.int64))


@pytest.mark.parametrize("Z", [8, 16])
def test_full_words_equal_the_little_endian_byte_view(Z):
    # with 8 images per 64-bit word, image i is byte i of the word on a little-endian machine
    X = _rand(Z, 257, 2 + Z)
    words = D.to_words(D.encode(X), Z // 8)
    view = np.ascontiguousarray(X.T).view("<u8")  # [P, Z / 8]
    assert np.array_equal(words, view)


@pytest.mark.parametrize("Z", [1, 2, 3, 5, 7, 8, 9, 12, 15, 16])
def test_encode_matches_int_from_bytes_and_decode_matches_to_bytes(Z):
    X = _rand(Z, 40, 30 + Z)
    A = D.encode(X)
    for p in range(X.shape[1]):
        assert int(A[p]) == int.from_bytes(bytes(int(v) for v in X[:, p]), "little")
        assert bytes(D.decode(A[p:p + 1], Z)[:, 0].tolist()) == int(A[p]).to_bytes(Z, "little")


@pytest.mark.parametrize("Z", list(range(1, 17)))
def test_round_trip_and_bound(Z):
    X = _rand(Z, 64, 100 + Z)
    A = D.encode(X)
    assert all(0 <= int(a) < 256 ** Z for a in A)
    assert np.array_equal(D.decode(A, Z), X)


def test_capacity_extremes():
    for Z in (8, 16):
        X = np.full((Z, 3), 255, dtype=np.uint8)
        assert all(int(a) == 2 ** (8 * Z) - 1 for a in D.encode(X))
        assert np.all(D.to_words(D.encode(X), Z // 8) == np.uint64(2 ** 64 - 1))
    X = np.zeros((16, 3), dtype=np.uint8)
    assert all(int(a) == 0 for a in D.encode(X))


def test_decoding_fewer_images_than_encoded_returns_the_first_ones():
    X = _rand(6, 20, 9)
    assert np.array_equal(D.decode(D.encode(X), 4), X[:4])


@pytest.mark.parametrize("Z", [1, 2, 7, 9, 10, 18, 19, 27, 28, 32])
def test_lossless_round_trip_digits_and_bound(Z):
    X = _rand(Z, 48, 200 + Z)
    A, O = D.encode_lossless(X)
    assert all(0 <= int(a) < 128 ** Z for a in A)
    assert np.array_equal(O, (X & 1).astype(bool))
    for i in range(Z):  # digit i by shifting: bits 7i .. 7i+6
        digits = np.array([(int(a) >> (7 * i)) & 127 for a in A])
        assert np.array_equal(digits, X[i] >> 1)
    assert np.array_equal(D.decode_lossless(A, O), X)
    nw = D.words_needed(Z, 7)
    assert nw == -(-7 * Z // 64)
    assert np.array_equal(D.from_words(D.to_words(A, nw)), A)
    assert np.array_equal(D.unpack_offsets(D.pack_offsets(O), Z), O)


def test_lossless_as_printed_would_not_be_decodable():
    # img * 128^i without halving: (128, 0) and (0, 1) give the same number, so the halved reading is the usable one
    def printed(pix):
        return sum(v * 128 ** i for i, v in enumerate(pix))
    assert printed([128, 0]) == printed([0, 1])
    a, oa = D.encode_lossless(np.array([[128], [0]], dtype=np.uint8))
    b, ob = D.encode_lossless(np.array([[0], [1]], dtype=np.uint8))
    assert (int(a[0]), int(D.pack_offsets(oa)[0])) == (64, 0)
    assert (int(b[0]), int(D.pack_offsets(ob)[0])) == (0, 2)


def test_words_needed():
    assert [D.words_needed(z, 8) for z in (1, 8, 9, 16)] == [1, 1, 2, 2]
    assert [D.words_needed(z, 7) for z in (1, 9, 10, 18, 19, 27, 28, 32)] == [1, 1, 2, 2, 3, 3, 4, 4]


def test_batch_grouping_and_ragged_last_group():
    X = W.make_pixels_u8(11, 4, 4, 3, seed=5).reshape(11, -1)
    Wd = D.encode_batch_words(X, 4)
    assert Wd.shape == (3, 48, 1) and Wd.dtype == np.uint64
    # the last group holds 3 images: its fourth byte is zero
    assert np.all((Wd[2, :, 0] >> np.uint64(24)) == 0)
    assert np.array_equal(Wd[1, :, 0] & np.uint64(0xFF), X[4].astype(np.uint64))
    assert np.array_equal(D.decode_batch_words(Wd, 4, 11), X)
    Wl, Ol = D.encode_lossless_batch_words(X, 10)
    assert Wl.shape == (2, 48, 2) and Ol.shape == (2, 48) and Ol.dtype == np.uint32
    assert np.array_equal(D.decode_lossless_batch_words(Wl, Ol, 10, 11), X)


def test_decode_normalized_closed_forms():
    X = W.make_pixels_u8(5, 2, 3, 3, seed=6).reshape(5, -1)
    Wd = D.encode_batch_words(X, 5)
    # scale 1/255, shift 0: the usual map to [0, 1]
    y = D.decode_normalized(Wd, 5, 5, 3, [1 / 255.0] * 3, [0.0] * 3)
    assert np.allclose(y, X / 255.0, rtol=0, atol=1e-15)
    # (pixel / 255 - mean_c) / std_c written as scale and shift; channel = position mod 3
    mean, std = np.array([0.49, 0.48, 0.45]), np.array([0.25, 0.24, 0.26])
    y = D.decode_normalized(Wd, 5, 5, 3, 1.0 / (255.0 * std), -mean / std)
    want = (X.reshape(5, 2, 3, 3) / 255.0 - mean) / std
    assert np.allclose(y.reshape(5, 2, 3, 3), want, rtol=1e-13, atol=1e-13)
    assert y[0, 4] == pytest.approx((X[0, 4] / 255.0 - mean[1]) / std[1], rel=1e-13)


def test_pixel_generator_is_seeded_and_8_bit():
    a = W.make_pixels_u8(4, 8, 8, 3, seed=3)
    b = W.make_pixels_u8(4, 8, 8, 3, seed=3)
    c = W.make_pixels_u8(4, 8, 8, 3, seed=4)
    assert a.dtype == np.uint8 and a.shape == (4, 8, 8, 3)
    assert np.array_equal(a, b) and not np.array_equal(a, c)
    u = W.make_pixels_u8(64, 8, 8, 3, seed=3, pixels="uniform")
    assert u.min() == 0 and u.max() == 255
