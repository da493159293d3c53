"""CPU oracle for the image data-flow path (encode / decode).  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the CPU-baseline leg of the benchmark may use
this module; the product path never does.  It shares no code with the HIP
library.

What it computes (paper, Section "Image Data-flow Optimization").  Pixels are
integers 0..255, so the pixels that Z images hold at one position can be kept as
the digits of one number.  Algorithm "Encode" adds image i times 256^i, i = 0 ..
Z-1, into one matrix of the image's size; Algorithm "Decode" takes the matrix
modulo 256 and divides it by 256 (integer division), Z times, which returns the
images in order.  Algorithm "Loss-less Forced Encoding" halves every pixel so
that the digits are base 128, and keeps the lost low bit of every pixel in a
boolean offset array.

The result of each algorithm has a plain definition -- a positional numeral in
base 256 (or 128) whose digits are the pixels -- and the oracle is that
definition written out per position in exact Python integers, which never
overflow (Horner evaluation of the digits; digits back by repeated divmod).

Readings (the text is at odds with itself in three places):
  * the displayed sum runs i = 1..N while the algorithm starts at i = 0; the
    algorithm's exponents 0..Z-1 are taken, so that a single image encodes to
    itself;
  * the capacity remarks (16, or 32, images in one 64-bit float) exceed
    what 53 or 64 bits hold; the numbers here are exact integers of as many bits
    as needed (8 Z, or 7 Z), and `to_words` cuts them into 64-bit words;
  * the loss-less algorithm as printed adds the unhalved image times 128^i,
    which two different batches can map to the same number; the text's own
    description (halve, keep the parity) is taken: A += (img div 2) * 128^i.
    The paper gives no decoder for it; the one here inverts it digit by digit.

`to_words`, `pack_offsets` and `group_batch` fix the memory format that a
fixed-width machine needs (little-endian 64-bit words, one offset bit per image
in a 32-bit word, a batch cut into groups of Z images); they contain no
arithmetic of the method.  `decode_normalized` is the decode step followed by
the affine map a network input usually gets, value = pixel * scale[c] + shift[c]
with c the channel of the position (channels vary fastest), in float64.
"""
from __future__ import annotations

import numpy as np

MASK64 = (1 << 64) - 1


def _digits_to_number(digits, base: int) -> int:
    """Value of a positional numeral: digits[0] is the least significant digit."""
    value = 0
    for d in reversed(digits):
        value = value * base + int(d)
    return value


def _number_to_digits(value: int, base: int, count: int):
    """The `count` least significant digits of a non-negative integer, least significant first."""
    out = []
    for _ in range(count):
        value, d = divmod(int(value), base)
        out.append(d)
    return out


def encode(X: np.ndarray) -> np.ndarray:
    """Algorithm "Encode".  X: uint8 [Z, ...] -> Python integers [...]: at every position the number whose base-256
    digits are the pixels of images 0 .. Z-1 there, image 0 least significant."""
    X = np.asarray(X)
    assert X.dtype == np.uint8
    columns = X.reshape(X.shape[0], -1)
    out = np.empty(columns.shape[1], dtype=object)
    for p in range(columns.shape[1]):
        out[p] = _digits_to_number(columns[:, p], 256)
    return out.reshape(X.shape[1:])


def decode(A: np.ndarray, Z: int) -> np.ndarray:
    """Algorithm "Decode".  Integers [...] -> uint8 [Z, ...]: image i is base-256 digit i of every number."""
    A = np.asarray(A, dtype=object)
    flat = A.reshape(-1)
    X = np.zeros((Z, flat.size), dtype=np.uint8)
    for p in range(flat.size):
        X[:, p] = _number_to_digits(flat[p], 256, Z)
    return X.reshape((Z,) + A.shape)


def encode_lossless(X: np.ndarray):
    """Algorithm "Loss-less Forced Encoding": the halved pixels are the base-128 digits, the low bit of every pixel
    goes to the offset array.  X: uint8 [Z, ...] -> (integers [...], bool [Z, ...])."""
    X = np.asarray(X)
    assert X.dtype == np.uint8
    columns = X.reshape(X.shape[0], -1)
    A = np.empty(columns.shape[1], dtype=object)
    for p in range(columns.shape[1]):
        A[p] = _digits_to_number([int(v) >> 1 for v in columns[:, p]], 128)
    return A.reshape(X.shape[1:]), (X & 1).astype(bool)


def decode_lossless(A: np.ndarray, O: np.ndarray) -> np.ndarray:
    """Inverse of `encode_lossless`: pixel of image i = 2 * (base-128 digit i) + offset bit."""
    A = np.asarray(A, dtype=object)
    O = np.asarray(O, dtype=bool)
    Z = O.shape[0]
    flat = A.reshape(-1)
    half = np.zeros((Z, flat.size), dtype=np.uint8)
    for p in range(flat.size):
        half[:, p] = _number_to_digits(flat[p], 128, Z)
    return (2 * half.reshape(O.shape) + O.astype(np.uint8)).astype(np.uint8)


# ---- memory format -----------------------------------------------------------------------------------------------

def words_needed(Z: int, bits_per_image: int) -> int:
    """64-bit words that hold Z digits of the given width."""
    return (Z * bits_per_image + 63) // 64


def to_words(A: np.ndarray, n_words: int) -> np.ndarray:
    """Integers [...] -> uint64 [..., n_words], least significant word first."""
    A = np.asarray(A, dtype=object)
    out = np.zeros(A.shape + (n_words,), dtype=np.uint64)
    flat = A.reshape(-1)
    o = out.reshape(-1, n_words)
    for p in range(flat.size):
        v = int(flat[p])
        assert 0 <= v < (1 << (64 * n_words)), "value does not fit the words"
        for j in range(n_words):
            o[p, j] = (v >> (64 * j)) & MASK64
    return out


def from_words(Wd: np.ndarray) -> np.ndarray:
    """uint64 [..., n_words] -> integers [...]."""
    Wd = np.asarray(Wd, dtype=np.uint64)
    n_words = Wd.shape[-1]
    flat = Wd.reshape(-1, n_words)
    out = np.zeros(flat.shape[0], dtype=object)
    for p in range(flat.shape[0]):
        v = 0
        for j in range(n_words):
            v |= int(flat[p, j]) << (64 * j)
        out[p] = v
    return out.reshape(Wd.shape[:-1])


def pack_offsets(O: np.ndarray) -> np.ndarray:
    """bool [Z, ...] (Z <= 32) -> uint32 [...], bit i = O[i]."""
    Z = O.shape[0]
    assert Z <= 32
    out = np.zeros(O.shape[1:], dtype=np.uint32)
    for i in range(Z):
        out |= O[i].astype(np.uint32) << np.uint32(i)
    return out


def unpack_offsets(P: np.ndarray, Z: int) -> np.ndarray:
    P = np.asarray(P, dtype=np.uint32)
    return np.stack([((P >> np.uint32(i)) & np.uint32(1)).astype(bool) for i in range(Z)])


def group_batch(X: np.ndarray, Z: int):
    """A batch uint8 [B, P] as the list of its groups of Z consecutive images (the last may hold fewer)."""
    return [X[s:s + Z] for s in range(0, X.shape[0], Z)]


def encode_batch_words(X: np.ndarray, Z: int) -> np.ndarray:
    """uint8 [B, P] -> uint64 [ceil(B / Z), P, words_needed(Z, 8)]: every group encoded by `encode`."""
    nw = words_needed(Z, 8)
    return np.stack([to_words(encode(g), nw) for g in group_batch(X, Z)])


def decode_batch_words(Wd: np.ndarray, Z: int, B: int) -> np.ndarray:
    """Inverse of `encode_batch_words`: uint64 [G, P, words] -> uint8 [B, P]."""
    imgs = []
    for g in range(Wd.shape[0]):
        zg = min(Z, B - g * Z)
        imgs.append(decode(from_words(Wd[g]), zg))
    return np.concatenate(imgs, axis=0)


def encode_lossless_batch_words(X: np.ndarray, Z: int):
    """uint8 [B, P] -> (uint64 [G, P, words_needed(Z, 7)], uint32 [G, P])."""
    nw = words_needed(Z, 7)
    ws, os_ = [], []
    for g in group_batch(X, Z):
        A, O = encode_lossless(g)
        ws.append(to_words(A, nw))
        os_.append(pack_offsets(O))
    return np.stack(ws), np.stack(os_)


def decode_lossless_batch_words(Wd: np.ndarray, Ob: np.ndarray, Z: int, B: int) -> np.ndarray:
    imgs = []
    for g in range(Wd.shape[0]):
        zg = min(Z, B - g * Z)
        imgs.append(decode_lossless(from_words(Wd[g]), unpack_offsets(Ob[g], zg)))
    return np.concatenate(imgs, axis=0)


def decode_normalized(Wd: np.ndarray, Z: int, B: int, channels: int, scale, shift) -> np.ndarray:
    """Decode, then pixel * scale[c] + shift[c] in float64; c = position mod channels.  Returns float64 [B, P]."""
    X = decode_batch_words(Wd, Z, B).astype(np.float64)
    c = np.arange(X.shape[1]) % channels
    s = np.asarray(scale, dtype=np.float64)[c]
    t = np.asarray(shift, dtype=np.float64)[c]
    return X * s[None, :] + t[None, :]
