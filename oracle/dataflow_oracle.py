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

These are encodings, so the oracle takes the algorithms' steps in their order
and notation (X batch, A encoded matrix, O offsets, Z images, i counter, domain
= base^i), in exact integer arithmetic: A is a numpy array of Python integers,
which never overflow.  Nothing is blocked or reordered.

Readings (the text is at odds with itself in three places):
  * the displayed sum runs i = 1..N while the algorithm starts at i = 0; the
    algorithm's exponents 0..Z-1 are taken, so that a single image encodes to
    itself;
  * the capacity remarks ("16 images", "32 images" in a 64-bit float) exceed
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


def encode(X: np.ndarray) -> np.ndarray:
    """Algorithm "Encode".  X: uint8 [Z, ...] -> A: Python integers [...], A = sum_i X[i] * 256^i."""
    X = np.asarray(X)
    assert X.dtype == np.uint8
    Z = X.shape[0]
    A = np.zeros(X.shape[1:], dtype=object)
    i = 0
    while i != Z:
        img = X[i].astype(object)
        domain = 256 ** i
        A = A + (img * domain)
        i = i + 1
    return A


def decode(A: np.ndarray, Z: int) -> np.ndarray:
    """Algorithm "Decode".  A: integers [...] -> X: uint8 [Z, ...]; modulo 256, then integer division by 256."""
    A = np.array(A, dtype=object, copy=True)
    X = np.zeros((Z,) + A.shape, dtype=np.uint8)
    i = 0
    while i != Z:
        X[i] = (A % 256).astype(np.uint8)
        A = A // 256
        i = i + 1
    return X


def encode_lossless(X: np.ndarray):
    """Algorithm "Loss-less Forced Encoding" (halved pixels as base-128 digits, parities kept).

    X: uint8 [Z, ...] -> (A: integers [...], O: bool [Z, ...])."""
    X = np.asarray(X)
    assert X.dtype == np.uint8
    Z = X.shape[0]
    A = np.zeros(X.shape[1:], dtype=object)
    O = np.zeros(X.shape, dtype=bool)
    i = 0
    while i != Z:
        img = X[i].astype(object)
        offset = img % 2
        domain = 128 ** i
        A = A + ((img // 2) * domain)
        O[i] = offset.astype(bool)
        i = i + 1
    return A, O


def decode_lossless(A: np.ndarray, O: np.ndarray) -> np.ndarray:
    """Inverse of `encode_lossless`: digit = A mod 128, A = A div 128, pixel = 2 * digit + offset."""
    A = np.array(A, dtype=object, copy=True)
    Z = O.shape[0]
    X = np.zeros(O.shape, dtype=np.uint8)
    i = 0
    while i != Z:
        digit = A % 128
        X[i] = (2 * digit + O[i].astype(object)).astype(np.uint8)
        A = A // 128
        i = i + 1
    return X


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
