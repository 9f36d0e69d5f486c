"""TEST INFRASTRUCTURE ONLY: CPU oracle, never imported by the product path.

b-bit affine quantisation of the guided basis for transmission (Data Transmission
Controller, Sec. 4.4, the quantise / restore pair of its first equation):

    x_q = round(x / lambda + delta),      x_hat = lambda * (x_q - delta),
    lambda = (max - min) / (2^b - 1)

over one tensor (max, min over all its entries).  Reading of the zero point: the
printed delta = round(-2^b / (max - min)) does not have the dimension of a code;
delta = round(-min / lambda) is used, which maps min to code 0 and max to code
2^b - 1 (up to the rounding of delta itself), and codes are clipped to
[0, 2^b - 1] so that they fit b bits.  All arithmetic in fp32, round = nearest,
ties to even: the decision of an integer code is taken in the precision the
device uses.  A constant tensor (max = min) gets lambda = 1, delta = -min rounded.
"""
import numpy as np


def affine_params(x, bits=4):
    """(lambda, delta) as fp32 scalars for the tensor x."""
    x = np.asarray(x, dtype=np.float32)
    lo, hi = np.float32(x.min()), np.float32(x.max())
    levels = np.float32(2 ** bits - 1)
    lam = np.float32((hi - lo) / levels)
    if not lam > 0:
        lam = np.float32(1.0)
    delta = np.float32(np.rint(np.float32(-lo) / lam))
    return lam, delta


def quantize(x, lam, delta, bits=4):
    """Codes x_q in [0, 2^b - 1] as uint8, same shape as x."""
    x = np.asarray(x, dtype=np.float32)
    t = (x / np.float32(lam)).astype(np.float32) + np.float32(delta)
    q = np.rint(t.astype(np.float32))
    return np.clip(q, 0, 2 ** bits - 1).astype(np.uint8)


def dequantize(q, lam, delta):
    """x_hat = lambda * (x_q - delta) in fp32 (the difference is an exact small integer)."""
    return (np.float32(lam) * (np.asarray(q).astype(np.float32) - np.float32(delta))).astype(np.float32)


def pack_nibbles(q):
    """Rows of 4-bit codes [rows, k] -> bytes [rows, ceil(k/2)]: element l sits in byte l // 2,
    low nibble for even l, high nibble for odd l."""
    q = np.asarray(q, dtype=np.uint8)
    rows, k = q.shape
    if k % 2:
        q = np.concatenate([q, np.zeros((rows, 1), np.uint8)], axis=1)
    return (q[:, 0::2] | (q[:, 1::2] << 4)).astype(np.uint8)


def unpack_nibbles(b, k):
    b = np.asarray(b, dtype=np.uint8)
    q = np.empty((b.shape[0], b.shape[1] * 2), np.uint8)
    q[:, 0::2] = b & 15
    q[:, 1::2] = b >> 4
    return q[:, :k]
