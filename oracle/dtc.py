"""TEST INFRASTRUCTURE ONLY: CPU oracle, never imported by the product path.

b-bit affine quantisation of the guided basis for transmission (Data Transmission
Controller, Sec. 3.4, the quantise / restore pair of its first equation):

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


# ----------------------------------------------------------------------------------------------------
# How much to compress (Data Transmission Controller, Sec. 3.4, the three latency relations and the
# memory relation that close the section).  A layer's guided data of D0 bytes crosses a link of B0
# bytes/s; a share omega of it travels compressed to theta of its size and costs the client T(D0 omega)
# of restoring on top of its computation T_cc; the transfer hides when T_t <= T_cc + T(D0 omega).
# Reading: the paper prints T_t = D0 / B0, which does not depend on omega; the transfer time of partly
# compressed data, D0 (1 - omega (1 - theta)) / B0, is used (the same factor omega (1 - theta) appears in
# the printed memory relation).  T is taken linear in its argument ("obtained offline": one figure per byte).

def transfer_time(data_bytes, bandwidth, omega, theta):
    return data_bytes * (1.0 - omega * (1.0 - theta)) / bandwidth


def client_time(t_cc, data_bytes, omega, restore_s_per_byte):
    return t_cc + restore_s_per_byte * data_bytes * omega


def choose_omega(data_bytes, bandwidth, t_cc, restore_s_per_byte, theta, iters=200):
    """Smallest omega in [0, 1] for which the transfer hides, and whether it does at that omega.
    transfer - client is non-increasing in omega, so the set of good omegas is an interval ending at 1."""
    def gap(w):
        return transfer_time(data_bytes, bandwidth, w, theta) - client_time(t_cc, data_bytes, w, restore_s_per_byte)
    if gap(0.0) <= 0.0:
        return 0.0, True
    if gap(1.0) > 0.0:
        return 1.0, False
    lo, hi = 0.0, 1.0          # gap(lo) > 0 >= gap(hi)
    for _ in range(iters):
        mid = 0.5 * (lo + hi)
        if gap(mid) > 0.0:
            lo = mid
        else:
            hi = mid
    return hi, True


def memory_factor(n_layers, omega, theta):
    """Client memory in units of Mem_0: (1 + 2/L) with the layer pipeline alone (omega = 0),
    (1 + 2/L - omega (1 - theta) / L) with compression."""
    return 1.0 + 2.0 / n_layers - omega * (1.0 - theta) / n_layers
