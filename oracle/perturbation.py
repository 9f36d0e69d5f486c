"""TEST INFRASTRUCTURE ONLY: CPU oracle, never imported by the product path.

Seeded hybrid perturbation of one parameter tensor (Sec. 3.2, Eq. (10) and
Algorithm 1, client block):

    z_h = sqrt(alpha/n) z + sqrt((1-alpha)/m) V z_g,
    z ~ N(0, I),  z_g ~ N(0, I_m),  V orthonormal basis of the gradient subspace.

Per weight matrix W [rows, cols] the basis is U [rows, k] and the subspace
coefficients are R [k, cols] (V = I_cols (x) U, m = k cols, n = rows cols), so
Z = a G + b U R with G [rows, cols] and R drawn from the shared seed.  In a
non-guided round, and for tensors without a basis, Z = G (Algorithm 1,
"use local perturbation").

Everything random is a pure function of (seed, step, tensor_id, stream,
flat element index) through Philox4x32-10 and Box-Muller, evaluated in fp64
and rounded once to fp32, so the edge server can regenerate exactly what the
client applied (Algorithm 1, edge-server block).

Counter layout (this repository's convention; the paper fixes none):
    element e = i*cols + j of stream s in {0: G, 1: R} of tensor id at step t
    32-bit mode: call q = e // 4, lane = e % 4
    16-bit mode: call q = e // 8, lane = e % 8
    ctr = (q mod 2^32, q >> 32, id | s << 31, t mod 2^32),  key = (seed mod 2^32, seed >> 32)
"""
import numpy as np

from .philox import philox4x32

SCALE_UNIT = 0    # Eq. (10) times sqrt(n): unit average variance per coordinate
SCALE_PAPER = 1   # Eq. (10) as printed


def counters(q, tensor_id: int, stream: int, step: int):
    q = np.asarray(q, dtype=np.uint64)
    ctr = np.empty(q.shape + (4,), dtype=np.uint64)
    ctr[..., 0] = q & np.uint64(0xFFFFFFFF)
    ctr[..., 1] = q >> np.uint64(32)
    ctr[..., 2] = np.uint64((int(tensor_id) & 0x7FFFFFFF) | (int(stream) << 31))
    ctr[..., 3] = np.uint64(int(step) & 0xFFFFFFFF)
    return ctr


def key_of(seed: int):
    return np.array([int(seed) & 0xFFFFFFFF, (int(seed) >> 32) & 0xFFFFFFFF], dtype=np.uint64)


def uniforms32(wa, wb):
    """Radius uniform u in (0,1) from the top 23 bits of wa (centred so that
    u is never 0 or 1) and angle uniform v in [0,1) from the top 24 bits of
    wb.  Both are exactly representable in fp32."""
    u = ((np.asarray(wa, dtype=np.uint64) >> np.uint64(9)).astype(np.float64) + 0.5) * 2.0 ** -23
    v = (np.asarray(wb, dtype=np.uint64) >> np.uint64(8)).astype(np.float64) * 2.0 ** -24
    return u, v


def uniforms16(ha, hb):
    u = (np.asarray(ha, dtype=np.float64) + 0.5) * 2.0 ** -16
    v = np.asarray(hb, dtype=np.float64) * 2.0 ** -16
    return u, v


def cos_sin_2pi(v):
    """cos(2 pi v), sin(2 pi v) for v in [0,1), exact in the quadrant: the
    angle is reduced to |r| <= 1/8 turn without rounding (v is a dyadic
    rational) so that zeros of either function come out as exact zeros and
    values next to them keep full relative accuracy."""
    v = np.asarray(v, dtype=np.float64)
    quad = np.rint(v * 4.0)
    r = v - quad * 0.25                      # exact, |r| <= 1/8
    q = quad.astype(np.int64) & 3
    c, s = np.cos(2.0 * np.pi * r), np.sin(2.0 * np.pi * r)
    cos_v = np.choose(q, [c, -s, -c, s])
    sin_v = np.choose(q, [s, c, -s, -c])
    return cos_v, sin_v


def box_muller(u, v):
    """(rho cos 2 pi v, rho sin 2 pi v) with rho = sqrt(-2 ln u), fp64 in,
    one rounding to fp32 out."""
    rho = np.sqrt(-2.0 * np.log(u))
    c, s = cos_sin_2pi(v)
    return (rho * c).astype(np.float32), (rho * s).astype(np.float32)


def gauss_at(seed: int, step: int, tensor_id: int, stream: int, e, bits: int = 32):
    """Standard normal value (fp32) of flat elements e (any integer array)."""
    e = np.asarray(e, dtype=np.uint64)
    per_call = 4 if bits == 32 else 8
    q = e // np.uint64(per_call)
    lane = (e % np.uint64(per_call)).astype(np.int64)
    w = philox4x32(counters(q, tensor_id, stream, step), key_of(seed)).astype(np.uint64)
    if bits == 32:
        pair = lane >> 1                                  # lanes (0,1) <- words (0,1); (2,3) <- (2,3)
        wa = np.take_along_axis(w, (2 * pair)[..., None], axis=-1)[..., 0]
        wb = np.take_along_axis(w, (2 * pair + 1)[..., None], axis=-1)[..., 0]
        u, v = uniforms32(wa, wb)
    elif bits == 16:
        pair = lane >> 1                                  # pair p <- word p: low half radius, high half angle
        wp = np.take_along_axis(w, pair[..., None], axis=-1)[..., 0]
        u, v = uniforms16(wp & np.uint64(0xFFFF), wp >> np.uint64(16))
    else:
        raise ValueError("bits must be 32 or 16")
    g_even, g_odd = box_muller(u, v)
    return np.where((lane & 1) == 0, g_even, g_odd).astype(np.float32)


def gauss_field(seed: int, step: int, tensor_id: int, stream: int, rows: int, cols: int,
                bits: int = 32, chunk: int = 1 << 22):
    """All rows*cols Gaussians of one stream, as fp32 [rows, cols]."""
    n = rows * cols
    out = np.empty(n, dtype=np.float32)
    for lo in range(0, n, chunk):
        hi = min(n, lo + chunk)
        out[lo:hi] = gauss_at(seed, step, tensor_id, stream, np.arange(lo, hi, dtype=np.uint64), bits)
    return out.reshape(rows, cols)


def mix_coefficients(alpha: float, rows: int, cols: int, k: int, scale_mode: int):
    """(a, b) of Z = a G + b U R, rounded to fp32.  PAPER: Eq. (10) with
    n = rows*cols and m = k*cols.  UNIT: the same times sqrt(n), so that the
    mean variance per coordinate is alpha + (1 - alpha) = 1, which is the
    scale of the non-guided z ~ N(0, I)."""
    if scale_mode == SCALE_UNIT:
        a, b = np.sqrt(alpha), np.sqrt((1.0 - alpha) * rows / k)
    elif scale_mode == SCALE_PAPER:
        a, b = np.sqrt(alpha / (rows * cols)), np.sqrt((1.0 - alpha) / (k * cols))
    else:
        raise ValueError("scale_mode")
    return np.float32(a), np.float32(b)


def hybrid_z(seed: int, step: int, tensor_id: int, rows: int, cols: int, U=None, k: int = 0,
             alpha: float = 0.5, scale_mode: int = SCALE_UNIT, bits: int = 32, parts: bool = False):
    """Z [rows, cols] fp32.  U: [rows, >=k] (first k columns are used) or None."""
    G = gauss_field(seed, step, tensor_id, 0, rows, cols, bits)
    if U is None or k == 0:
        return (G, None, G) if parts else G
    R = gauss_field(seed, step, tensor_id, 1, k, cols, bits)
    a, b = mix_coefficients(alpha, rows, cols, k, scale_mode)
    Uk = np.asarray(U, dtype=np.float64)[:, :k]
    Z = (np.float64(a) * G.astype(np.float64) + np.float64(b) * (Uk @ R.astype(np.float64))).astype(np.float32)
    return (G, R, Z) if parts else Z


def hybrid_z_at(seed: int, step: int, tensor_id: int, rows: int, cols: int, i, j, U=None, k: int = 0,
                alpha: float = 0.5, scale_mode: int = SCALE_UNIT, bits: int = 32):
    """Z at sampled positions (i[n], j[n]) of a large tensor, one by one."""
    i = np.asarray(i, dtype=np.int64)
    j = np.asarray(j, dtype=np.int64)
    G = gauss_at(seed, step, tensor_id, 0, i * cols + j, bits)
    if U is None or k == 0:
        return G
    l = np.arange(k, dtype=np.int64)
    R = gauss_at(seed, step, tensor_id, 1, l[None, :] * cols + j[:, None], bits)      # [n, k]
    a, b = mix_coefficients(alpha, rows, cols, k, scale_mode)
    Ui = np.asarray(U, dtype=np.float64)[i, :k]
    ur = np.sum(Ui * R.astype(np.float64), axis=1)
    return (np.float64(a) * G.astype(np.float64) + np.float64(b) * ur).astype(np.float32)


# ---------------------------------------------------------------- storage types

def bf16_round(x):
    """fp32 -> nearest bf16 (ties to even), returned as fp32.  Finite inputs."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    b = b + np.uint64(0x7FFF) + ((b >> np.uint64(16)) & np.uint64(1))
    b = (b & np.uint64(0xFFFF0000)).astype(np.uint32)
    return b.view(np.float32)


def axpy_inplace_value(theta, c, Z, dtype: str):
    """theta + c Z as the in-place pass stores it: one fp32 fused
    multiply-add, then, for bf16 storage, one round-to-nearest-even.
    theta is fp32 (holding bf16 values when dtype == 'bf16')."""
    t = (np.float64(np.float32(c)) * Z.astype(np.float64) + theta.astype(np.float64)).astype(np.float32)
    if dtype == "bf16":
        t = bf16_round(t)
    elif dtype != "f32":
        raise ValueError("dtype")
    return t
