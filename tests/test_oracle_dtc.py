"""Pins of the affine quantiser (Sec. 4.4, first equation) against closed forms."""
import numpy as np
import pytest

from oracle import dtc as D
from oracle import perturbation as P


def test_grid_values_round_trip_exactly():
    # min = -1.5, max = 2.25, 4 bits: lambda = 0.25, delta = 6; the 16 grid points are their own codes
    x = (-1.5 + 0.25 * np.arange(16)).astype(np.float32)
    lam, delta = D.affine_params(x, 4)
    assert lam == np.float32(0.25) and delta == np.float32(6.0)
    q = D.quantize(x, lam, delta, 4)
    assert np.array_equal(q, np.arange(16, dtype=np.uint8))
    assert np.array_equal(D.dequantize(q, lam, delta), x)


def test_identity_on_integer_range():
    x = np.arange(16, dtype=np.float32)[::-1].copy()
    lam, delta = D.affine_params(x, 4)
    assert lam == 1 and delta == 0
    assert np.array_equal(D.quantize(x, lam, delta), x.astype(np.uint8))
    x8 = np.arange(256, dtype=np.float32)
    lam, delta = D.affine_params(x8, 8)
    assert lam == 1 and delta == 0 and np.array_equal(D.dequantize(D.quantize(x8, lam, delta, 8), lam, delta), x8)


@pytest.mark.parametrize("bits", [4, 8])
def test_error_bound_monotonicity_and_range(bits):
    g = np.random.default_rng(5)
    x = (g.standard_normal((300, 16)) * 0.07).astype(np.float32)
    lam, delta = D.affine_params(x, bits)
    assert np.isclose(lam, (x.max() - x.min()) / (2 ** bits - 1), rtol=1e-6)
    q = D.quantize(x, lam, delta, bits)
    assert q.min() == 0 and q.max() == 2 ** bits - 1 and q.dtype == np.uint8
    xh = D.dequantize(q, lam, delta)
    # half a step from rounding x, up to half a step more from the rounding of delta at the clipped ends
    assert np.all(np.abs(xh - x) <= 0.5 * lam * (1 + 1e-5) + 0.5 * lam * ((q == 0) | (q == 2 ** bits - 1)))
    assert np.abs(xh - x).max() > 0.4 * lam                    # a dropped delta or a truncation instead of round would show
    order = np.argsort(x, axis=None)
    assert np.all(np.diff(q.reshape(-1)[order].astype(int)) >= 0)
    # ties to even at the half-way points between codes
    mid = (np.float32(lam) * (np.arange(2 ** bits - 1, dtype=np.float32) + np.float32(0.5) - delta)).astype(np.float32)
    qm = D.quantize(mid, lam, delta, bits).astype(int)
    exact = (mid / lam).astype(np.float32) + delta
    is_tie = exact == np.floor(exact) + 0.5
    assert np.all(qm[is_tie] % 2 == 0)


def test_constant_tensor_and_packing():
    x = np.full((3, 5), 0.25, np.float32)
    lam, delta = D.affine_params(x)
    assert lam == 1 and np.all(np.abs(D.dequantize(D.quantize(x, lam, delta), lam, delta) - x) <= 0.5)
    q = np.arange(15, dtype=np.uint8).reshape(3, 5)
    b = D.pack_nibbles(q)
    assert b.shape == (3, 3) and b[0, 0] == (0 | (1 << 4)) and b[0, 2] == 4
    assert np.array_equal(D.unpack_nibbles(b, 5), q)


def test_quantised_basis_keeps_the_guided_term_in_its_span():
    """Z - a G = b U_hat R lies in span(U_hat); U_hat is close to U: ||U_hat^T U_hat - I|| = O(lambda sqrt(rows))."""
    g = np.random.default_rng(3)
    U = np.linalg.qr(g.standard_normal((96, 8)))[0].astype(np.float32)
    lam, delta = D.affine_params(U)
    Uh = D.dequantize(D.quantize(U, lam, delta), lam, delta)
    assert np.abs(Uh - U).max() <= 0.5001 * lam + 0.5 * lam
    gram = Uh.astype(np.float64).T @ Uh.astype(np.float64)
    assert np.abs(gram - np.eye(8)).max() < 0.25
    a, b = P.mix_coefficients(0.5, 96, 40, 8, P.SCALE_UNIT)
    Z = P.hybrid_z(42, 3, 9, 96, 40, Uh, 8, 0.5, P.SCALE_UNIT, 32)
    G = P.gauss_field(42, 3, 9, 0, 96, 40, 32)
    guided = Z.astype(np.float64) - a * G.astype(np.float64)
    Q, _ = np.linalg.qr(Uh.astype(np.float64))
    resid = guided - Q @ (Q.T @ guided)
    assert np.abs(resid).max() <= 1e-5 * np.abs(guided).max()
