"""Pins of the affine quantiser (Sec. 3.4, first equation) against closed forms."""
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


# ------------------------------------------------------------------ how much to compress (Sec. 3.4)

def test_omega_zero_when_plain_transfer_already_hides():
    # 1 MB over 1 GB/s = 1 ms <= T_cc = 2 ms
    w, ok = D.choose_omega(1e6, 1e9, 2e-3, 0.0, 0.125)
    assert w == 0.0 and ok


def test_omega_closed_form_with_free_restore():
    # restore costs nothing: D0 (1 - w (1 - theta)) / B0 = T_cc  ->  w = (1 - T_cc B0 / D0) / (1 - theta)
    D0, B0, Tcc, theta = 8e6, 1e9, 3e-3, 0.125
    w, ok = D.choose_omega(D0, B0, Tcc, 0.0, theta)
    assert ok and abs(w - (1 - Tcc * B0 / D0) / (1 - theta)) < 1e-12
    # at that omega the two sides meet
    assert abs(D.transfer_time(D0, B0, w, theta) - D.client_time(Tcc, D0, w, 0.0)) < 1e-15


def test_omega_closed_form_with_restore_cost():
    D0, B0, Tcc, tau, theta = 4e6, 5e8, 2e-3, 1e-10, 0.25
    w, ok = D.choose_omega(D0, B0, Tcc, tau, theta)
    want = (D0 / B0 - Tcc) / (D0 * (1 - theta) / B0 + tau * D0)
    assert ok and 0 < want < 1 and abs(w - want) < 1e-12


def test_omega_saturates_when_even_full_compression_cannot_hide():
    # 10 Mbit/s link (1.25e6 B/s), 1 MB, theta = 1/8: 0.1 s even when everything is compressed, T_cc = 1 ms
    w, ok = D.choose_omega(1e6, 1.25e6, 1e-3, 0.0, 0.125)
    assert w == 1.0 and not ok


def test_omega_is_the_smallest_on_a_grid_and_monotone_in_bandwidth():
    D0, Tcc, tau, theta = 6e6, 1e-3, 2e-11, 0.125
    prev = 2.0
    for B0 in (1e9, 2e9, 4e9, 8e9):
        w, ok = D.choose_omega(D0, B0, Tcc, tau, theta)
        grid = np.linspace(0, 1, 100001)
        good = D.transfer_time(D0, B0, grid, theta) <= D.client_time(Tcc, D0, grid, tau)
        assert ok == bool(good.any())
        if ok:
            assert abs(grid[np.argmax(good)] - w) <= 1e-5 + 1e-12
        assert w <= prev          # a faster link never needs more compression
        prev = w


def test_memory_factor_matches_the_printed_relations():
    # layer pipeline alone: (1 + 2/L); with compression: minus omega (1 - theta) / L
    assert D.memory_factor(24, 0.0, 0.125) == pytest.approx(1 + 2 / 24)
    assert D.memory_factor(24, 1.0, 0.125) == pytest.approx(1 + 2 / 24 - 0.875 / 24)
    assert D.memory_factor(12, 0.5, 0.25) == pytest.approx(1 + 2 / 12 - 0.5 * 0.75 / 12)
