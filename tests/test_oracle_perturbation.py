"""Pins for the oracle's hybrid perturbation Z = a G + b U R (Eq. (10)) and
the in-place storage arithmetic: subspace membership, covariance / trace
identity, special cases that reduce to plain Gaussians, and the bf16
rounding against torch's conversion."""
import numpy as np
import pytest
import torch

import zgr_inputs as I
from oracle import perturbation as P


def _basis(rows, k, seed=0):
    q, r = np.linalg.qr(np.random.default_rng(seed).standard_normal((rows, k)))
    return (q * np.sign(np.diag(r))).astype(np.float32)


def test_input_basis_is_orthonormal():
    cfg = I.CONFIGS["cfg1"]
    spec = I.tensor_specs(cfg)[0]
    U = I.make_basis(cfg, spec).astype(np.float64)
    assert U.shape == (256, 4)
    assert np.allclose(U.T @ U, np.eye(4), atol=1e-6)


@pytest.mark.parametrize("mode", [P.SCALE_UNIT, P.SCALE_PAPER])
def test_guided_component_lies_in_span_U(mode):
    rows, cols, k = 96, 40, 6
    U = _basis(rows, k)
    G, R, Z = P.hybrid_z(42, 1, 3, rows, cols, U, k, 0.3, mode, parts=True)
    a, b = P.mix_coefficients(0.3, rows, cols, k, mode)
    guided = Z.astype(np.float64) - np.float64(a) * G
    U64 = U.astype(np.float64)
    resid = guided - U64 @ (U64.T @ guided)
    assert np.abs(resid).max() <= 4e-7 * max(np.abs(Z).max(), np.abs(guided).max())
    assert np.linalg.matrix_rank(guided, tol=1e-5 * np.abs(guided).max()) == k
    # and its coordinates in the basis are b R
    assert np.allclose(U64.T @ guided, np.float64(b) * R, atol=5e-6 * float(b) + 1e-7)


def test_mix_coefficients_trace_identity():
    # alpha + (1 - alpha) = 1: E||Z||_F^2 = rows*cols (UNIT) or 1 (PAPER)
    for alpha in (0.0, 0.25, 0.5, 1.0):
        a, b = P.mix_coefficients(alpha, 256, 512, 4, P.SCALE_UNIT)
        assert np.isclose(a * a * 256 * 512 + b * b * 4 * 512, 256 * 512, rtol=1e-6)
        a, b = P.mix_coefficients(alpha, 256, 512, 4, P.SCALE_PAPER)
        assert np.isclose(float(a) ** 2 * 256 * 512 + float(b) ** 2 * 4 * 512, 1.0, rtol=1e-6)


def test_column_covariance_monte_carlo():
    """Each column of Z has covariance a^2 I + b^2 U U^T."""
    rows, cols, k, alpha = 12, 8, 3, 0.5
    U = _basis(rows, k, 3)
    a, b = P.mix_coefficients(alpha, rows, cols, k, P.SCALE_UNIT)
    acc = np.zeros((rows, rows))
    n_steps = 6000
    for t in range(n_steps):
        Z = P.hybrid_z(11, t, 1, rows, cols, U, k, alpha).astype(np.float64)
        acc += Z @ Z.T
    cov = acc / (n_steps * cols)
    want = float(a) ** 2 * np.eye(rows) + float(b) ** 2 * (U.astype(np.float64) @ U.T)
    # standard error of an entry ~ sqrt(2) * scale / sqrt(n_steps*cols)
    assert np.abs(cov - want).max() < 6 * np.sqrt(2.0) * want.max() / np.sqrt(n_steps * cols)
    assert np.isclose(np.trace(cov), rows, rtol=0.02)


def test_special_cases():
    rows, cols = 16, 24
    G = P.gauss_field(42, 5, 2, 0, rows, cols)
    # no basis / k = 0: non-guided round, Z = G
    assert np.array_equal(P.hybrid_z(42, 5, 2, rows, cols), G)
    assert np.array_equal(P.hybrid_z(42, 5, 2, rows, cols, _basis(rows, 4), 0), G)
    # alpha = 1: the guided term vanishes, Z = G (plain two-point ZO-SGD, Eq. (9))
    assert np.array_equal(P.hybrid_z(42, 5, 2, rows, cols, _basis(rows, 4), 4, alpha=1.0), G)
    # k = rows, U = I: Z = a G + b R, i.i.d. with variance a^2 + b^2 = 1
    R = P.gauss_field(42, 5, 2, 1, rows, cols)
    Z = P.hybrid_z(42, 5, 2, rows, cols, np.eye(rows, dtype=np.float32), rows, alpha=0.36)
    assert np.allclose(Z, 0.6 * G + 0.8 * R, atol=1e-6)
    # only the first k columns of a wider basis are used (truncated transmission)
    U8 = _basis(rows, 8)
    assert np.array_equal(P.hybrid_z(42, 5, 2, rows, cols, U8, 3), P.hybrid_z(42, 5, 2, rows, cols, U8[:, :3].copy(), 3))


def test_sampled_z_equals_field():
    rows, cols, k = 50, 36, 5
    U = _basis(rows, k)
    Z = P.hybrid_z(9, 4, 7, rows, cols, U, k, 0.5)
    rng = np.random.default_rng(0)
    i, j = rng.integers(0, rows, 200), rng.integers(0, cols, 200)
    zs = P.hybrid_z_at(9, 4, 7, rows, cols, i, j, U, k, 0.5)
    assert np.allclose(zs, Z[i, j], rtol=0, atol=3e-7 * np.abs(Z).max())
    Z16 = P.hybrid_z(9, 4, 7, rows, cols, U, k, 0.5, bits=16)
    assert np.allclose(P.hybrid_z_at(9, 4, 7, rows, cols, i, j, U, k, 0.5, bits=16), Z16[i, j], atol=3e-7 * np.abs(Z16).max())


def test_bf16_round_matches_torch():
    rng = np.random.default_rng(0)
    x = np.concatenate([
        rng.standard_normal(200000).astype(np.float32) * np.float32(0.02),
        rng.integers(0, 2 ** 31 - 2 ** 24, 200000, dtype=np.int64).astype(np.uint32).view(np.float32),
        # exact ties: low half == 0x8000 with even and odd upper halves
        np.array([0x3F808000, 0x3F818000, 0xBF808000, 0xBF818000, 0x00008000, 0x3F7FFFFF], dtype=np.uint32).view(np.float32),
    ])
    x = x[np.isfinite(x)]
    want = torch.from_numpy(x.copy()).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(P.bf16_round(x).view(np.uint32), want.view(np.uint32))


def test_axpy_value_is_one_fused_multiply_add():
    rng = np.random.default_rng(1)
    th = (rng.standard_normal(100000) * 0.02).astype(np.float32)
    z = rng.standard_normal(100000).astype(np.float32)
    c = np.float32(1e-3)
    got = P.axpy_inplace_value(th, c, z, "f32")
    exact = th.astype(np.float64) + np.float64(c) * z.astype(np.float64)
    # correctly rounded result of the exact sum: at most half an ulp away
    ulp = np.spacing(np.abs(got))
    assert np.all(np.abs(got.astype(np.float64) - exact) <= 0.5 * ulp * (1 + 1e-9))
    # bf16 storage: value is a bf16 number, at most half a bf16 ulp (<= 2^-8 relative, + the fp32 rounding) away
    thb = P.bf16_round(th)
    gb = P.axpy_inplace_value(thb, c, z, "bf16")
    assert np.array_equal(gb.view(np.uint32) & 0xFFFF, np.zeros_like(gb, dtype=np.uint32))
    exact = thb.astype(np.float64) + np.float64(c) * z.astype(np.float64)
    assert np.all(np.abs(gb - exact) <= np.abs(exact) * 2.0 ** -8 * (1 + 1e-3) + 1e-30)
