"""HIP path vs CPU oracle for the compressed basis (Sec. 3.4, first equation): the device quantiser's
4-bit codes, lambda and delta bit for bit, and Z = a G + b U_hat R with U_hat restored from the codes
inside the kernels, in the VALU (k < 16) and the matrix-core (k >= 16) tile kernels."""
import numpy as np
import pytest

from oracle import dtc as D
from oracle import perturbation as P
from tests.test_gpu_perturb import PARAM_SCALE, _basis, _session_for, _z_bound

pytestmark = pytest.mark.gpu

CASES = [
    # rows, cols, k, ldu
    (256, 512, 4, 4),
    (100, 72, 5, 5),        # odd k: the last byte of a row holds one code
    (300, 136, 16, 16),     # matrix cores, ragged tile
    (130, 256, 64, 64),
    (64, 128, 8, 24),       # truncated basis: codes of the first 8 of 24 columns
    (2048, 256, 16, 64),    # several row blocks, k' = 16 of 64 as in the largest workload
]


@pytest.mark.parametrize("rows,cols,k,ldu", CASES)
def test_device_quantiser_matches_oracle_bit_for_bit(rows, cols, k, ldu):
    sess, cfg, W, U = _session_for(rows, cols, k, ldu=ldu)
    q_dev, lam_dev, delta_dev = sess.quantize_basis(U, k)
    lam, delta = D.affine_params(U[:, :k], 4)
    assert np.float32(lam_dev) == lam and np.float32(delta_dev) == delta
    want = D.pack_nibbles(D.quantize(U[:, :k], lam, delta, 4))
    assert q_dev.shape == want.shape and np.array_equal(q_dev, want)
    codes = D.unpack_nibbles(q_dev, k)
    assert codes.min() == 0 and codes.max() == 15
    sess.close()


@pytest.mark.parametrize("bits", [32, 16])
@pytest.mark.parametrize("rows,cols,k,ldu", CASES)
def test_z_with_restored_basis_matches_oracle(rows, cols, k, ldu, bits):
    if cols % (4 if bits == 32 else 8):
        pytest.skip("guided tensors need cols to be a multiple of the Philox group")
    sess, cfg, W, U = _session_for(rows, cols, k, bits=bits, ldu=ldu)
    lam, delta = D.affine_params(U[:, :k], 4)
    codes = D.quantize(U[:, :k], lam, delta, 4)
    Uh = D.dequantize(codes, lam, delta)
    sess.set_basis_q4(0, D.pack_nibbles(codes), k, lam, delta)
    step = 7
    got = sess.fill_z(0, step)
    G, R, Z = P.hybrid_z(cfg.seed, step, 3, rows, cols, Uh, k, cfg.alpha, P.SCALE_UNIT, bits, parts=True)
    assert np.all(np.isfinite(got))
    assert np.all(np.abs(got.astype(np.float64) - Z) <= _z_bound(cfg, G, R, Uh, k, rows, cols, P.SCALE_UNIT))
    # it is the restored basis that is used, not the original: the two Z differ by far more than the bound
    Z0 = P.hybrid_z(cfg.seed, step, 3, rows, cols, U, k, cfg.alpha, P.SCALE_UNIT, bits)
    assert np.abs(Z - Z0).max() > 100 * _z_bound(cfg, G, R, Uh, k, rows, cols, P.SCALE_UNIT).max()
    # switching back to the fp32 basis restores the uncompressed Z
    sess.set_basis(0, U, k)
    got0 = sess.fill_z(0, step)
    assert np.all(np.abs(got0.astype(np.float64) - Z0) <= _z_bound(cfg, G, R, U, k, rows, cols, P.SCALE_UNIT))
    sess.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_inplace_pass_and_batched_update_with_restored_basis(dtype):
    rows, cols, k = 384, 256, 16
    sess, cfg, W, U = _session_for(rows, cols, k, dtype=dtype)
    lam, delta = D.affine_params(U, 4)
    codes = D.quantize(U, lam, delta, 4)
    Uh = D.dequantize(codes, lam, delta)
    sess.set_basis_q4(0, D.pack_nibbles(codes), k, lam, delta)
    c = np.float32(1e-3)
    sess.perturb(5, float(c))
    Z = P.hybrid_z(cfg.seed, 5, 3, rows, cols, Uh, k, cfg.alpha, P.SCALE_UNIT, 32)
    want = P.axpy_inplace_value(W, c, Z, dtype)
    got = sess.get_theta(0)
    if dtype == "f32":
        assert np.all(np.abs(got - want) <= 1e-5 * (np.abs(want) + PARAM_SCALE))
    else:
        assert np.all(np.abs(got - want) <= 1e-2 * np.abs(want) + 1e-30) and np.mean(got != want) < 0.005
    sess.close()


def test_q4_basis_rejects_bad_arguments():
    sess, cfg, W, U = _session_for(64, 128, 8)
    lam, delta = D.affine_params(U, 4)
    packed = D.pack_nibbles(D.quantize(U, lam, delta, 4))
    with pytest.raises(Exception):
        sess.set_basis_q4(0, packed, 16, lam, delta)          # ldq = 4 bytes < 8
    with pytest.raises(Exception):
        sess.set_basis_q4(0, packed, 8, 0.0, delta)           # lambda must be positive
    with pytest.raises(Exception):
        sess.set_basis_q4(3, packed, 8, lam, delta)           # no such tensor
    sess.set_basis_q4(0, packed, 8, lam, delta)
    sess.close()
