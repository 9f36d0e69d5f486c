"""HIP path vs CPU oracle for the perturbation itself: Z = a G + b U R of every
kind of tensor, and the in-place passes theta <- rnd(theta + c Z) in fp32 and
bf16.  Tolerances: parameters within 1e-5 (fp32) / 1e-2 (bf16) relative."""
import numpy as np
import pytest

import zgr_inputs as I
from oracle import perturbation as P
from tests.util import make_session

pytestmark = pytest.mark.gpu

F32_RTOL, BF16_RTOL = 1e-5, 1e-2
PARAM_SCALE = 0.02          # std of the random init: the scale 'relative' refers to for values near zero


def _basis(rows, k, seed=0):
    q, r = np.linalg.qr(np.random.default_rng(seed).standard_normal((rows, k)))
    return (q * np.sign(np.diag(r))).astype(np.float32)


def _single_tensor_cfg(rows, cols, k, dtype="f32", scale_mode=0, ldu=None):
    return I.shrink(I.CONFIGS["cfg1"], name=f"t{rows}x{cols}k{k}", dtype=dtype, lsq_out=rows, lsq_in=cols, k=k,
                    k_full=ldu or k, scale_mode=scale_mode)


def _session_for(rows, cols, k, dtype="f32", bits=32, scale_mode=0, ldu=None, tensor_id=3):
    cfg = _single_tensor_cfg(rows, cols, k, dtype, scale_mode, ldu)
    spec = I.TensorSpec("W", I.ROLE_LSQ_W, -1, rows, cols, tensor_id, k > 0)
    rng = np.random.default_rng(rows * 131 + cols)
    W = (rng.standard_normal((rows, cols)) * PARAM_SCALE).astype(np.float32)
    if dtype == "bf16":
        W = P.bf16_round(W)
    U = _basis(rows, ldu or k, seed=rows + k) if k > 0 else None
    sess = make_session(cfg, [spec], [W], [U], bits=bits, arch=-1)
    return sess, cfg, W, U


def _z_bound(cfg, G, R, U, k, rows, cols, mode):
    """|Z_gpu - Z_oracle| allowed: 2 ulp on each Gaussian plus fp32 accumulation of the k-term dot."""
    if U is None or k == 0:
        return 2.0 * np.spacing(np.abs(G)) + 1e-45
    a, b = P.mix_coefficients(cfg.alpha, rows, cols, k, mode)
    absdot = np.abs(U[:, :k]).astype(np.float64) @ np.abs(R).astype(np.float64)
    return 2.0 ** -23 * (float(a) * np.abs(G) * 2 + (k + 4) * float(b) * absdot) + 1e-30


SHAPES = [
    # rows, cols, k, ldu
    (256, 512, 4, 4),       # cfg1
    (100, 72, 5, 5),        # ragged in both directions, odd k
    (300, 136, 16, 16),     # two row blocks of a tile, ragged tail
    (130, 256, 64, 64),     # maximum k
    (300, 136, 20, 20),     # matrix-core kernel with a rank that is no multiple of 8: the padded contraction steps are masked
    (200, 264, 36, 40),     # the same with a truncated basis (36 of 40 columns) and ragged tiles in both directions
    (70, 128, 17, 17),      # one step past the smallest matrix-core rank
    (64, 128, 8, 24),       # truncated basis: first 8 of 24 columns
    (1, 1000, 0, 0),        # 1-D, isotropic
    (1, 7, 0, 0),           # shorter than two Philox calls
    (3, 5, 0, 0),           # rows of a matrix straddling Philox calls
    (2, 1024, 0, 0),        # classification head: rows < k keeps it isotropic
]


@pytest.mark.parametrize("bits", [32, 16])
@pytest.mark.parametrize("rows,cols,k,ldu", SHAPES)
def test_z_matches_oracle(rows, cols, k, ldu, bits):
    if k > 0 and cols % (4 if bits == 32 else 8):
        pytest.skip("guided tensors need cols to be a multiple of the Philox group")
    for mode in (P.SCALE_UNIT, P.SCALE_PAPER):
        sess, cfg, W, U = _session_for(rows, cols, k, bits=bits, scale_mode=mode, ldu=ldu)
        step = 11
        got = sess.fill_z(0, step)
        G, R, Z = P.hybrid_z(cfg.seed, step, 3, rows, cols, U, k, cfg.alpha, mode, bits, parts=True)
        assert got.shape == Z.shape and np.all(np.isfinite(got))
        assert np.all(np.abs(got.astype(np.float64) - Z) <= _z_bound(cfg, G, R, U, k, rows, cols, mode))
        sess.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("rows,cols,k,ldu", SHAPES)
def test_inplace_pass_matches_oracle(rows, cols, k, ldu, dtype):
    sess, cfg, W, U = _session_for(rows, cols, k, dtype=dtype, ldu=ldu)
    step, c = 4, np.float32(1e-3)
    Z = P.hybrid_z(cfg.seed, step, 3, rows, cols, U, k, cfg.alpha, P.SCALE_UNIT, 32)
    want = W
    for coef in (c, np.float32(-2) * c, c, np.float32(-3.7e-4)):        # the four passes of a step + update
        sess.perturb(step, float(coef))
        want = P.axpy_inplace_value(want, coef, Z, dtype)
        got = sess.get_theta(0)
        if dtype == "f32":
            assert np.all(np.abs(got - want) <= F32_RTOL * (np.abs(want) + PARAM_SCALE))
            assert np.abs(got - want).max() <= 4e-9 + 4 * np.spacing(np.abs(want)).max()   # in fact within an ulp or two
        else:
            assert np.all(np.abs(got - want) <= BF16_RTOL * np.abs(want) + 1e-30)
            assert np.mean(got == want) > 0.98
        want = got          # later passes start from what the device holds, so errors do not compound in the check
    sess.close()


def test_set_basis_switches_between_guided_and_non_guided_rounds():
    rows, cols, k = 96, 64, 8
    sess, cfg, W, U = _session_for(rows, cols, k)
    G = P.gauss_field(cfg.seed, 2, 3, 0, rows, cols)
    Zg = P.hybrid_z(cfg.seed, 2, 3, rows, cols, U, k, cfg.alpha)
    assert np.allclose(sess.fill_z(0, 2), Zg, atol=2e-6)
    sess.set_basis(0, None, 0)                       # non-guided round: Z = G
    assert np.all(np.abs(sess.fill_z(0, 2) - G) <= 2 * np.spacing(np.abs(G)))
    U2 = _basis(rows, 4, seed=77)
    sess.set_basis(0, U2, 4)                         # a new basis from the cloud
    Z2 = P.hybrid_z(cfg.seed, 2, 3, rows, cols, U2, 4, cfg.alpha)
    assert np.allclose(sess.fill_z(0, 2), Z2, atol=2e-6)
    sess.close()


def test_alpha_one_and_identity_basis_special_cases():
    rows, cols = 32, 64
    cfg = I.shrink(_single_tensor_cfg(rows, cols, rows), alpha=0.36)
    spec = I.TensorSpec("W", I.ROLE_LSQ_W, -1, rows, cols, 3, True)
    W = np.zeros((rows, cols), np.float32)
    sess = make_session(cfg, [spec], [W], [np.eye(rows, dtype=np.float32)], arch=-1)
    G = P.gauss_field(cfg.seed, 0, 3, 0, rows, cols)
    R = P.gauss_field(cfg.seed, 0, 3, 1, rows, cols)
    assert np.allclose(sess.fill_z(0, 0), 0.6 * G + 0.8 * R, atol=3e-6)      # k = rows, U = I
    sess.close()
    cfg1 = I.shrink(cfg, alpha=1.0, k=4, k_full=4)
    sess = make_session(cfg1, [spec], [W], [_basis(rows, 4)], arch=-1)
    assert np.all(np.abs(sess.fill_z(0, 0) - G) <= 2 * np.spacing(np.abs(G)))  # alpha = 1: plain ZO-SGD direction
    sess.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("ranks", [(8, 16), (16, 4), (20, 5, 64)])
def test_mixed_ranks_in_one_context(ranks, dtype):
    """Tensors with ranks on both sides of 16 in one table: each rank class is served by its own kernel (matrix
    cores from 16 on, vector FMAs below), and every tensor's Z and in-place pass match the oracle."""
    from paper_2601_12917_amd.session import ParamSpec, Session
    rng = np.random.default_rng(sum(ranks))
    shapes = [(192, 256), (150, 136), (256, 128)][:len(ranks)]
    params, Ws, Us = [], [], []
    for j, ((rows, cols), k) in enumerate(zip(shapes, ranks)):
        W = (rng.standard_normal((rows, cols)) * PARAM_SCALE).astype(np.float32)
        if dtype == "bf16":
            W = P.bf16_round(W)
        U = _basis(rows, k, seed=40 + j)
        params.append(ParamSpec(f"W{j}", I.ROLE_LSQ_W, -1, 10 + j, W, U, k))
        Ws.append(W); Us.append(U)
    # plus an isotropic tensor, so the flat kernel runs in the same pass
    b = (rng.standard_normal((1, 300)) * PARAM_SCALE).astype(np.float32)
    if dtype == "bf16":
        b = P.bf16_round(b)
    params.append(ParamSpec("b", I.ROLE_B1, 0, 20, b))
    cfg = _single_tensor_cfg(1, 1, 1, dtype)
    sess = Session(-1, dtype, params, cfg.seed, cfg.eps, cfg.alpha, P.SCALE_UNIT, 32)
    step, c = 6, np.float32(1e-3)
    for j, ((rows, cols), k) in enumerate(zip(shapes, ranks)):
        G, R, Z = P.hybrid_z(cfg.seed, step, 10 + j, rows, cols, Us[j], k, cfg.alpha, P.SCALE_UNIT, 32, parts=True)
        got = sess.fill_z(j, step)
        assert np.all(np.abs(got.astype(np.float64) - Z) <= _z_bound(cfg, G, R, Us[j], k, rows, cols, P.SCALE_UNIT)), (j, k)
    sess.perturb(step, float(c))
    for j, ((rows, cols), k) in enumerate(zip(shapes, ranks)):
        Z = P.hybrid_z(cfg.seed, step, 10 + j, rows, cols, Us[j], k, cfg.alpha, P.SCALE_UNIT, 32)
        want = P.axpy_inplace_value(Ws[j], c, Z, dtype)
        got = sess.get_theta(j)
        if dtype == "f32":
            assert np.all(np.abs(got - want) <= F32_RTOL * (np.abs(want) + PARAM_SCALE)), (j, k)
        else:
            assert np.all(np.abs(got - want) <= BF16_RTOL * np.abs(want) + 1e-30) and np.mean(got == want) > 0.98, (j, k)
    want_b = P.axpy_inplace_value(b, c, P.gauss_field(cfg.seed, step, 20, 0, 1, 300), dtype)
    assert np.all(np.abs(sess.get_theta(len(ranks)) - want_b) <= (F32_RTOL if dtype == "f32" else BF16_RTOL) * (np.abs(want_b) + PARAM_SCALE))
    sess.close()
