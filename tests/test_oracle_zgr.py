"""Pins for the oracle's ZGR step (Algorithm 1, Eq. (11)): the central
difference of a quadratic loss equals <grad L, Z> exactly, the brute-force
directional derivative of the transformer loss matches autograd's gradient
contracted with Z, the estimator's mean, collinearity of the update with Z,
restore error bounds, and replay of a trajectory from its scalar log."""
import numpy as np
import pytest
import torch
import torch.nn.functional as TF

import zgr_inputs as I
from oracle import forward as F
from oracle import perturbation as P
from oracle.zgr import Tensor, ZgrOracle, make_lm_loss, make_lsq_loss


def _cfg1_oracle(dtype="f32", eps=1e-3, alpha=0.5, k=None, scale_mode=P.SCALE_UNIT, bits=32):
    """cfg1's data; the default here is the unit-variance scaling (cfg1 itself runs Eq. (10) as printed)."""
    cfg = I.CONFIGS["cfg1"]
    spec = I.tensor_specs(cfg)[0]
    W = I.make_params(cfg)[0]
    U = I.make_basis(cfg, spec)
    X, Y = I.make_lsq_data(cfg)
    k = cfg.k if k is None else k
    t = Tensor("W", W, spec.tensor_id, U if k > 0 else None, k)
    return ZgrOracle([t], make_lsq_loss(X, Y), cfg.seed, eps, alpha, dtype, scale_mode, bits), X, Y


@pytest.mark.parametrize("eps", [1e-3, 0.25])
def test_central_difference_of_quadratic_is_exact_directional_derivative(eps):
    """The LSQ loss is quadratic, so (L+ - L-)/(2 eps) = <grad L, Z> for any eps."""
    o, X, Y = _cfg1_oracle(eps=eps)
    # evaluate in fp64 on the exact (unrounded) perturbed points
    W = o.tensors[0].theta.astype(np.float64)
    Z = o.z_of(o.tensors[0], 0).astype(np.float64)
    e = float(o.eps)
    g_fd = (F.lsq_loss(W + e * Z, X, Y) - F.lsq_loss(W - e * Z, X, Y)) / (2 * e)
    X64, Y64 = X.astype(np.float64), Y.astype(np.float64)
    grad = (X64 @ W.T - Y64).T @ X64 / X.shape[0]
    assert np.isclose(g_fd, np.sum(grad * Z), rtol=1e-6 if eps < 0.1 else 1e-10)
    # the oracle's step (fp32 storage of the perturbed weights) gives the same g
    lp, lm, g = o.step(0)
    assert np.isclose(g, np.sum(grad * Z), rtol=2e-3 if eps < 0.1 else 1e-5)
    assert lp != lm


def test_step_restores_parameters_fp32_and_bf16():
    o, _, _ = _cfg1_oracle()
    before = o.tensors[0].theta.copy()
    o.step(3)
    after = o.tensors[0].theta
    Z = o.z_of(o.tensors[0], 3)
    bound = 2 * np.spacing(np.abs(before) + np.float32(1e-3) * np.abs(Z))
    assert np.all(np.abs(after - before) <= bound)
    assert np.mean(after == before) > 0.5
    ob, _, _ = _cfg1_oracle(dtype="bf16")
    ob.tensors[0].theta = P.bf16_round(ob.tensors[0].theta)
    before = ob.tensors[0].theta.copy()
    ob.step(3)
    after = ob.tensors[0].theta
    # three roundings to bf16, each at most 2^-8 relative to a value of size <= |theta| + eps |Z|
    assert np.array_equal(after.view(np.uint32) & 0xFFFF, np.zeros(after.shape, np.uint32))
    Zb = ob.z_of(ob.tensors[0], 3)
    assert np.all(np.abs(after - before) <= 3.1 * 2.0 ** -8 * (np.abs(before) + 1e-3 * np.abs(Zb)))
    assert np.mean(after == before) > 0.3


def test_fused_restore_update_equals_restore_then_update():
    """One pass with eps - lr g equals the restoring pass followed by the update: in fp32 to rounding,
    and against the exact theta0 - lr g Z it is at least as close as the two-pass sequence."""
    lr = 1e-2
    a, _, _ = _cfg1_oracle()
    b, _, _ = _cfg1_oracle()
    theta0 = a.tensors[0].theta.astype(np.float64)
    lp, lm, g = a.step(5)
    a.apply_update(5, g, lr)
    lp2, lm2, g2 = b.step(5, fuse_lr=lr)
    assert (lp, lm, g) == (lp2, lm2, g2) and g != 0
    Z = a.z_of(a.tensors[0], 5).astype(np.float64)
    exact = theta0 - np.float64(np.float32(lr) * g) * Z
    scale = np.spacing(np.maximum(np.abs(theta0) + 1e-3 * np.abs(Z), np.abs(exact)).astype(np.float32))
    # storage roundings (three against two) plus, fused, the rounding of the coefficient eps - lr g
    assert np.all(np.abs(a.tensors[0].theta - exact) <= 3 * scale)
    assert np.all(np.abs(b.tensors[0].theta - exact) <= 3 * scale)
    # a wrong sign of the lr g term would move theta the other way
    assert np.sum((b.tensors[0].theta - theta0) * (-g * Z)) > 0
    # bf16 storage: same statement with bf16 spacing
    ab, _, _ = _cfg1_oracle(dtype="bf16"); bb, _, _ = _cfg1_oracle(dtype="bf16")
    for o in (ab, bb):
        o.tensors[0].theta = P.bf16_round(o.tensors[0].theta)
    t0 = ab.tensors[0].theta.astype(np.float64)
    _, _, gb = ab.step(5); ab.apply_update(5, gb, lr)
    _, _, gb2 = bb.step(5, fuse_lr=lr)
    assert gb == gb2
    Zb = ab.z_of(ab.tensors[0], 5).astype(np.float64)
    exact = t0 - np.float64(np.float32(lr) * gb) * Zb
    mag = np.maximum(np.abs(t0) + 1e-3 * np.abs(Zb), np.abs(exact))
    assert np.all(np.abs(bb.tensors[0].theta - exact) <= 3.1 * 2.0 ** -8 * mag)
    assert np.abs(bb.tensors[0].theta - exact).mean() <= np.abs(ab.tensors[0].theta - exact).mean()
    assert np.array_equal(bb.tensors[0].theta.view(np.uint32) & 0xFFFF, np.zeros(t0.shape, np.uint32))


def test_batched_update_is_the_sum_of_single_updates():
    """theta - lr sum_q g_q Z_q in one pass: n = 1 is apply_update bit for bit; n = 3 matches three
    successive updates to a few roundings, is within one rounding of the exact sum, and in bf16 is closer
    to the exact sum than three passes that each round to bf16."""
    steps, gs = [4, 9, 2], [0.75, -1.5, 0.3125]
    for dtype in ("f32", "bf16"):
        lr = 1e-2 if dtype == "f32" else 2.0          # large enough to move bf16 weights by many ulps
        a, _, _ = _cfg1_oracle(dtype=dtype); b, _, _ = _cfg1_oracle(dtype=dtype); c, _, _ = _cfg1_oracle(dtype=dtype)
        if dtype == "bf16":
            for o in (a, b, c):
                o.tensors[0].theta = P.bf16_round(o.tensors[0].theta)
        theta0 = a.tensors[0].theta.astype(np.float64)
        a.apply_update(7, gs[0], lr); b.apply_updates([7], [gs[0]], lr)
        assert np.array_equal(a.tensors[0].theta, b.tensors[0].theta)
        a.tensors[0].theta = theta0.astype(np.float32); b.tensors[0].theta = theta0.astype(np.float32)
        for s, g in zip(steps, gs):
            a.apply_update(s, g, lr)
        b.apply_updates(steps, gs, lr)
        exact = theta0.copy()
        mag = np.abs(theta0)
        for s, g in zip(steps, gs):
            term = np.float64(np.float32(np.float32(lr) * np.float32(g))) * c.z_of(c.tensors[0], s).astype(np.float64)
            exact -= term
            mag = mag + np.abs(term)
        ulp_mag = np.spacing(mag.astype(np.float32)).astype(np.float64) * (1.0 if dtype == "f32" else 2.0 ** 16)
        ulp = np.spacing(np.abs(exact).astype(np.float32)).astype(np.float64) * (1.0 if dtype == "f32" else 2.0 ** 16)
        assert np.all(np.abs(b.tensors[0].theta - exact) <= 0.5001 * ulp + 1e-12)          # one rounding (+ the fp32 one)
        assert np.all(np.abs(a.tensors[0].theta - b.tensors[0].theta) <= 2.0 * ulp_mag)    # three roundings at intermediate magnitudes
        assert np.abs(b.tensors[0].theta - exact).mean() <= np.abs(a.tensors[0].theta - exact).mean()
        assert np.mean(np.abs(b.tensors[0].theta - theta0) > 4 * ulp) > 0.5                 # the update is not a no-op
    # the same step twice is one step with the summed coefficient (linearity in g)
    d1, _, _ = _cfg1_oracle(); d2, _, _ = _cfg1_oracle()
    d1.apply_updates([5, 5], [0.5, 0.25], 1e-2); d2.apply_updates([5], [0.75], 1e-2)
    assert np.allclose(d1.tensors[0].theta, d2.tensors[0].theta, rtol=0, atol=2e-8)


def test_update_is_collinear_with_z():
    o, _, _ = _cfg1_oracle()
    before = o.tensors[0].theta.astype(np.float64)
    g, lr = np.float32(0.37), np.float32(1e-2)
    o.apply_update(2, g, lr)
    d = o.tensors[0].theta.astype(np.float64) - before
    Z = o.z_of(o.tensors[0], 2).astype(np.float64)
    c = -float(np.float32(lr * g))
    assert np.allclose(d, c * Z, rtol=0, atol=8e-9)     # half an fp32 ulp of theta ~ 0.1
    assert np.isclose(np.sum(d * Z), c * np.sum(Z * Z), rtol=1e-6)


def test_alpha_one_is_plain_two_point_zo_sgd():
    o1, _, _ = _cfg1_oracle(alpha=1.0)
    o0, _, _ = _cfg1_oracle(k=0)
    assert o1.step(0) == o0.step(0)


def test_estimator_mean_is_preconditioned_gradient():
    """E[g Z] = (a^2 I + b^2 U U^T) grad L, column-wise (Eq. (11) with Eq. (10))."""
    rng = np.random.default_rng(0)
    rows, cols, k, B, alpha = 8, 16, 2, 6, 0.5
    W = (rng.standard_normal((rows, cols)) * 0.3).astype(np.float32)
    X = rng.standard_normal((B, cols)).astype(np.float32)
    Y = rng.standard_normal((B, rows)).astype(np.float32)
    q, r = np.linalg.qr(rng.standard_normal((rows, k)))
    U = (q * np.sign(np.diag(r))).astype(np.float32)
    t = Tensor("W", W, 1, U, k)
    o = ZgrOracle([t], make_lsq_loss(X, Y), 7, 1e-2, alpha)
    W64, X64, Y64 = W.astype(np.float64), X.astype(np.float64), Y.astype(np.float64)
    grad = (X64 @ W64.T - Y64).T @ X64 / B
    a, b = P.mix_coefficients(alpha, rows, cols, k, P.SCALE_UNIT)
    want = (float(a) ** 2 * np.eye(rows) + float(b) ** 2 * U.astype(np.float64) @ U.T) @ grad
    n, acc = 12000, np.zeros((rows, cols))
    for s in range(n):
        Z = o.z_of(t, s).astype(np.float64)
        acc += np.sum(grad * Z) * Z           # quadratic loss: g = <grad, Z> exactly
    est = acc / n
    err = np.linalg.norm(est - want) / np.linalg.norm(want)
    assert err < 0.08
    # without the guided covariance the match is much worse: the test can tell the two apart
    assert np.linalg.norm(est - grad) / np.linalg.norm(grad) > 3 * err


def test_directional_derivative_of_transformer_loss_matches_autograd():
    """Brute force: (L(th + hZ) - L(th - hZ))/(2h) -> <grad L, Z> as O(h^2), with the
    gradient from torch autograd on library layers."""
    cfg = I.shrink(I.CONFIGS["cfg2"], name="tiny_lm_dd", n_layer=1, d_model=16, n_head=2, d_ff=32, vocab=37,
                   max_pos=8, batch=2, seq=8, k=2, k_full=2)
    specs = I.tensor_specs(cfg)
    vals = [v * np.float32(10.0) if s.role not in (I.ROLE_LN1_G, I.ROLE_LN2_G, I.ROLE_LNF_G) else v
            for s, v in zip(specs, I.make_params(cfg, 0, specs))]
    tokens = I.make_tokens(cfg)
    tens = [Tensor(s.name, v, s.tensor_id, I.make_basis(cfg, s), cfg.k if s.guided else 0) for s, v in zip(specs, vals)]
    assert sum(t.k > 0 for t in tens) == 6
    o = ZgrOracle(tens, make_lm_loss(tokens, cfg.n_layer, cfg.n_head), 42, 1e-3, 0.5)
    Zs = {t.name: o.z_of(t, 0).astype(np.float64) for t in tens}
    base = {t.name: t.theta.astype(np.float64) for t in tens}

    def L(h):
        return o.loss_fn({n: base[n] + h * Zs[n] for n in base})

    # autograd gradient of the same loss written with torch ops
    Pt = {n: torch.tensor(v, requires_grad=True) for n, v in base.items()}
    tok = torch.tensor(tokens, dtype=torch.long)
    x = Pt["tok_emb"][tok] + Pt["pos_emb"][: cfg.seq][None]
    d, H = cfg.d_model, cfg.n_head
    ln = lambda x, g, b: TF.layer_norm(x, (d,), Pt[g].reshape(-1), Pt[b].reshape(-1), cfg.ln_eps)
    h1 = ln(x, "l0.ln1_g", "l0.ln1_b")
    q, k_, v = (TF.linear(h1, Pt[f"l0.w{c}"], Pt[f"l0.b{c}"].reshape(-1)) for c in "qkv")
    sp = lambda t: t.reshape(cfg.batch, cfg.seq, H, d // H).transpose(1, 2)
    a = TF.scaled_dot_product_attention(sp(q), sp(k_), sp(v), is_causal=True).transpose(1, 2).reshape(cfg.batch, cfg.seq, d)
    x = x + TF.linear(a, Pt["l0.wo"], Pt["l0.bo"].reshape(-1))
    h2 = ln(x, "l0.ln2_g", "l0.ln2_b")
    x = x + TF.linear(TF.gelu(TF.linear(h2, Pt["l0.w1"], Pt["l0.b1"].reshape(-1))), Pt["l0.w2"], Pt["l0.b2"].reshape(-1))
    hf = ln(x, "lnf_g", "lnf_b")
    loss = TF.cross_entropy((hf[:, :-1] @ Pt["tok_emb"].T).reshape(-1, cfg.vocab), tok[:, 1:].reshape(-1))
    assert np.isclose(float(loss), L(0.0), rtol=1e-12)
    loss.backward()
    dd = sum(float((Pt[n].grad.numpy() * Zs[n]).sum()) for n in base)
    errs = [abs((L(h) - L(-h)) / (2 * h) - dd) for h in (4e-3, 2e-3, 1e-3)]
    assert errs[2] < 1e-4 * abs(dd)
    assert 3.0 < errs[0] / errs[1] < 5.0 and 3.0 < errs[1] / errs[2] < 5.0      # O(h^2)


def test_trajectory_replays_from_scalar_log_and_descends():
    """theta_T = theta_0 - sum_t lr g_t Z_t: the edge server needs only (step, g)."""
    cfg = I.CONFIGS["cfg1"]
    assert cfg.scale_mode == P.SCALE_PAPER
    o, X, Y = _cfg1_oracle(scale_mode=cfg.scale_mode)
    w0 = o.tensors[0].theta.copy()
    l0 = o.loss()
    log = []
    for s in range(cfg.steps):
        lp, lm, g = o.step(s)
        o.apply_update(s, g, cfg.lr)
        log.append((s, g))
    assert o.loss() < l0
    replay, _, _ = _cfg1_oracle(scale_mode=cfg.scale_mode)
    replay.tensors[0].theta = w0.copy()
    for s, g in log:
        replay.apply_update(s, g, cfg.lr)
    # the live run also perturbed and restored (rounding), the replay did not
    assert np.allclose(replay.tensors[0].theta, o.tensors[0].theta, rtol=0, atol=1.5e-7)   # 10 steps x 2 ulp of restore rounding
    ref = w0.astype(np.float64)
    for s, g in log:
        ref = ref - float(np.float32(np.float32(cfg.lr) * g)) * o.z_of(o.tensors[0], s).astype(np.float64)
    assert np.allclose(o.tensors[0].theta, ref, rtol=0, atol=1.5e-7)


def test_paper_scale_mode_and_16bit_mode_run():
    o, _, _ = _cfg1_oracle(scale_mode=P.SCALE_PAPER, eps=1.0)
    Z = o.z_of(o.tensors[0], 0).astype(np.float64)
    assert 0.9 < np.sum(Z * Z) < 1.1                    # ||z_h||^2 ~ alpha + (1 - alpha) = 1 as printed
    lp, lm, g = o.step(0)
    assert np.isfinite(g)
    o16, _, _ = _cfg1_oracle(bits=16)
    assert o16.step(0) != _cfg1_oracle()[0].step(0)
