"""Pins for the cloud-side oracle (Algorithm 1, cloud block; Sec. 3.2 "Guided Perturbation Sampling on Cloud"):
the hand-written backward pass against PyTorch's autograd through its own library layers and against central
differences of the forward oracle; the gradient basis against what defines it (orthonormality, optimality of the
captured energy, exact recovery of a rank-k column space, invariance to the order of the snapshots)."""
import numpy as np
import pytest
import torch
import torch.nn.functional as TF

import zgr_inputs as I
from oracle import cloud as C
from oracle import forward as F
from tests.test_oracle_forward import TINY_CLS, TINY_LM, _params, _torch_trunk


def _torch_loss_and_grads(cfg, P, tokens, lengths=None, labels=None, act="gelu", post_ln=False):
    """Re-runs the library-layer trunk of the forward pins with gradients enabled, parameters as leaves."""
    import torch.nn as nn
    d = cfg.d_model
    leaves = {k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in P.items()}
    tok = torch.tensor(np.asarray(tokens), dtype=torch.long)
    B, T = tok.shape
    causal = cfg.arch == I.ARCH_DECODER_LM
    x = leaves["tok_emb"][tok] + leaves["pos_emb"][:T][None]
    activation = TF.gelu if act == "gelu" else TF.relu
    if post_ln:
        x = TF.layer_norm(x, (d,), leaves["lnf_g"].reshape(-1), leaves["lnf_b"].reshape(-1), cfg.ln_eps)
    for l in range(cfg.n_layer):
        g = lambda n: leaves[f"l{l}.{n}"]
        mask = torch.triu(torch.ones(T, T, dtype=torch.bool), 1) if causal else None
        kpm = None
        if lengths is not None:
            kpm = torch.arange(T)[None, :] >= torch.tensor(np.asarray(lengths), dtype=torch.long)[:, None]
        h = x if post_ln else TF.layer_norm(x, (d,), g("ln1_g").reshape(-1), g("ln1_b").reshape(-1), cfg.ln_eps)
        a, _ = TF.multi_head_attention_forward(
            h.transpose(0, 1), h.transpose(0, 1), h.transpose(0, 1), d, cfg.n_head,
            torch.cat([g("wq"), g("wk"), g("wv")], 0), torch.cat([g("bq"), g("bk"), g("bv")], 1).reshape(-1),
            None, None, False, 0.0, g("wo"), g("bo").reshape(-1), training=True, key_padding_mask=kpm, need_weights=False, attn_mask=mask)
        x = x + a.transpose(0, 1)
        if post_ln:
            x = TF.layer_norm(x, (d,), g("ln1_g").reshape(-1), g("ln1_b").reshape(-1), cfg.ln_eps)
        h = x if post_ln else TF.layer_norm(x, (d,), g("ln2_g").reshape(-1), g("ln2_b").reshape(-1), cfg.ln_eps)
        x = x + TF.linear(activation(TF.linear(h, g("w1"), g("b1").reshape(-1))), g("w2"), g("b2").reshape(-1))
        if post_ln:
            x = TF.layer_norm(x, (d,), g("ln2_g").reshape(-1), g("ln2_b").reshape(-1), cfg.ln_eps)
    hf = x if post_ln else TF.layer_norm(x, (d,), leaves["lnf_g"].reshape(-1), leaves["lnf_b"].reshape(-1), cfg.ln_eps)
    if causal:
        logits = hf[:, :-1] @ leaves["tok_emb"].T
        loss = TF.cross_entropy(logits.reshape(-1, cfg.vocab), tok[:, 1:].reshape(-1))
    else:
        logits = hf[:, 0] @ leaves["cls_w"].T + leaves["cls_b"].reshape(-1)
        loss = TF.cross_entropy(logits, torch.tensor(np.asarray(labels), dtype=torch.long))
    loss.backward()
    return float(loss.detach()), {k: v.grad.numpy() for k, v in leaves.items()}


def test_lm_backward_matches_autograd_through_library_layers():
    cfg = TINY_LM
    P = _params(cfg, scale=15.0)
    tokens = I.make_tokens(cfg)
    loss, grads = C.lm_loss_and_gradients(P, tokens, cfg.n_layer, cfg.n_head, cfg.ln_eps)
    tl, tg = _torch_loss_and_grads(cfg, P, tokens)
    assert np.isclose(loss, tl, rtol=1e-12) and np.isclose(loss, F.lm_loss(P, tokens, cfg.n_layer, cfg.n_head, cfg.ln_eps), rtol=1e-13)
    assert set(grads) == set(P)
    for k in P:
        assert grads[k].shape == P[k].shape, k
        scale = np.abs(tg[k]).max() + 1e-30
        assert np.abs(grads[k] - tg[k]).max() <= 1e-10 * scale + 1e-14, (k, np.abs(grads[k] - tg[k]).max(), scale)
    # every tensor takes part, except the key biases: a constant added to all keys shifts every score of a query alike
    assert min(np.abs(g).max() for k, g in grads.items() if not k.endswith(".bk")) > 1e-6
    assert max(np.abs(g).max() for k, g in grads.items() if k.endswith(".bk")) < 1e-12


def test_cls_backward_matches_autograd_through_library_layers():
    cfg = TINY_CLS
    P = _params(cfg, scale=15.0)
    tokens, labels = I.make_tokens(cfg), I.make_labels(cfg)
    lengths = np.array([14, 5, 9, 1], dtype=np.int32)
    loss, grads = C.cls_loss_and_gradients(P, tokens, lengths, labels, cfg.n_layer, cfg.n_head, cfg.ln_eps)
    tl, tg = _torch_loss_and_grads(cfg, P, tokens, lengths, labels)
    assert np.isclose(loss, tl, rtol=1e-12)
    for k in P:
        scale = np.abs(tg[k]).max() + 1e-30
        assert np.abs(grads[k] - tg[k]).max() <= 1e-10 * scale + 1e-14, k


@pytest.mark.parametrize("act,post_ln", [("relu", False), ("gelu", True), ("relu", True)])
def test_backward_of_the_model_family_variants(act, post_ln):
    """ReLU feed-forward and post-LayerNorm blocks: autograd through the library layers in the same order, and an
    extrapolated central difference of the forward oracle along a whole-model direction."""
    cfg = TINY_LM
    P = _params(cfg, scale=15.0)
    tokens = I.make_tokens(cfg)
    loss, grads = C.lm_loss_and_gradients(P, tokens, cfg.n_layer, cfg.n_head, cfg.ln_eps, act, post_ln)
    tl, tg = _torch_loss_and_grads(cfg, P, tokens, act=act, post_ln=post_ln)
    assert np.isclose(loss, tl, rtol=1e-12) and np.isclose(loss, F.lm_loss(P, tokens, cfg.n_layer, cfg.n_head, cfg.ln_eps, act, post_ln), rtol=1e-13)
    for k in P:
        scale = np.abs(tg[k]).max() + 1e-30
        assert np.abs(grads[k] - tg[k]).max() <= 1e-10 * scale + 1e-14, (k, np.abs(grads[k] - tg[k]).max(), scale)
    cfgc = TINY_CLS
    Pc = _params(cfgc, scale=15.0)
    tok, labels = I.make_tokens(cfgc), I.make_labels(cfgc)
    lengths = np.array([14, 5, 9, 1], dtype=np.int32)
    lossc, gradsc = C.cls_loss_and_gradients(Pc, tok, lengths, labels, cfgc.n_layer, cfgc.n_head, cfgc.ln_eps, act, post_ln)
    tlc, tgc = _torch_loss_and_grads(cfgc, Pc, tok, lengths, labels, act, post_ln)
    assert np.isclose(lossc, tlc, rtol=1e-12)
    for k in Pc:
        scale = np.abs(tgc[k]).max() + 1e-30
        assert np.abs(gradsc[k] - tgc[k]).max() <= 1e-10 * scale + 1e-14, k
    if act == "gelu":                                    # smooth: the difference quotient converges
        f = lambda Q: F.lm_loss(Q, tokens, cfg.n_layer, cfg.n_head, cfg.ln_eps, act, post_ln)
        rng = np.random.default_rng(4)
        D = {k: rng.standard_normal(v.shape) for k, v in P.items()}
        want = sum(float((grads[k] * D[k]).sum()) for k in P)
        cd = lambda h: (f({k: P[k] + h * D[k] for k in P}) - f({k: P[k] - h * D[k] for k in P})) / (2 * h)
        fd = (4.0 * cd(1e-4) - cd(2e-4)) / 3.0
        assert abs(fd - want) <= 1e-8 * max(1.0, abs(want)), (fd, want)


@pytest.mark.parametrize("which", ["lm", "cls"])
def test_backward_matches_central_differences_of_the_forward_oracle(which):
    cfg = TINY_LM if which == "lm" else TINY_CLS
    P = _params(cfg, scale=10.0)
    tokens = I.make_tokens(cfg)
    lengths, labels = np.array([14, 5, 9, 2], dtype=np.int32), I.make_labels(TINY_CLS)
    if which == "lm":
        f = lambda Q: F.lm_loss(Q, tokens, cfg.n_layer, cfg.n_head, cfg.ln_eps)
        _, grads = C.lm_loss_and_gradients(P, tokens, cfg.n_layer, cfg.n_head, cfg.ln_eps)
    else:
        f = lambda Q: F.cls_loss(Q, tokens, lengths, labels, cfg.n_layer, cfg.n_head, cfg.ln_eps)
        _, grads = C.cls_loss_and_gradients(P, tokens, lengths, labels, cfg.n_layer, cfg.n_head, cfg.ln_eps)
    rng = np.random.default_rng(3)
    for trial in range(3):                                # whole-model directions
        D = {k: rng.standard_normal(v.shape) for k, v in P.items()}
        want = sum(float((grads[k] * D[k]).sum()) for k in P)
        cd = lambda h: (f({k: P[k] + h * D[k] for k in P}) - f({k: P[k] - h * D[k] for k in P})) / (2 * h)
        fd = (4.0 * cd(1e-4) - cd(2e-4)) / 3.0            # Richardson: the h^2 term of the central difference cancels
        assert abs(fd - want) <= 1e-8 * max(1.0, abs(want)), (trial, fd, want)
    for name in ("l0.wq", "l1.w2", "l0.ln2_g", "pos_emb", "l1.bv"):   # single coordinates
        idx = tuple(rng.integers(0, s) for s in P[name].shape)
        h = 1e-5
        up, dn = {k: v.copy() for k, v in P.items()}, {k: v.copy() for k, v in P.items()}
        up[name][idx] += h; dn[name][idx] -= h
        fd = (f(up) - f(dn)) / (2 * h)
        assert abs(fd - grads[name][idx]) <= 1e-7 * max(1.0, abs(fd)) + 1e-9, (name, fd, grads[name][idx])


def test_lsq_gradient_is_the_closed_form_and_the_autograd_one():
    cfg = I.CONFIGS["cfg1"]
    W = I.make_params(cfg)[0].astype(np.float64)
    X, Y = I.make_lsq_data(cfg)
    Wt = torch.tensor(W, requires_grad=True)
    (TF.mse_loss(torch.tensor(X.astype(np.float64)) @ Wt.T, torch.tensor(Y.astype(np.float64)), reduction="sum") / (2 * X.shape[0])).backward()
    assert np.allclose(C.lsq_gradient(W, X, Y), Wt.grad.numpy(), rtol=1e-11, atol=1e-14)


def _snapshots(rows, cols, s, rank, noise, seed):
    rng = np.random.default_rng(seed)
    A = np.linalg.qr(rng.standard_normal((rows, rank)))[0] * (2.0 ** -np.arange(rank))[None, :]
    return [A @ rng.standard_normal((rank, cols)) + noise * rng.standard_normal((rows, cols)) for _ in range(s)], A


def test_gradient_basis_is_orthonormal_and_optimal():
    snaps, _ = _snapshots(40, 24, 3, 12, 0.01, 0)
    k = 5
    U, sv = C.gradient_basis(snaps, k)
    assert U.shape == (40, k) and np.allclose(U.T @ U, np.eye(k), atol=1e-12)
    assert np.all(U[np.abs(U).argmax(axis=0), np.arange(k)] > 0)
    # captured energy = sum of the k largest squared singular values over all of them, and no other subspace does better
    e = C.captured_energy(U, snaps)
    assert np.isclose(e, (sv[:k] ** 2).sum() / (sv ** 2).sum(), rtol=1e-12)
    rng = np.random.default_rng(1)
    for _ in range(50):
        Q = np.linalg.qr(rng.standard_normal((40, k)))[0]
        assert C.captured_energy(Q, snaps) <= e + 1e-12
    # a small rotation of U towards any direction outside it loses energy (local optimality)
    for _ in range(10):
        Q = np.linalg.qr(U + 1e-3 * rng.standard_normal(U.shape))[0]
        assert C.captured_energy(Q, snaps) <= e + 1e-12


def test_gradient_basis_recovers_a_rank_k_column_space_exactly_and_ignores_snapshot_order():
    snaps, A = _snapshots(64, 16, 4, 6, 0.0, 5)
    U, sv = C.gradient_basis(snaps, 6)
    Pa = A @ np.linalg.pinv(A)                               # projector onto the true column space
    assert np.allclose(U @ U.T, Pa, atol=1e-10)
    assert sv[6] <= 1e-12 * sv[0]
    for g in snaps:
        assert np.allclose(U @ (U.T @ g), g, atol=1e-10)     # every stored gradient lies in the subspace
    U2, _ = C.gradient_basis(snaps[::-1], 6)
    assert np.allclose(U2 @ U2.T, U @ U.T, atol=1e-10)
    # one snapshot: the leading left singular vectors of that matrix (textbook special case)
    U1, _ = C.gradient_basis(snaps[:1], 3)
    u, _, _ = np.linalg.svd(snaps[0])
    assert np.allclose(U1 @ U1.T, u[:, :3] @ u[:, :3].T, atol=1e-10)
