"""Pins for the oracle's loss functions: PyTorch's own library layers
(nn.TransformerEncoderLayer with norm_first, F.cross_entropy, autograd) in
fp64 on the same weights, invariants (causality, padding), the value ln V at
a near-uniform init, and the closed-form least-squares gradient."""
import numpy as np
import pytest
import torch
import torch.nn as nn
import torch.nn.functional as TF

import zgr_inputs as I
from oracle import forward as F

TINY_LM = I.shrink(I.CONFIGS["cfg2"], name="tiny_lm", n_layer=2, d_model=32, n_head=4, d_ff=64, vocab=97,
                   max_pos=16, batch=3, seq=12)
TINY_CLS = I.shrink(I.CONFIGS["cfg4"], name="tiny_cls", dtype="f32", n_layer=2, d_model=32, n_head=2, d_ff=48,
                    vocab=89, max_pos=16, batch=4, seq=14, tokens="uniform")


def _params(cfg, scale=1.0):
    specs = I.tensor_specs(cfg)
    vals = I.make_params(cfg, 0, specs)
    # a larger init than N(0,0.02) makes every term of the block matter in the comparison
    out = {}
    for s, v in zip(specs, vals):
        v = v.astype(np.float64)
        if s.role in (I.ROLE_LN1_G, I.ROLE_LN2_G, I.ROLE_LNF_G):
            out[s.name] = 1.0 + (v - 1.0) * scale
        else:
            out[s.name] = v * scale
    return out


@torch.no_grad()
def _torch_trunk(cfg, P, tokens, causal, lengths, act="gelu", post_ln=False):
    d = cfg.d_model
    tt = lambda a: torch.tensor(a, dtype=torch.float64)
    tok = torch.tensor(tokens, dtype=torch.long)
    B, T = tok.shape
    x = tt(P["tok_emb"])[tok] + tt(P["pos_emb"])[:T][None]
    if post_ln:
        x = TF.layer_norm(x, (d,), tt(P["lnf_g"]).reshape(-1), tt(P["lnf_b"]).reshape(-1), cfg.ln_eps)
    for l in range(cfg.n_layer):
        layer = nn.TransformerEncoderLayer(d, cfg.n_head, cfg.d_ff, dropout=0.0, activation=act,
                                           layer_norm_eps=cfg.ln_eps, batch_first=True, norm_first=not post_ln,
                                           dtype=torch.float64)
        g = lambda n: tt(P[f"l{l}.{n}"])
        sd = {
            "self_attn.in_proj_weight": torch.cat([g("wq"), g("wk"), g("wv")], 0),
            "self_attn.in_proj_bias": torch.cat([g("bq"), g("bk"), g("bv")], 1).reshape(-1),
            "self_attn.out_proj.weight": g("wo"), "self_attn.out_proj.bias": g("bo").reshape(-1),
            "linear1.weight": g("w1"), "linear1.bias": g("b1").reshape(-1),
            "linear2.weight": g("w2"), "linear2.bias": g("b2").reshape(-1),
            "norm1.weight": g("ln1_g").reshape(-1), "norm1.bias": g("ln1_b").reshape(-1),
            "norm2.weight": g("ln2_g").reshape(-1), "norm2.bias": g("ln2_b").reshape(-1),
        }
        layer.load_state_dict(sd)
        layer.train()      # keeps the plain (non fused) code path; dropout is 0
        mask = torch.triu(torch.ones(T, T, dtype=torch.bool), 1) if causal else None
        kpm = None
        if lengths is not None:
            kpm = torch.arange(T)[None, :] >= torch.tensor(lengths, dtype=torch.long)[:, None]
        x = layer(x, src_mask=mask, src_key_padding_mask=kpm)
    if post_ln:
        return x
    return TF.layer_norm(x, (d,), tt(P["lnf_g"]).reshape(-1), tt(P["lnf_b"]).reshape(-1), cfg.ln_eps)


def test_lm_loss_matches_torch_library_layers():
    cfg = TINY_LM
    P = _params(cfg, scale=15.0)
    tokens = I.make_tokens(cfg)
    h = _torch_trunk(cfg, P, tokens, True, None)
    logits = h[:, :-1] @ torch.tensor(P["tok_emb"]).T
    tgt = torch.tensor(tokens[:, 1:], dtype=torch.long)
    want_tok = TF.cross_entropy(logits.reshape(-1, cfg.vocab), tgt.reshape(-1), reduction="none").reshape(tgt.shape)
    got_tok = F.lm_token_losses(P, tokens, cfg.n_layer, cfg.n_head, cfg.ln_eps)
    assert np.allclose(got_tok, want_tok.numpy(), rtol=1e-10, atol=1e-12)
    assert np.isclose(F.lm_loss(P, tokens, cfg.n_layer, cfg.n_head, cfg.ln_eps), float(want_tok.mean()), rtol=1e-12)
    assert got_tok.std() > 0.05          # the scaled init makes the comparison non-trivial


def test_cls_loss_matches_torch_library_layers():
    cfg = TINY_CLS
    P = _params(cfg, scale=15.0)
    tokens, labels = I.make_tokens(cfg), I.make_labels(cfg)
    lengths = np.array([14, 5, 9, 1], dtype=np.int32)
    h = _torch_trunk(cfg, P, tokens, False, lengths)
    logits = h[:, 0] @ torch.tensor(P["cls_w"]).T + torch.tensor(P["cls_b"]).reshape(-1)
    want = TF.cross_entropy(logits, torch.tensor(labels, dtype=torch.long), reduction="none").numpy()
    got = F.cls_row_losses(P, tokens, lengths, labels, cfg.n_layer, cfg.n_head, cfg.ln_eps)
    assert np.allclose(got, want, rtol=1e-10, atol=1e-12)
    assert np.isclose(F.cls_loss(P, tokens, lengths, labels, cfg.n_layer, cfg.n_head, cfg.ln_eps), want.mean(), rtol=1e-12)


@pytest.mark.parametrize("act,post_ln", [("relu", False), ("gelu", True), ("relu", True)])
def test_model_family_variants_match_torch_library_layers(act, post_ln):
    """ReLU feed-forward and post-LayerNorm blocks (with the embedding LayerNorm) against the library layer built
    with the same two switches, for the decoder loss and the classifier loss."""
    cfg = TINY_LM
    P = _params(cfg, scale=15.0)
    tokens = I.make_tokens(cfg)
    h = _torch_trunk(cfg, P, tokens, True, None, act, post_ln)
    logits = h[:, :-1] @ torch.tensor(P["tok_emb"]).T
    tgt = torch.tensor(tokens[:, 1:], dtype=torch.long)
    want_tok = TF.cross_entropy(logits.reshape(-1, cfg.vocab), tgt.reshape(-1), reduction="none").reshape(tgt.shape).numpy()
    got_tok = F.lm_token_losses(P, tokens, cfg.n_layer, cfg.n_head, cfg.ln_eps, act, post_ln)
    assert np.allclose(got_tok, want_tok, rtol=1e-10, atol=1e-12)
    assert not np.allclose(got_tok, F.lm_token_losses(P, tokens, cfg.n_layer, cfg.n_head, cfg.ln_eps), rtol=1e-3)   # the switches matter
    cfgc = TINY_CLS
    Pc = _params(cfgc, scale=15.0)
    tok, labels = I.make_tokens(cfgc), I.make_labels(cfgc)
    lengths = np.array([14, 5, 9, 1], dtype=np.int32)
    hc = _torch_trunk(cfgc, Pc, tok, False, lengths, act, post_ln)
    lc = hc[:, 0] @ torch.tensor(Pc["cls_w"]).T + torch.tensor(Pc["cls_b"]).reshape(-1)
    want = TF.cross_entropy(lc, torch.tensor(labels, dtype=torch.long), reduction="none").numpy()
    got = F.cls_row_losses(Pc, tok, lengths, labels, cfgc.n_layer, cfgc.n_head, cfgc.ln_eps, act, post_ln)
    assert np.allclose(got, want, rtol=1e-10, atol=1e-12)


def test_causality_and_padding_invariants():
    cfg = TINY_LM
    P = _params(cfg, scale=10.0)
    tokens = I.make_tokens(cfg)
    base = F.lm_token_losses(P, tokens, cfg.n_layer, cfg.n_head)
    t2 = tokens.copy()
    t2[:, 8:] = (t2[:, 8:] + 1) % cfg.vocab       # change tokens at positions >= 8
    other = F.lm_token_losses(P, t2, cfg.n_layer, cfg.n_head)
    # the loss at position t predicts token t+1 from tokens <= t: positions < 7 are untouched
    assert np.array_equal(base[:, :7], other[:, :7]) and not np.allclose(base[:, 7:], other[:, 7:])
    cfgc = TINY_CLS
    Pc = _params(cfgc, scale=10.0)
    tok, lab = I.make_tokens(cfgc), I.make_labels(cfgc)
    lengths = np.array([14, 5, 9, 2], dtype=np.int32)
    a = F.cls_row_losses(Pc, tok, lengths, lab, cfgc.n_layer, cfgc.n_head)
    tok2 = tok.copy()
    for b, n in enumerate(lengths):
        tok2[b, n:] = (tok2[b, n:] + 3) % cfgc.vocab          # padded positions only
    b_ = F.cls_row_losses(Pc, tok2, lengths, lab, cfgc.n_layer, cfgc.n_head)
    assert np.allclose(a, b_, rtol=1e-13)
    tok3 = tok.copy()
    tok3[1, 4] = (tok3[1, 4] + 1) % cfgc.vocab                # a valid position
    assert not np.isclose(F.cls_row_losses(Pc, tok3, lengths, lab, cfgc.n_layer, cfgc.n_head)[1], a[1], rtol=1e-9)


def test_loss_at_small_init_is_log_vocab():
    cfg = I.CONFIGS["cfg2"]
    specs = I.tensor_specs(cfg)
    P = {s.name: v.astype(np.float64) for s, v in zip(specs, I.make_params(cfg, 0, specs))}
    loss = F.lm_loss(P, I.make_tokens(cfg), cfg.n_layer, cfg.n_head)
    # logits of a unit-variance LayerNorm output against N(0, 0.02^2) embeddings are ~N(0, d 0.02^2):
    # E[logsumexp] - E[target logit] = ln V + sigma^2 / 2 to first order
    assert abs(loss - (np.log(cfg.vocab) + cfg.d_model * 0.02 ** 2 / 2)) < 1e-2
    cfgc = TINY_CLS
    Pc = _params(cfgc, 1.0)
    l2 = F.cls_loss(Pc, I.make_tokens(cfgc), I.make_lengths(cfgc, lo=2), I.make_labels(cfgc), cfgc.n_layer, cfgc.n_head)
    assert abs(l2 - np.log(2)) < 3e-2


def test_softmax_rows_and_gelu_and_layernorm_against_torch():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((5, 33)) * 3
    assert np.allclose(np.exp(F.log_softmax(x)).sum(-1), 1.0, rtol=1e-13)
    assert np.allclose(F.log_softmax(x), TF.log_softmax(torch.tensor(x), -1).numpy(), rtol=1e-12, atol=1e-13)
    assert np.allclose(F.gelu(x), TF.gelu(torch.tensor(x)).numpy(), rtol=1e-12, atol=1e-14)
    g, b = rng.standard_normal(33), rng.standard_normal(33)
    want = TF.layer_norm(torch.tensor(x), (33,), torch.tensor(g), torch.tensor(b), 1e-5).numpy()
    assert np.allclose(F.layer_norm(x, g, b, 1e-5), want, rtol=1e-12, atol=1e-13)


def test_lsq_loss_and_gradient_closed_form():
    cfg = I.CONFIGS["cfg1"]
    W = I.make_params(cfg)[0].astype(np.float64)
    X, Y = I.make_lsq_data(cfg)
    X64, Y64 = X.astype(np.float64), Y.astype(np.float64)
    Wt = torch.tensor(W, requires_grad=True)
    lt = TF.mse_loss(torch.tensor(X64) @ Wt.T, torch.tensor(Y64), reduction="sum") / (2 * X.shape[0])
    assert np.isclose(F.lsq_loss(W, X, Y), float(lt), rtol=1e-13)
    lt.backward()
    grad = (X64 @ W.T - Y64).T @ X64 / X.shape[0]
    assert np.allclose(Wt.grad.numpy(), grad, rtol=1e-11, atol=1e-14)
