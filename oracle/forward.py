"""TEST INFRASTRUCTURE ONLY: CPU oracle, never imported by the product path.

The loss L(W; x) that the two forward passes of the ZGR step evaluate
(Sec. 3.2, Eq. (9) and Eq. (11); workflow step 6 of Sec. 3.1).  The paper uses
off-the-shelf transformer checkpoints; here the model is the plain textbook
one: pre-LayerNorm blocks, multi-head softmax attention scaled by
1/sqrt(d_head), erf-GELU feed-forward, learned positions, final LayerNorm, and
either a next-token cross-entropy through the tied embedding (decoder) or a
linear classification head on the first token (encoder with key padding mask).

The two model families of the paper's experiments (Sec. 4, models and
datasets) differ from that default in two textbook choices, both offered here:
act = "relu" (the decoder family's feed-forward activation) and post_ln = True
(the encoder family's blocks: LayerNorm after each residual sum, x <- LN(x +
sublayer(x)), a LayerNorm on the embeddings and none at the end; the tensors
lnf_g / lnf_b then are that embedding LayerNorm).

Everything is evaluated in fp64 with numpy on the stored parameter values,
with no blocking or fusion: each line is the definition of the layer.
`params` maps tensor names (as in zgr_inputs.tensor_specs) to arrays.
"""
import numpy as np
from scipy.special import erf


def layer_norm(x, g, b, eps):
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps) * g.reshape(-1) + b.reshape(-1)


def gelu(x):
    return 0.5 * x * (1.0 + erf(x / np.sqrt(2.0)))


def relu(x):
    return np.maximum(x, 0.0)


def log_softmax(z):
    m = z.max(axis=-1, keepdims=True)
    return z - m - np.log(np.exp(z - m).sum(axis=-1, keepdims=True))


def attention(q, k, v, n_head, causal, lengths):
    """q, k, v: [B, T, d].  Returns [B, T, d]."""
    B, T, d = q.shape
    dh = d // n_head
    qh = q.reshape(B, T, n_head, dh).transpose(0, 2, 1, 3)
    kh = k.reshape(B, T, n_head, dh).transpose(0, 2, 1, 3)
    vh = v.reshape(B, T, n_head, dh).transpose(0, 2, 1, 3)
    s = qh @ kh.transpose(0, 1, 3, 2) / np.sqrt(dh)            # [B, H, T, T]
    if causal:
        s = np.where(np.tril(np.ones((T, T), dtype=bool))[None, None], s, -np.inf)
    if lengths is not None:
        keep = np.arange(T)[None, :] < np.asarray(lengths)[:, None]   # [B, T] valid keys
        s = np.where(keep[:, None, None, :], s, -np.inf)
    p = np.exp(log_softmax(s))
    return (p @ vh).transpose(0, 2, 1, 3).reshape(B, T, d)


def block(x, P, l, n_head, causal, lengths, ln_eps, act="gelu", post_ln=False):
    g = lambda n: P[f"l{l}.{n}"]
    activation = {"gelu": gelu, "relu": relu}[act]
    h = x if post_ln else layer_norm(x, g("ln1_g"), g("ln1_b"), ln_eps)
    q = h @ g("wq").T + g("bq").reshape(-1)
    k = h @ g("wk").T + g("bk").reshape(-1)
    v = h @ g("wv").T + g("bv").reshape(-1)
    a = attention(q, k, v, n_head, causal, lengths)
    x = x + a @ g("wo").T + g("bo").reshape(-1)
    if post_ln:
        x = layer_norm(x, g("ln1_g"), g("ln1_b"), ln_eps)
    h = x if post_ln else layer_norm(x, g("ln2_g"), g("ln2_b"), ln_eps)
    f = activation(h @ g("w1").T + g("b1").reshape(-1))
    x = x + f @ g("w2").T + g("b2").reshape(-1)
    if post_ln:
        x = layer_norm(x, g("ln2_g"), g("ln2_b"), ln_eps)
    return x


def trunk(P, tokens, n_layer, n_head, causal, lengths, ln_eps, act="gelu", post_ln=False):
    tokens = np.asarray(tokens)
    B, T = tokens.shape
    x = P["tok_emb"][tokens] + P["pos_emb"][:T][None]
    if post_ln:
        x = layer_norm(x, P["lnf_g"], P["lnf_b"], ln_eps)
    for l in range(n_layer):
        x = block(x, P, l, n_head, causal, lengths, ln_eps, act, post_ln)
    return x if post_ln else layer_norm(x, P["lnf_g"], P["lnf_b"], ln_eps)


def lm_token_losses(P, tokens, n_layer, n_head, ln_eps=1e-5, act="gelu", post_ln=False):
    """-log p(token[t+1] | tokens[..t]) for t < T-1: [B, T-1]."""
    tokens = np.asarray(tokens)
    h = trunk(P, tokens, n_layer, n_head, True, None, ln_eps, act, post_ln)
    logp = log_softmax(h[:, :-1] @ P["tok_emb"].T)
    return -np.take_along_axis(logp, tokens[:, 1:, None].astype(np.int64), axis=-1)[..., 0]


def lm_loss(P, tokens, n_layer, n_head, ln_eps=1e-5, act="gelu", post_ln=False):
    """Mean next-token cross-entropy over the B (T-1) shifted positions."""
    return float(lm_token_losses(P, tokens, n_layer, n_head, ln_eps, act, post_ln).mean())


def cls_row_losses(P, tokens, lengths, labels, n_layer, n_head, ln_eps=1e-5, act="gelu", post_ln=False):
    h = trunk(P, tokens, n_layer, n_head, False, lengths, ln_eps, act, post_ln)
    logits = h[:, 0] @ P["cls_w"].T + P["cls_b"].reshape(-1)
    logp = log_softmax(logits)
    return -np.take_along_axis(logp, np.asarray(labels)[:, None].astype(np.int64), axis=-1)[:, 0]


def cls_loss(P, tokens, lengths, labels, n_layer, n_head, ln_eps=1e-5, act="gelu", post_ln=False):
    """Mean cross-entropy of the classification head over the batch."""
    return float(cls_row_losses(P, tokens, lengths, labels, n_layer, n_head, ln_eps, act, post_ln).mean())


def lsq_loss(W, X, Y):
    """L = ||X W^T - Y||_F^2 / (2 B): mean over the batch, sum over outputs."""
    r = np.asarray(X, dtype=np.float64) @ np.asarray(W, dtype=np.float64).T - np.asarray(Y, dtype=np.float64)
    return float((r * r).sum() / (2.0 * r.shape[0]))
