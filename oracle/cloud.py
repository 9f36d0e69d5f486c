"""TEST INFRASTRUCTURE ONLY: CPU oracle, never imported by the product path.

Cloud block of Algorithm 1 (back-propagation on the public dataset with the
current weights, whose gradients build the basis) and the paragraph on guided
perturbation sampling on the cloud of Sec. 3.2: the cloud trains by backpropagation on a public dataset, stores the
gradients it computes, and keeps an orthonormal basis of the subspace they span.

Two parts, both in fp64 with numpy, one line per layer rule:

  * the gradient of the loss L(W; x) of oracle/forward.py with respect to every
    parameter tensor, by the chain rule written out layer by layer (no autograd
    here; the tests pin it against PyTorch's autograd through its own library
    layers and against central differences of oracle/forward.py);

  * the basis of one weight matrix.  Reading: the perturbation of a matrix
    W [rows, cols] is Z = a G + b U R with U [rows, k] acting on every column
    (oracle/perturbation.py), so the "subspace of gradients" of that matrix is a
    k-dimensional subspace of R^rows: the one that captures the most of the
    stored gradient snapshots G_1 .. G_s (each [rows, cols]), i.e. that maximises
    sum_t ||U^T G_t||_F^2 over orthonormal U.  That is the span of the k leading
    left singular vectors of [G_1 | ... | G_s]; the SVD is the library primitive
    that returns it.  The subspace is what is defined (a basis of it is fixed only
    up to a rotation), so comparisons use the projector U U^T.

The paper also says the mixing ratio is tuned from how large the two kinds of
perturbation are relative to each other, and gives no rule for it: nothing to build.
"""
import numpy as np
from scipy.special import erf

from . import forward as F


# ---------------------------------------------------------------- layer rules (forward with what backward needs, backward)

def _ln_fwd(x, g, b, eps):
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + eps)
    xhat = (x - mu) * rstd
    return xhat * g.reshape(-1) + b.reshape(-1), (xhat, rstd)


def _ln_bwd(dy, cache, g):
    xhat, rstd = cache
    dg = (dy * xhat).reshape(-1, xhat.shape[-1]).sum(axis=0)
    db = dy.reshape(-1, xhat.shape[-1]).sum(axis=0)
    dxhat = dy * g.reshape(-1)
    dx = rstd * (dxhat - dxhat.mean(axis=-1, keepdims=True) - xhat * (dxhat * xhat).mean(axis=-1, keepdims=True))
    return dx, dg, db


def _linear_bwd(dy, h, W):
    """y = h W^T + b  ->  (dh, dW, db)."""
    d2, h2 = dy.reshape(-1, dy.shape[-1]), h.reshape(-1, h.shape[-1])
    return dy @ W, d2.T @ h2, d2.sum(axis=0)


def _gelu_grad(u):
    return 0.5 * (1.0 + erf(u / np.sqrt(2.0))) + u * np.exp(-0.5 * u * u) / np.sqrt(2.0 * np.pi)


def _split(x, n_head):
    B, T, d = x.shape
    return x.reshape(B, T, n_head, d // n_head).transpose(0, 2, 1, 3)


def _merge(xh):
    B, H, T, dh = xh.shape
    return xh.transpose(0, 2, 1, 3).reshape(B, T, H * dh)


def _act_fwd(u, act):
    return F.gelu(u) if act == "gelu" else F.relu(u)


def _act_grad(u, act):
    return _gelu_grad(u) if act == "gelu" else (u > 0).astype(np.float64)


def _trunk_fwd(P, tokens, n_layer, n_head, causal, lengths, ln_eps, act="gelu", post_ln=False):
    """Forward of forward.trunk keeping what the backward rules need.  post_ln: see oracle/forward.py."""
    tokens = np.asarray(tokens)
    B, T = tokens.shape
    x = P["tok_emb"][tokens] + P["pos_emb"][:T][None]
    c_emb = None
    if post_ln:
        x, c_emb = _ln_fwd(x, P["lnf_g"], P["lnf_b"], ln_eps)
    caches = []
    for l in range(n_layer):
        g = lambda n: P[f"l{l}.{n}"]
        h1, c1 = (x, None) if post_ln else _ln_fwd(x, g("ln1_g"), g("ln1_b"), ln_eps)
        q = h1 @ g("wq").T + g("bq").reshape(-1)
        k = h1 @ g("wk").T + g("bk").reshape(-1)
        v = h1 @ g("wv").T + g("bv").reshape(-1)
        qh, kh, vh = _split(q, n_head), _split(k, n_head), _split(v, n_head)
        dh = qh.shape[-1]
        s = qh @ kh.transpose(0, 1, 3, 2) / np.sqrt(dh)
        if causal:
            s = np.where(np.tril(np.ones((T, T), dtype=bool))[None, None], s, -np.inf)
        if lengths is not None:
            keep = np.arange(T)[None, :] < np.asarray(lengths)[:, None]
            s = np.where(keep[:, None, None, :], s, -np.inf)
        p = np.exp(F.log_softmax(s))
        a = _merge(p @ vh)
        x1 = x + a @ g("wo").T + g("bo").reshape(-1)
        if post_ln:
            x1, c1 = _ln_fwd(x1, g("ln1_g"), g("ln1_b"), ln_eps)
        h2, c2 = (x1, None) if post_ln else _ln_fwd(x1, g("ln2_g"), g("ln2_b"), ln_eps)
        u = h2 @ g("w1").T + g("b1").reshape(-1)
        f = _act_fwd(u, act)
        x2 = x1 + f @ g("w2").T + g("b2").reshape(-1)
        if post_ln:
            x2, c2 = _ln_fwd(x2, g("ln2_g"), g("ln2_b"), ln_eps)
        caches.append((h1, c1, qh, kh, vh, p, a, h2, c2, u, f))
        x = x2
    if post_ln:
        return x, c_emb, caches
    hf, cf = _ln_fwd(x, P["lnf_g"], P["lnf_b"], ln_eps)
    return hf, cf, caches


def _trunk_bwd(P, tokens, n_layer, n_head, dhf, cf, caches, grads, act="gelu", post_ln=False):
    """cf: what _trunk_fwd returned second (the final LayerNorm's cache, or the embedding LayerNorm's with post_ln)."""
    tokens = np.asarray(tokens)
    B, T = tokens.shape
    if post_ln:
        dx = dhf
    else:
        dx, dg, db = _ln_bwd(dhf, cf, P["lnf_g"])
        grads["lnf_g"], grads["lnf_b"] = dg.reshape(1, -1), db.reshape(1, -1)
    for l in reversed(range(n_layer)):
        g = lambda n: P[f"l{l}.{n}"]
        h1, c1, qh, kh, vh, p, a, h2, c2, u, f = caches[l]
        dh_scale = 1.0 / np.sqrt(qh.shape[-1])
        if post_ln:                                                # x2 = LN2(y2), y2 = x1 + f W2^T + b2
            dx, dg2, db2 = _ln_bwd(dx, c2, g("ln2_g"))
            grads[f"l{l}.ln2_g"], grads[f"l{l}.ln2_b"] = dg2.reshape(1, -1), db2.reshape(1, -1)
        # (pre-LN: x2 = x1 + f W2^T + b2)
        df, grads[f"l{l}.w2"], b2 = _linear_bwd(dx, f, g("w2"))
        grads[f"l{l}.b2"] = b2.reshape(1, -1)
        du = df * _act_grad(u, act)
        dh2, grads[f"l{l}.w1"], b1 = _linear_bwd(du, h2, g("w1"))
        grads[f"l{l}.b1"] = b1.reshape(1, -1)
        if post_ln:                                                # h2 = x1 = LN1(y1), y1 = x + a Wo^T + bo
            dx1, dg1, db1 = _ln_bwd(dx + dh2, c1, g("ln1_g"))
            grads[f"l{l}.ln1_g"], grads[f"l{l}.ln1_b"] = dg1.reshape(1, -1), db1.reshape(1, -1)
        else:                                                      # h2 = LN2(x1)
            d1, dg2, db2 = _ln_bwd(dh2, c2, g("ln2_g"))
            grads[f"l{l}.ln2_g"], grads[f"l{l}.ln2_b"] = dg2.reshape(1, -1), db2.reshape(1, -1)
            dx1 = dx + d1
        # x1 (or y1) = x + a Wo^T + bo
        da, grads[f"l{l}.wo"], bo = _linear_bwd(dx1, a, g("wo"))
        grads[f"l{l}.bo"] = bo.reshape(1, -1)
        dah = _split(da, n_head)
        dp = dah @ vh.transpose(0, 1, 3, 2)
        dvh = p.transpose(0, 1, 3, 2) @ dah
        ds = p * (dp - (p * dp).sum(axis=-1, keepdims=True))          # softmax rule; masked entries have p = 0
        dqh = ds @ kh * dh_scale
        dkh = ds.transpose(0, 1, 3, 2) @ qh * dh_scale
        dh1 = np.zeros_like(h1)
        for name, dyh in (("q", dqh), ("k", dkh), ("v", dvh)):
            dpart, grads[f"l{l}.w{name}"], bb = _linear_bwd(_merge(dyh), h1, g("w" + name))
            grads[f"l{l}.b{name}"] = bb.reshape(1, -1)
            dh1 = dh1 + dpart
        if post_ln:                                                # h1 = x
            dx = dx1 + dh1
        else:                                                      # h1 = LN1(x)
            d0, dg1, db1 = _ln_bwd(dh1, c1, g("ln1_g"))
            grads[f"l{l}.ln1_g"], grads[f"l{l}.ln1_b"] = dg1.reshape(1, -1), db1.reshape(1, -1)
            dx = dx1 + d0
    if post_ln:                                                    # x0 = LN_emb(embeddings)
        dx, dg, db = _ln_bwd(dx, cf, P["lnf_g"])
        grads["lnf_g"], grads["lnf_b"] = dg.reshape(1, -1), db.reshape(1, -1)
    # embeddings: tok_emb[tokens] + pos_emb[:T]
    demb = np.zeros_like(P["tok_emb"])
    np.add.at(demb, tokens.reshape(-1), dx.reshape(-1, dx.shape[-1]))
    dpos = np.zeros_like(P["pos_emb"])
    dpos[:T] = dx.sum(axis=0)
    grads["tok_emb"] = grads.get("tok_emb", 0.0) + demb
    grads["pos_emb"] = dpos


def lm_loss_and_gradients(P, tokens, n_layer, n_head, ln_eps=1e-5, act="gelu", post_ln=False):
    """(loss, {name: dL/dtensor}) of forward.lm_loss."""
    tokens = np.asarray(tokens)
    hf, cf, caches = _trunk_fwd(P, tokens, n_layer, n_head, True, None, ln_eps, act, post_ln)
    E = P["tok_emb"]
    logp = F.log_softmax(hf[:, :-1] @ E.T)
    tgt = tokens[:, 1:].astype(np.int64)
    n = tgt.size
    loss = float(-np.take_along_axis(logp, tgt[..., None], axis=-1).mean())
    dlogits = np.exp(logp)
    np.put_along_axis(dlogits, tgt[..., None], np.take_along_axis(dlogits, tgt[..., None], axis=-1) - 1.0, axis=-1)
    dlogits /= n
    grads = {"tok_emb": dlogits.reshape(-1, E.shape[0]).T @ hf[:, :-1].reshape(-1, E.shape[1])}      # the tied head
    dhf = np.zeros_like(hf)
    dhf[:, :-1] = dlogits @ E
    _trunk_bwd(P, tokens, n_layer, n_head, dhf, cf, caches, grads, act, post_ln)
    return loss, grads


def cls_loss_and_gradients(P, tokens, lengths, labels, n_layer, n_head, ln_eps=1e-5, act="gelu", post_ln=False):
    """(loss, {name: dL/dtensor}) of forward.cls_loss."""
    tokens = np.asarray(tokens)
    hf, cf, caches = _trunk_fwd(P, tokens, n_layer, n_head, False, lengths, ln_eps, act, post_ln)
    logits = hf[:, 0] @ P["cls_w"].T + P["cls_b"].reshape(-1)
    logp = F.log_softmax(logits)
    lab = np.asarray(labels).astype(np.int64)
    loss = float(-np.take_along_axis(logp, lab[:, None], axis=-1).mean())
    dlogits = np.exp(logp)
    dlogits[np.arange(lab.size), lab] -= 1.0
    dlogits /= lab.size
    grads = {"cls_w": dlogits.T @ hf[:, 0], "cls_b": dlogits.sum(axis=0).reshape(1, -1)}
    dhf = np.zeros_like(hf)
    dhf[:, 0] = dlogits @ P["cls_w"]
    _trunk_bwd(P, tokens, n_layer, n_head, dhf, cf, caches, grads, act, post_ln)
    return loss, grads


def lsq_gradient(W, X, Y):
    """dL/dW of forward.lsq_loss: (X W^T - Y)^T X / B."""
    X, Y, W = (np.asarray(a, dtype=np.float64) for a in (X, Y, W))
    return (X @ W.T - Y).T @ X / X.shape[0]


# ---------------------------------------------------------------- the basis of one matrix

def gradient_basis(snapshots, k):
    """Orthonormal U [rows, k] spanning the k-dimensional subspace of R^rows that captures the most of the
    stored gradients: the k leading left singular vectors of [G_1 | ... | G_s].  Each column's sign is fixed
    by making its entry of largest magnitude positive (the subspace does not depend on it)."""
    S = np.concatenate([np.asarray(g, dtype=np.float64) for g in snapshots], axis=1)
    U, sv, _ = np.linalg.svd(S, full_matrices=False)
    U = U[:, :k]
    pick = np.abs(U).argmax(axis=0)
    return U * np.sign(U[pick, np.arange(k)])[None, :], sv


def captured_energy(U, snapshots):
    """sum_t ||U^T G_t||_F^2 / sum_t ||G_t||_F^2."""
    U = np.asarray(U, dtype=np.float64)
    num = sum(float(((U.T @ np.asarray(g, dtype=np.float64)) ** 2).sum()) for g in snapshots)
    den = sum(float((np.asarray(g, dtype=np.float64) ** 2).sum()) for g in snapshots)
    return num / den
