"""HIP path vs CPU oracle on seeded random model shapes: layer counts, widths, head sizes, sequence lengths on
both sides of the tile and chunk sizes of the kernels, vocabulary sizes that are multiples of nothing, both
architectures, both storage types and the model-family switches.  One forward loss and one whole ZGR step
(L+, L-, g; restored parameters) per model, at the tolerances of the step tests."""
import numpy as np
import pytest

import zgr_inputs as I
from tests.util import inputs_of, make_batch_arrays, make_oracle, make_session, oracle_loss_fn, session_batch
from tests.test_gpu_step import LOSS_RTOL, _close_params

pytestmark = pytest.mark.gpu


def _random_config(i):
    rng = np.random.default_rng(7100 + i)
    bf16 = bool(i % 2)
    arch = I.ARCH_DECODER_LM if (i // 2) % 2 == 0 else I.ARCH_ENCODER_CLS
    dh = int(rng.choice([64] if bf16 else [8, 16, 32, 64]))
    n_head = int(rng.integers(1, 5))
    d = dh * n_head
    if bf16 and d % 64:
        d = (d + 63) // 64 * 64
    d_ff = int(rng.integers(1, 7)) * 64
    seq = int(rng.choice([3, 17, 64, 129, 200, 333, 520])) if bf16 else int(rng.choice([3, 17, 40, 97]))
    batch = int(rng.integers(1, 5))
    k = int(rng.choice([4, 8, 16, 20]))
    k = min(k, d)
    return I.shrink(I.CONFIGS["cfg3"], name=f"random_{i}", arch=arch, dtype="bf16" if bf16 else "f32", n_layer=int(rng.integers(1, 4)),
                    d_model=d, n_head=n_head, d_ff=d_ff, vocab=int(rng.integers(50, 700)), max_pos=seq + int(rng.integers(0, 9)),
                    n_class=int(rng.integers(2, 6)) if arch == I.ARCH_ENCODER_CLS else 0, batch=batch, seq=seq, k=k, k_full=k + int(rng.choice([0, 4])),
                    tokens="uniform", act=str(rng.choice(["gelu", "relu"])), post_ln=bool(rng.integers(0, 2)))


@pytest.mark.parametrize("i", range(24))
def test_random_model_step_matches_oracle(i, say):
    cfg = _random_config(i)
    say(f"{cfg.name}: {'decoder' if cfg.arch == I.ARCH_DECODER_LM else 'encoder'} {cfg.dtype} L={cfg.n_layer} d={cfg.d_model} heads={cfg.n_head} ff={cfg.d_ff} "
        f"vocab={cfg.vocab} batch={cfg.batch} seq={cfg.seq} k={cfg.k}/{cfg.k_full} {cfg.act}{' post-LN' if cfg.post_ln else ''}")
    specs, values, bases = inputs_of(cfg)
    arrays = make_batch_arrays(cfg)
    o = make_oracle(cfg, specs, values, bases, oracle_loss_fn(cfg, arrays))
    sess = make_session(cfg, specs, values, bases)
    batch = session_batch(sess, cfg, arrays)
    got, want = sess.loss(batch), o.loss()
    assert abs(got - want) <= LOSS_RTOL[cfg.dtype] * abs(want), (got, want)
    lp, lm, g = sess.step(1, batch)
    olp, olm, og = o.step(1)
    assert abs(lp - olp) <= LOSS_RTOL[cfg.dtype] * abs(olp), (lp, olp)
    assert abs(lm - olm) <= LOSS_RTOL[cfg.dtype] * abs(olm), (lm, olm)
    for j, t in enumerate(o.tensors):
        eps_z = np.float32(cfg.eps) * np.abs(o.z_of(t, 1))
        assert _close_params(sess.get_theta(j), t.theta, cfg.dtype, eps_z), t.name
    sess.close()


@pytest.mark.parametrize("i", range(16))
def test_random_model_cloud_gradients_match_oracle(i, say):
    """The cloud's backward pass on the same random shapes: fp32 models entry by entry (2e-4 of a tensor's largest entry),
    bf16 models by direction and norm of every tensor's gradient (their forward half keeps bf16-rounded activations)."""
    from oracle import cloud as C
    cfg = _random_config(i)
    say(f"{cfg.name}: cloud backward, {cfg.dtype}, seq={cfg.seq}, d={cfg.d_model}, {cfg.act}{' post-LN' if cfg.post_ln else ''}")
    specs, values, bases = inputs_of(cfg)
    # matrices scaled up so that attention and the activation leave their linear regime
    gains = (I.ROLE_LN1_G, I.ROLE_LN2_G, I.ROLE_LNF_G)
    values = [v if s.role in gains else (v * np.float32(4)) for s, v in zip(specs, values)]
    arrays = make_batch_arrays(cfg)
    sess = make_session(cfg, specs, values, [None] * len(specs))
    loss, grads = sess.cloud_backward(session_batch(sess, cfg, arrays))
    grads = [g.cpu().numpy().astype(np.float64) for g in grads]
    P = {s.name: v.astype(np.float64) for s, v in zip(specs, values)}
    if cfg.arch == I.ARCH_DECODER_LM:
        loss_or, grads_or = C.lm_loss_and_gradients(P, arrays["x"], cfg.n_layer, cfg.n_head, cfg.ln_eps, cfg.act, cfg.post_ln)
    else:
        loss_or, grads_or = C.cls_loss_and_gradients(P, arrays["x"], arrays["lengths"], arrays["y"], cfg.n_layer, cfg.n_head, cfg.ln_eps, cfg.act, cfg.post_ln)
    assert abs(loss - loss_or) <= LOSS_RTOL[cfg.dtype] * max(1.0, abs(loss_or)), (loss, loss_or)
    top = max(np.abs(g).max() for g in grads_or.values())
    for j, s in enumerate(specs):
        want = grads_or[s.name]
        assert grads[j].shape == want.shape, s.name
        if cfg.dtype == "f32":
            err = np.abs(grads[j] - want).max()
            assert err <= 2e-4 * np.abs(want).max() + 1e-6 * top, (s.name, err, np.abs(want).max())
        elif s.role != I.ROLE_BK and np.linalg.norm(want) > 1e-3 * top:       # the key bias has an identically zero gradient
            cos = float((grads[j] * want).sum() / (np.linalg.norm(grads[j]) * np.linalg.norm(want)))
            ratio = float(np.linalg.norm(grads[j]) / np.linalg.norm(want))
            assert cos >= 0.99 and abs(ratio - 1.0) <= 0.05, (s.name, cos, ratio)
    sess.close()
