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
