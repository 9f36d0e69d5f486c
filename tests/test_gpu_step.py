"""HIP path vs CPU oracle for the losses and the whole ZGR step (Algorithm 1):
per-pass losses within 1e-4 (fp32) / 2e-2 (bf16) relative, updated parameters
within 1e-5 (fp32) / 1e-2 (bf16) relative when fed the oracle's g."""
import numpy as np
import pytest

import zgr_inputs as I
from oracle import forward as F
from oracle import perturbation as P
from tests.util import inputs_of, make_batch_arrays, make_oracle, make_session, oracle_loss_fn, session_batch

pytestmark = pytest.mark.gpu

LOSS_RTOL = {"f32": 1e-4, "bf16": 2e-2}
PARAM_RTOL = {"f32": 1e-5, "bf16": 1e-2}
PARAM_SCALE = 0.02

TINY_LM = I.shrink(I.CONFIGS["cfg2"], name="tiny_lm", n_layer=2, d_model=32, n_head=4, d_ff=64, vocab=97,
                   max_pos=16, batch=3, seq=12, k=4, k_full=4)
TINY_CLS = I.shrink(I.CONFIGS["cfg4"], name="tiny_cls", dtype="f32", n_layer=2, d_model=32, n_head=2, d_ff=48,
                    vocab=89, max_pos=16, batch=4, seq=14, tokens="uniform", k=4, k_full=4)
SMALL_BF16_LM = I.shrink(I.CONFIGS["cfg3"], name="small_bf16_lm", n_layer=2, d_model=128, n_head=2, d_ff=256, vocab=1000,
                         max_pos=64, batch=3, seq=40, k=16, k_full=16)
SMALL_BF16_CLS = I.shrink(I.CONFIGS["cfg4"], name="small_bf16_cls", n_layer=2, d_model=128, n_head=2, d_ff=192, vocab=777,
                          max_pos=64, batch=5, seq=33, k=32, k_full=32)
# sequences past the 512 keys the matrix-core attention kernel holds in LDS at a time: three key chunks with a ragged last one
# (decoder, causal), two chunks with padded sequences that end in the first or the second (encoder)
LONG_BF16_LM = I.shrink(SMALL_BF16_LM, name="long_bf16_lm", max_pos=1100, batch=1, seq=1100)
LONG_BF16_CLS = I.shrink(SMALL_BF16_CLS, name="long_bf16_cls", max_pos=700, batch=4, seq=700)
# the two model families of the paper's experiments: ReLU feed-forward (decoder), post-LayerNorm blocks (encoder), and both
VARIANTS = [I.shrink(TINY_LM, name="tiny_lm_relu", act="relu"),
            I.shrink(TINY_CLS, name="tiny_cls_postln", post_ln=True),
            I.shrink(TINY_LM, name="tiny_lm_relu_postln", act="relu", post_ln=True),
            I.shrink(SMALL_BF16_LM, name="small_bf16_lm_relu", act="relu"),
            I.shrink(SMALL_BF16_CLS, name="small_bf16_cls_postln", post_ln=True)]


def _params_dict(specs, values):
    return {s.name: v.astype(np.float64) for s, v in zip(specs, values)}


def _close_params(got, want, dtype, eps_z=None):
    """fp32: 1e-5 relative to the parameter scale.  bf16: 1e-2 relative to the magnitude the value was
    rounded at, |theta| + eps |Z| (a one-ulp flip of theta + eps Z survives the restore pass), and all
    but a few elements identical.  One bf16 ulp is between 2^-8 and 2^-7 of the value, so a single flip
    stays under 1e-2; a value next to a power of two that flips in two of the three passes of a step
    (the device's Z and the oracle's differ by up to 2 ulp fp32, enough to cross a rounding tie) ends
    up to 2^-6 away: allowed for at most max(2, 1e-4 n) elements."""
    if dtype == "f32":
        return np.all(np.abs(got - want) <= PARAM_RTOL["f32"] * (np.abs(want) + PARAM_SCALE))
    worst, beyond, differ = _bf16_margin(got, want, eps_z)
    return worst <= 2.0 ** -6 and beyond <= max(2, 1e-4 * got.size) and differ <= max(2, 0.005 * got.size)


def _bf16_margin(got, want, eps_z=None):
    """(largest |got - want| relative to the rounding magnitude, elements beyond 1e-2 of it, elements that differ)."""
    mag = np.abs(want) + (0.0 if eps_z is None else eps_z)
    dev = np.abs(got - want)
    nz = dev > 1e-30
    worst = float(np.max(dev[nz] / mag[nz])) if np.any(nz) and np.all(mag[nz] > 0) else (float("inf") if np.any(nz) else 0.0)
    return worst, int(np.sum(dev > PARAM_RTOL["bf16"] * mag + 1e-30)), int(np.sum(got != want))


@pytest.mark.parametrize("cfg", [TINY_LM, TINY_CLS, I.CONFIGS["cfg2"], SMALL_BF16_LM, SMALL_BF16_CLS, LONG_BF16_LM, LONG_BF16_CLS] + VARIANTS, ids=lambda c: c.name)
def test_loss_and_row_losses_match_oracle(cfg):
    specs, values, bases = inputs_of(cfg)
    # a 10x larger init than N(0, 0.02) so that attention and the MLP are far from trivial
    values = [v if s.role in (I.ROLE_LN1_G, I.ROLE_LN2_G, I.ROLE_LNF_G) else (P.bf16_round(v * np.float32(8)) if cfg.dtype == "bf16" else v * np.float32(8))
              for s, v in zip(specs, values)]
    arrays = make_batch_arrays(cfg)
    if cfg.name == "long_bf16_cls":
        arrays["lengths"] = np.array([700, 513, 300, 640], dtype=np.int32)      # ends in the second key chunk, one key into it, in the first
    sess = make_session(cfg, specs, values, bases)
    got = sess.loss(session_batch(sess, cfg, arrays))
    Pd = _params_dict(specs, values)
    if cfg.arch == I.ARCH_DECODER_LM:
        rows = F.lm_token_losses(Pd, arrays["x"], cfg.n_layer, cfg.n_head, cfg.ln_eps, cfg.act, cfg.post_ln)
        got_rows = sess.last_row_losses(cfg.batch * cfg.seq).reshape(cfg.batch, cfg.seq)[:, :-1]
    else:
        rows = F.cls_row_losses(Pd, arrays["x"], arrays["lengths"], arrays["y"], cfg.n_layer, cfg.n_head, cfg.ln_eps, cfg.act, cfg.post_ln)
        got_rows = sess.last_row_losses(cfg.batch)
    want = rows.mean()
    assert abs(got - want) <= LOSS_RTOL[cfg.dtype] * abs(want), (got, want)
    tol = 1e-4 if cfg.dtype == "f32" else 6e-2
    assert np.all(np.abs(got_rows - rows) <= tol * np.maximum(np.abs(rows), 1.0)), np.abs(got_rows - rows).max()
    assert rows.std() > 0.05
    sess.close()


@pytest.mark.parametrize("base,kw", [
    (TINY_LM, dict(batch=1, seq=2)),            # the shortest sequence with a next-token target
    (TINY_LM, dict(batch=1, seq=13)),           # odd length, a single sequence
    (SMALL_BF16_LM, dict(batch=1, seq=2)),
    (SMALL_BF16_LM, dict(batch=2, seq=37)),     # not a multiple of any tile
    (SMALL_BF16_LM, dict(batch=2, seq=512)),    # exactly one full key chunk of the matrix-core attention kernel
    (SMALL_BF16_LM, dict(batch=1, seq=513)),    # one key into the second chunk
    (TINY_CLS, dict(batch=1, seq=1)),           # one token: attention over a single key
    (SMALL_BF16_CLS, dict(batch=3, seq=5)),
], ids=lambda x: x.name if hasattr(x, "name") else "-".join(f"{k}{v}" for k, v in x.items()))
def test_degenerate_batch_shapes(base, kw):
    """Loss parity at the smallest and at ragged batch shapes, and with every valid length down to one key."""
    cfg = I.shrink(base, name=base.name + "_edge", max_pos=max(base.max_pos, kw["seq"]), **kw)
    specs, values, bases = inputs_of(cfg)
    arrays = make_batch_arrays(cfg)
    if arrays["lengths"] is not None:
        arrays["lengths"] = np.minimum(np.arange(1, cfg.batch + 1, dtype=np.int32), cfg.seq).astype(np.int32)   # 1, 2, 3 ... valid tokens
    sess = make_session(cfg, specs, values, bases)
    got = sess.loss(session_batch(sess, cfg, arrays))
    Pd = _params_dict(specs, values)
    if cfg.arch == I.ARCH_DECODER_LM:
        want = F.lm_token_losses(Pd, arrays["x"], cfg.n_layer, cfg.n_head, cfg.ln_eps).mean()
    else:
        want = F.cls_row_losses(Pd, arrays["x"], arrays["lengths"], arrays["y"], cfg.n_layer, cfg.n_head, cfg.ln_eps).mean()
    assert np.isfinite(got) and abs(got - want) <= LOSS_RTOL[cfg.dtype] * abs(want), (got, want)
    sess.close()


def test_cfg1_trajectory_matches_oracle():
    cfg = I.CONFIGS["cfg1"]
    specs, values, bases = inputs_of(cfg)
    arrays = make_batch_arrays(cfg)
    o = make_oracle(cfg, specs, values, bases, oracle_loss_fn(cfg, arrays))
    sess = make_session(cfg, specs, values, bases)
    batch = session_batch(sess, cfg, arrays)
    worst_own = 0.0
    for step in range(cfg.steps):
        lp, lm, g = sess.step(step, batch)
        olp, olm, og = o.step(step)
        assert abs(lp - olp) <= LOSS_RTOL["f32"] * abs(olp) and abs(lm - olm) <= LOSS_RTOL["f32"] * abs(olm)
        # restore: parameters are back (to rounding) on both sides
        assert _close_params(sess.get_theta(0), o.tensors[0].theta, "f32")
        # g amplifies loss error by 1/(2 eps): the bound is |dL| / (2 eps) with fp32 losses ~1e-6 relative
        assert abs(g - og) <= 2e-6 * abs(olp) / (2 * cfg.eps) + 1e-4 * abs(og)
        worst_own = max(worst_own, abs(g - og))
        # decoupled update: both sides apply the oracle's g
        sess.apply_update(step, float(og), cfg.lr)
        o.apply_update(step, og, cfg.lr)
        assert _close_params(sess.get_theta(0), o.tensors[0].theta, "f32")
    final = sess.loss(batch)
    assert abs(final - o.loss()) <= 1e-6 * abs(final)
    sess.close()


@pytest.mark.parametrize("cfg", [I.CONFIGS["cfg2"], SMALL_BF16_LM, SMALL_BF16_CLS, TINY_CLS] + VARIANTS[2:], ids=lambda c: c.name)
@pytest.mark.parametrize("bits", [32, 16])
def test_step_and_update_match_oracle(cfg, bits, say):
    steps = 3 if cfg.name == "cfg2" else 2
    loss_dev, worst, beyond, differ, n_el = 0.0, 0.0, 0, 0, 0
    specs, values, bases = inputs_of(cfg)
    arrays = make_batch_arrays(cfg)
    o = make_oracle(cfg, specs, values, bases, oracle_loss_fn(cfg, arrays), bits=bits)
    sess = make_session(cfg, specs, values, bases, bits=bits)
    batch = session_batch(sess, cfg, arrays)
    for step in range(steps):
        lp, lm, g = sess.step(step, batch)
        olp, olm, og = o.step(step)
        assert abs(lp - olp) <= LOSS_RTOL[cfg.dtype] * abs(olp), (lp, olp)
        assert abs(lm - olm) <= LOSS_RTOL[cfg.dtype] * abs(olm), (lm, olm)
        loss_dev = max(loss_dev, abs(lp - olp) / abs(olp), abs(lm - olm) / abs(olm))
        eps_z = [np.float32(cfg.eps) * np.abs(o.z_of(t, step)) for t in o.tensors]
        for i, t in enumerate(o.tensors):
            assert _close_params(sess.get_theta(i), t.theta, cfg.dtype, eps_z[i]), t.name
        sess.apply_update(step, float(og), cfg.lr)
        o.apply_update(step, og, cfg.lr)
        for i, t in enumerate(o.tensors):
            got = sess.get_theta(i)
            assert _close_params(got, t.theta, cfg.dtype, eps_z[i]), t.name
            if cfg.dtype == "bf16":
                w, b, d = _bf16_margin(got, t.theta, eps_z[i])
                worst, beyond, differ, n_el = max(worst, w), beyond + b, differ + d, n_el + got.size
            # keep the two sides on the same trajectory: bf16 roundings may legitimately differ by one ulp
            t.theta = got.copy()
    # the achieved maxima beside their bounds, so that the margin shows in the log
    if cfg.dtype == "bf16":
        say("%s %d-bit: losses within %.1e of the oracle's (bound %.0e); after the updates %d of %d elements differ (bound %.1f %%), "
            "%d beyond 1e-2 of the rounding magnitude, largest %.2e (bound 2^-6 = 1.56e-2)"
            % (cfg.name, bits, loss_dev, LOSS_RTOL["bf16"], differ, n_el, 0.5, beyond, worst))
    else:
        say("%s %d-bit: losses within %.1e of the oracle's (bound %.0e)" % (cfg.name, bits, loss_dev, LOSS_RTOL["f32"]))
    sess.close()


@pytest.mark.parametrize("cfg", [I.CONFIGS["cfg1"], I.CONFIGS["cfg2"], SMALL_BF16_LM, SMALL_BF16_CLS], ids=lambda c: c.name)
def test_fused_restore_update_matches_oracle(cfg):
    """zgr_step with fuse_restore_update = 1: the last pass adds (eps - lr g) Z.  Each side uses its own g
    (it cannot be injected), so the parameter bound carries lr |Z| |g - g_oracle| on top of the usual one."""
    lr = cfg.lr if cfg.dtype == "f32" else 1e-4        # large enough to move bf16 weights
    specs, values, bases = inputs_of(cfg)
    arrays = make_batch_arrays(cfg)
    o = make_oracle(cfg, specs, values, bases, oracle_loss_fn(cfg, arrays))
    sess = make_session(cfg, specs, values, bases, fuse_lr=lr)
    batch = session_batch(sess, cfg, arrays)
    for step in range(2):
        before = [t.theta.copy() for t in o.tensors]
        lp, lm, g = sess.step(step, batch)
        olp, olm, og = o.step(step, fuse_lr=lr)
        assert abs(lp - olp) <= LOSS_RTOL[cfg.dtype] * abs(olp) and abs(lm - olm) <= LOSS_RTOL[cfg.dtype] * abs(olm)
        moved = 0
        for i, t in enumerate(o.tensors):
            z = np.abs(o.z_of(t, step))
            got = sess.get_theta(i)
            slack = lr * z * abs(g - og)
            if cfg.dtype == "f32":
                assert np.all(np.abs(got - t.theta) <= PARAM_RTOL["f32"] * (np.abs(t.theta) + PARAM_SCALE) + slack), t.name
            else:
                mag = np.abs(t.theta) + np.float32(cfg.eps) * z
                # the device's own g shifts the pre-rounding value by slack: allow that plus one bf16 ulp of it
                assert np.all(np.abs(got - t.theta) <= PARAM_RTOL["bf16"] * mag + 1.01 * slack + 1e-30), t.name
            moved += int(np.sum(t.theta != before[i]))
            t.theta = got.copy()
        assert moved > 0 and og != 0
    sess.close()


@pytest.mark.parametrize("cfg", [I.CONFIGS["cfg1"], I.CONFIGS["cfg2"], SMALL_BF16_LM, SMALL_BF16_CLS], ids=lambda c: c.name)
@pytest.mark.parametrize("n,bits", [(1, 32), (3, 32), (8, 16), (11, 32)])
def test_batched_update_matches_oracle(cfg, n, bits):
    """zgr_apply_updates: theta - lr sum_q g_q Z(seed, step_q) in one pass per 8 perturbations (n = 11 takes two
    passes; the oracle is then applied in the same two groups)."""
    rng = np.random.default_rng(100 + n)
    steps = [int(x) for x in rng.integers(0, 1000, size=n)]
    gs = [float(x) for x in rng.standard_normal(n)]
    lr = cfg.lr if cfg.dtype == "f32" else 3e-3          # moves bf16 weights by several ulps
    specs, values, bases = inputs_of(cfg)
    arrays = make_batch_arrays(cfg)
    o = make_oracle(cfg, specs, values, bases, oracle_loss_fn(cfg, arrays), bits=bits)
    sess = make_session(cfg, specs, values, bases, bits=bits, arch=-1)
    before = [t.theta.copy() for t in o.tensors]
    sess.apply_updates(steps, gs, lr)
    for i0 in range(0, n, 8):
        o.apply_updates(steps[i0:i0 + 8], gs[i0:i0 + 8], lr)
    moved = 0
    for i, t in enumerate(o.tensors):
        got = sess.get_theta(i)
        if cfg.dtype == "f32":
            assert np.all(np.abs(got - t.theta) <= PARAM_RTOL["f32"] * (np.abs(t.theta) + PARAM_SCALE)), t.name
            # far tighter in fact: two roundings of theta plus 1e-5 of the coefficients (2-ulp Gaussians and k-term
            # fp32 dot products, both O(1) before scaling; a G and U R may cancel in Z, so |Z| itself is no yardstick)
            csum = sum(abs(np.float32(lr) * np.float32(g)) for g in gs)
            assert np.all(np.abs(got - t.theta) <= 2 * np.spacing(np.abs(t.theta)) + 1e-5 * csum), t.name
        else:
            # relative to the magnitude of what was summed: theta and the update may cancel
            mag = np.abs(before[i]).astype(np.float64)
            for st, g in zip(steps, gs):
                mag = mag + abs(np.float32(lr) * np.float32(g)) * np.abs(o.z_of(t, st))
            assert _close_params(got, t.theta, "bf16", mag), t.name
        moved += int(np.sum(t.theta != before[i]))
    assert moved > 0.2 * sum(t.theta.size for t in o.tensors)
    sess.close()


@pytest.mark.parametrize("name", ["cfg1", "cfg2"])
def test_multi_query_client_round(name):
    """The n-query client of Algorithm 1 (local steps t = 1..n before one aggregation): n client blocks with
    different step indices, each leaving the parameters restored, then one batched update with weights 1/n.
    Losses and g of every query against the oracle; the update is decoupled (both sides apply the oracle's g)."""
    cfg = I.CONFIGS[name]
    n = 3
    specs, values, bases = inputs_of(cfg)
    arrays = make_batch_arrays(cfg)
    o = make_oracle(cfg, specs, values, bases, oracle_loss_fn(cfg, arrays))
    sess = make_session(cfg, specs, values, bases)
    batch = session_batch(sess, cfg, arrays)
    for rnd in range(2):
        steps = [rnd * n + q for q in range(n)]
        ogs = []
        for st in steps:
            lp, lm, g = sess.step(st, batch)
            olp, olm, og = o.step(st)
            assert abs(lp - olp) <= LOSS_RTOL[cfg.dtype] * abs(olp) and abs(lm - olm) <= LOSS_RTOL[cfg.dtype] * abs(olm)
            assert abs(g - og) <= 2e-6 * abs(olp) / (2 * cfg.eps) + 1e-4 * abs(og)
            ogs.append(float(og) / n)
        sess.apply_updates(steps, ogs, cfg.lr)
        o.apply_updates(steps, ogs, cfg.lr)
        for i, t in enumerate(o.tensors):
            assert _close_params(sess.get_theta(i), t.theta, cfg.dtype), (rnd, t.name)
    sess.close()


def test_batched_update_rejects_bad_arguments():
    cfg = I.CONFIGS["cfg1"]
    specs, values, bases = inputs_of(cfg)
    sess = make_session(cfg, specs, values, bases, arch=-1)
    before = sess.get_theta(0).copy()
    sess.apply_updates([], [], 1e-2)                       # n = 0: no-op
    assert np.array_equal(sess.get_theta(0), before)
    with pytest.raises(Exception):
        sess.apply_updates([1 << 32], [1.0], 1e-2)
    with pytest.raises(Exception):
        sess.apply_updates([1, 2], [1.0, float("nan")], 1e-2)
    assert np.array_equal(sess.get_theta(0), before)
    sess.close()


def test_cfg2_full_trajectory_with_own_g():
    """20 steps of cfg2 driven by the device's own g; the deviation from the oracle's trajectory is
    bounded by lr |Z| |dL_err| / (2 eps) per step and reported."""
    cfg = I.CONFIGS["cfg2"]
    specs, values, bases = inputs_of(cfg)
    arrays = make_batch_arrays(cfg)
    o = make_oracle(cfg, specs, values, bases, oracle_loss_fn(cfg, arrays))
    sess = make_session(cfg, specs, values, bases)
    batch = session_batch(sess, cfg, arrays)
    for step in range(cfg.steps):
        lp, lm, g = sess.step(step, batch)
        olp, olm, og = o.step(step)
        assert abs(lp - olp) <= 1e-4 * abs(olp) and abs(lm - olm) <= 1e-4 * abs(olm)
        sess.apply_update(step, g, cfg.lr)
        o.apply_update(step, og, cfg.lr)
    dev = max(np.abs(sess.get_theta(i) - t.theta).max() for i, t in enumerate(o.tensors))
    # fp32 loss error ~1e-6 * 7 -> g error ~4e-3 -> lr * 6 sigma * that per step, 20 steps
    assert dev <= 20 * cfg.lr * 6.0 * 5e-3 + 1e-7, dev
    sess.close()


def test_seed_replay_by_a_context_without_model():
    """The edge server regenerates the update from (step, g) alone."""
    cfg = I.CONFIGS["cfg1"]
    specs, values, bases = inputs_of(cfg)
    arrays = make_batch_arrays(cfg)
    client = make_session(cfg, specs, values, bases)
    server = make_session(cfg, specs, values, bases, arch=-1)
    batch = session_batch(client, cfg, arrays)
    for step in range(4):
        _, _, g = client.step(step, batch)
        client.apply_update(step, g, cfg.lr)
        server.apply_update(step, g, cfg.lr)
    assert np.allclose(client.get_theta(0), server.get_theta(0), rtol=0, atol=1e-7)
    with pytest.raises(Exception):
        server.loss(batch)
    client.close(); server.close()


@pytest.mark.parametrize("fused", [False, True])
def test_non_finite_loss_is_reported_and_parameters_are_restored_lsq(fused):
    """A NaN in the batch makes both losses NaN: zgr_step must say so (ZGR_ERR_NONFINITE), leave the parameters
    restored within the restore bound, and, with the fused last pass, apply no update."""
    from paper_2601_12917_amd import binding as B
    cfg = I.CONFIGS["cfg1"]
    specs, values, bases = inputs_of(cfg)
    arrays = make_batch_arrays(cfg)
    bad = {k: (None if v is None else v.copy()) for k, v in arrays.items()}
    bad["x"][3, 17] = np.nan
    sess = make_session(cfg, specs, values, bases, fuse_lr=cfg.lr if fused else None)
    batch_bad = session_batch(sess, cfg, bad)
    with pytest.raises(B.ZgrError) as ei:
        sess.step(0, batch_bad)
    assert ei.value.status == B.ZGR_ERR_NONFINITE
    got = sess.get_theta(0)
    # three fp32 passes +eps Z, -2 eps Z, +eps Z: back to within a few ulp of the magnitude reached in between
    o = make_oracle(cfg, specs, values, bases, oracle_loss_fn(cfg, arrays))
    z = np.abs(o.z_of(o.tensors[0], 0))
    bound = 4 * np.spacing((np.abs(values[0]) + np.float32(cfg.eps) * z).astype(np.float32))
    assert np.all(np.isfinite(got)) and np.all(np.abs(got - values[0]) <= bound)
    # the context is still usable: a clean batch gives the oracle's losses, from the restored parameters
    good = session_batch(sess, cfg, arrays)
    lp, lm, g = sess.step(1, good)
    olp, olm, og = o.step(1, fuse_lr=cfg.lr if fused else None)
    assert abs(lp - olp) <= LOSS_RTOL["f32"] * abs(olp) and abs(lm - olm) <= LOSS_RTOL["f32"] * abs(olm)
    sess.close()


@pytest.mark.parametrize("cfg", [TINY_LM, SMALL_BF16_LM], ids=lambda c: c.name)
@pytest.mark.parametrize("fused", [False, True])
def test_non_finite_loss_is_reported_and_parameters_are_restored_lm(cfg, fused):
    """A loss out of range: a final LayerNorm gain of 3e38 overflows the hidden state, so the cross-entropy is not
    finite.  ZGR_ERR_NONFINITE, every parameter back within the restore bound, no update in fused mode."""
    from paper_2601_12917_amd import binding as B
    specs, values, bases = inputs_of(cfg)
    arrays = make_batch_arrays(cfg)
    values = [v.copy() for v in values]
    gi = [s.name for s in specs].index("lnf_g")
    values[gi][...] = np.float32(3e38) if cfg.dtype == "f32" else P.bf16_round(np.array([3e38], np.float32))[0]
    lr = cfg.lr if cfg.dtype == "f32" else 1e-4
    sess = make_session(cfg, specs, values, bases, fuse_lr=lr if fused else None)
    batch = session_batch(sess, cfg, arrays)
    with pytest.raises(B.ZgrError) as ei:
        sess.step(0, batch)
    assert ei.value.status == B.ZGR_ERR_NONFINITE
    o = make_oracle(cfg, specs, values, bases, oracle_loss_fn(cfg, arrays))
    eps = np.float32(cfg.eps)
    for c in (eps, np.float32(-2.0) * eps, eps):      # the three passes of the client block, and nothing else
        o.axpy_all(0, c)
    for i, t in enumerate(o.tensors):
        got = sess.get_theta(i)
        eps_z = eps * np.abs(o.z_of(t, 0))
        assert np.all(np.isfinite(got)), t.name
        if cfg.dtype == "f32":
            assert np.all(np.abs(got - values[i]) <= 4 * np.spacing((np.abs(values[i]) + eps_z).astype(np.float32))), t.name
        # bf16 storage does not return to the starting values exactly (three roundings): the oracle's three passes do the same
        assert _close_params(got, t.theta, cfg.dtype, eps_z), t.name
    sess.close()
