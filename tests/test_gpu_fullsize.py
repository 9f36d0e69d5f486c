"""HIP path vs CPU oracle at the full benchmark sizes, in the launch configuration bench.py times.
The oracle cannot afford whole passes at these sizes, so it computes sampled outputs one by one:
Z and the in-place result at random positions of large tensors, and the per-token losses of single
sequences (sequences are independent in the loss).  cfg3 is small enough for one whole step."""
import numpy as np
import pytest

import zgr_inputs as I
from oracle import forward as F
from oracle import perturbation as P
from tests.util import inputs_of, make_batch_arrays, make_oracle, make_session, oracle_loss_fn, session_batch

pytestmark = pytest.mark.gpu


def _sampled_pass_check(sess, cfg, specs, bases, names, step, coef, n_samples=1500, bits=32):
    import torch
    rng = np.random.default_rng(7)
    by_name = {s.name: i for i, s in enumerate(specs)}
    picks = {}
    for name in names:
        i = by_name[name]
        s = specs[i]
        r = rng.integers(0, s.rows, n_samples)
        c = rng.integers(0, s.cols, n_samples)
        # always include the corners and the last row / column
        r[:4] = [0, 0, s.rows - 1, s.rows - 1]
        c[:4] = [0, s.cols - 1, 0, s.cols - 1]
        rt, ct = torch.from_numpy(r).to(sess.dev), torch.from_numpy(c).to(sess.dev)
        picks[name] = (i, r, c, rt, ct, sess.theta[i][rt, ct].float().cpu().numpy())
    sess.perturb(step, float(coef))
    torch.cuda.synchronize()
    for name, (i, r, c, rt, ct, before) in picks.items():
        s = specs[i]
        after = sess.theta[i][rt, ct].float().cpu().numpy()
        U = bases[i]
        z = P.hybrid_z_at(cfg.seed, step, s.tensor_id, s.rows, s.cols, r, c, U, cfg.k if U is not None else 0, cfg.alpha,
                          cfg.scale_mode, bits)
        want = P.axpy_inplace_value(before, coef, z, cfg.dtype)
        assert np.all(np.abs(after - want) <= 1e-2 * np.abs(want) + 1e-30), name
        assert np.mean(after == want) > 0.99, name
        assert abs(np.mean(after != before) - np.mean(want != before)) < 0.02, name      # the pass touched what it should


def test_cfg5_perturbation_pass_sampled():
    cfg = I.CONFIGS["cfg5"]
    specs, values, bases = inputs_of(cfg)
    sess = make_session(cfg, specs, values, bases)
    del values
    names = ["tok_emb", "pos_emb", "l0.wq", "l0.wv", "l11.wo", "l23.w1", "l23.w2", "l5.b1", "l7.ln1_g", "lnf_b"]
    assert bases[[s.name for s in specs].index("l0.wq")].shape == (2048, 64) and cfg.k == 16      # first 16 of 64 columns
    _sampled_pass_check(sess, cfg, specs, bases, names, step=3, coef=np.float32(cfg.eps))
    _sampled_pass_check(sess, cfg, specs, bases, names, step=3, coef=np.float32(-2 * cfg.eps))
    sess.close()


def _sequence_loss_check(cfg, n_seq):
    specs, values, bases = inputs_of(cfg)
    arrays = make_batch_arrays(cfg)
    sess = make_session(cfg, specs, values, bases)
    got_mean = sess.loss(session_batch(sess, cfg, arrays))
    Pd = {s.name: v.astype(np.float64) for s, v in zip(specs, values)}
    del values
    if cfg.arch == I.ARCH_DECODER_LM:
        rows = sess.last_row_losses(cfg.batch * cfg.seq).reshape(cfg.batch, cfg.seq)[:, :-1]
        want = F.lm_token_losses(Pd, arrays["x"][:n_seq], cfg.n_layer, cfg.n_head, cfg.ln_eps)
        got = rows[:n_seq]
        tol = 6e-2 * np.maximum(np.abs(want), 1.0)
    else:
        rows = sess.last_row_losses(cfg.batch)
        want = F.cls_row_losses(Pd, arrays["x"][:n_seq], arrays["lengths"][:n_seq], arrays["y"][:n_seq], cfg.n_layer, cfg.n_head, cfg.ln_eps)
        got = rows[:n_seq]
        tol = 2e-2 * np.maximum(np.abs(want), 1.0)
    assert np.all(np.isfinite(rows)) and np.isfinite(got_mean)
    assert np.all(np.abs(got - want) <= tol), np.abs(got - want).max()
    assert abs(got.mean() - want.mean()) <= 2e-2 * abs(want.mean())          # the per-pass loss tolerance, on the sampled sequences
    if cfg.arch == I.ARCH_DECODER_LM:
        assert abs(got_mean - rows.mean()) <= 1e-5 * abs(got_mean)           # the device's mean is the mean of its rows
    sess.close()


def test_cfg5_forward_losses_of_sampled_sequences():
    _sequence_loss_check(I.CONFIGS["cfg5"], n_seq=1)


def test_cfg4_forward_losses_and_perturbation_sampled():
    cfg = I.CONFIGS["cfg4"]
    _sequence_loss_check(cfg, n_seq=3)
    specs, values, bases = inputs_of(cfg)
    sess = make_session(cfg, specs, values, bases)
    del values
    _sampled_pass_check(sess, cfg, specs, bases, ["tok_emb", "l0.wk", "l23.w2", "cls_w", "cls_b", "l3.b1"], step=1, coef=np.float32(cfg.eps))
    sess.close()


def test_cfg3_whole_step_matches_oracle():
    cfg = I.CONFIGS["cfg3"]
    specs, values, bases = inputs_of(cfg)
    arrays = make_batch_arrays(cfg)
    o = make_oracle(cfg, specs, values, bases, oracle_loss_fn(cfg, arrays))
    sess = make_session(cfg, specs, values, bases)
    batch = session_batch(sess, cfg, arrays)
    lp, lm, g = sess.step(0, batch)
    olp, olm, og = o.step(0)
    assert abs(lp - olp) <= 2e-2 * abs(olp) and abs(lm - olm) <= 2e-2 * abs(olm), (lp, olp, lm, olm)
    sess.apply_update(0, float(og), cfg.lr)
    o.apply_update(0, og, cfg.lr)
    for i, t in enumerate(o.tensors):
        if t.theta.size > 4_000_000 and t.name not in ("tok_emb",):
            continue                                   # the big matrices are covered by the sampled checks; keep the host copies few
        got = sess.get_theta(i)
        eps_z = np.float32(cfg.eps) * np.abs(o.z_of(t, 0))
        # four bf16 roundings lie between the two sides: a second one-ulp flip on the same element (two bf16
        # ulps, 2^-6 relative to the magnitude it was rounded at) may happen on a few elements in 10^7
        dev = np.abs(got - t.theta)
        mag = np.abs(t.theta) + eps_z
        assert np.all(dev <= 2.0 ** -6 * mag + 1e-30), t.name
        assert np.sum(dev > 1e-2 * mag) <= max(1, 1e-5 * got.size), t.name
        assert np.sum(got != t.theta) <= max(2, 0.005 * got.size), t.name
    sess.close()
