"""Workload plumbing shared by bench.py, the smoke entry and the tests: seeded inputs of a configuration
(zgr_inputs) turned into a Session of the HIP path and a device batch.  No arithmetic of the method and nothing
of the oracle in here."""
import zgr_inputs as I

PACK_AFTER_ROLES = (I.ROLE_WK, I.ROLE_WV, I.ROLE_BK, I.ROLE_BV)


def inputs_of(cfg, data_seed=0):
    specs = I.tensor_specs(cfg)
    values = I.make_params(cfg, data_seed, specs)
    bases = [I.make_basis(cfg, s, data_seed) for s in specs]
    return specs, values, bases


def make_batch_arrays(cfg, data_seed=0):
    if cfg.arch == I.ARCH_LINEAR_LSQ:
        x, y = I.make_lsq_data(cfg, data_seed)
        return {"x": x, "y": y, "lengths": None}
    tok = I.make_tokens(cfg, data_seed)
    if cfg.arch == I.ARCH_DECODER_LM:
        return {"x": tok, "y": None, "lengths": None}
    return {"x": tok, "y": I.make_labels(cfg, data_seed), "lengths": I.make_lengths(cfg, data_seed, lo=min(32, max(1, cfg.seq // 8)))}


def make_session(cfg, specs, values, bases, bits=32, scale_mode=None, arch=None, fuse_lr=None):
    from .session import ParamSpec, Session
    params = [ParamSpec(s.name, s.role, s.layer, s.tensor_id, v, u, cfg.k if u is not None else 0)
              for s, v, u in zip(specs, values, bases)]
    pack = tuple(s.name for s in specs if s.role in PACK_AFTER_ROLES)
    return Session(cfg.arch if arch is None else arch, cfg.dtype, params, cfg.seed, cfg.eps, cfg.alpha,
                   cfg.scale_mode if scale_mode is None else scale_mode, bits,
                   n_layer=cfg.n_layer, d_model=cfg.d_model, n_head=cfg.n_head, d_ff=cfg.d_ff, vocab=cfg.vocab,
                   max_pos=cfg.max_pos, n_class=cfg.n_class, ln_eps=cfg.ln_eps,
                   max_batch=max(cfg.batch, 1), max_seq=max(cfg.seq, 2), pack_after=pack, fuse_lr=fuse_lr,
                   act=cfg.act, post_ln=cfg.post_ln)


def session_batch(sess, cfg, arrays):
    return sess.make_batch(arrays["x"], arrays["y"], arrays["lengths"], cfg.seq)
