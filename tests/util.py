"""Shared helpers of the tests: the same seeded inputs for the CPU oracle and the HIP path."""
import numpy as np

import zgr_inputs as I
from paper_2601_12917_amd.workloads import PACK_AFTER_ROLES, inputs_of, make_batch_arrays, make_session, session_batch  # noqa: F401


def make_oracle(cfg, specs, values, bases, loss_fn, bits=32, scale_mode=None, dtype=None, keep_z=False):
    from oracle.zgr import Tensor, ZgrOracle
    tens = [Tensor(s.name, v, s.tensor_id, u, cfg.k if u is not None else 0) for s, v, u in zip(specs, values, bases)]
    return ZgrOracle(tens, loss_fn, cfg.seed, cfg.eps, cfg.alpha, dtype or cfg.dtype,
                     cfg.scale_mode if scale_mode is None else scale_mode, bits, keep_z=keep_z)


def oracle_loss_fn(cfg, batch):
    from oracle import zgr as Z
    if cfg.arch == I.ARCH_LINEAR_LSQ:
        return Z.make_lsq_loss(batch["x"], batch["y"])
    if cfg.arch == I.ARCH_DECODER_LM:
        return Z.make_lm_loss(batch["x"], cfg.n_layer, cfg.n_head, cfg.ln_eps, cfg.act, cfg.post_ln)
    return Z.make_cls_loss(batch["x"], batch["lengths"], batch["y"], cfg.n_layer, cfg.n_head, cfg.ln_eps, cfg.act, cfg.post_ln)


def ulp_diff(got, want):
    """|got - want| in units of ulp(want), fp32."""
    want = np.asarray(want, dtype=np.float32)
    ulp = np.spacing(np.abs(want)).astype(np.float64)
    return np.abs(np.asarray(got, dtype=np.float64) - want.astype(np.float64)) / ulp
