"""Bases streamed from host memory layer by layer (Sec. 3.3): every step of a session whose bases are
streamed is compared with the CPU oracle (losses, restored and updated parameters, Z of a streamed tensor),
for fp32 bases and for 4-bit codes, over several passes so that both staging slots are reused; as an extra,
the result of every pass is bit-identical to the resident-basis path (same kernels, same operands)."""
import numpy as np
import pytest

import zgr_inputs as I
from oracle import dtc as D
from oracle import perturbation as P
from tests.test_gpu_perturb import _z_bound
from tests.test_gpu_step import LOSS_RTOL, _close_params
from tests.util import inputs_of, make_batch_arrays, make_oracle, make_session, oracle_loss_fn, session_batch

pytestmark = pytest.mark.gpu

DEEP_F32 = I.shrink(I.CONFIGS["cfg2"], name="deep_f32", n_layer=5, d_model=64, n_head=4, d_ff=128, vocab=211,
                    max_pos=32, batch=2, seq=16, k=8, k_full=8)
DEEP_BF16 = I.shrink(I.CONFIGS["cfg3"], name="deep_bf16", n_layer=4, d_model=128, n_head=2, d_ff=256, vocab=500,
                     max_pos=32, batch=2, seq=24, k=16, k_full=24)


def _guided(specs, bases):
    return [i for i, (s, u) in enumerate(zip(specs, bases)) if u is not None]


@pytest.mark.parametrize("cfg", [DEEP_F32, DEEP_BF16], ids=lambda c: c.name)
@pytest.mark.parametrize("mode,stage_tiles", [("f32", 1), ("q4", 1), ("mixed", 1), ("f32", 20), ("q4", None)])
def test_streamed_bases_give_identical_steps(cfg, mode, stage_tiles):
    """stage_tiles = 1: one pipeline stage per layer; 20: two or three of these small layers per stage;
    None: the default, which puts all of such a small model into one stage."""
    specs, values, bases = inputs_of(cfg)
    arrays = make_batch_arrays(cfg)
    res = make_session(cfg, specs, values, bases)
    spc = make_session(cfg, specs, values, bases)
    if stage_tiles is not None:
        spc.set_stage_tiles(stage_tiles)
    for i in _guided(specs, bases):
        k = cfg.k
        if mode == "q4" or (mode == "mixed" and specs[i].layer % 2 == 1):
            lam, delta = D.affine_params(bases[i][:, :k], 4)
            packed = D.pack_nibbles(D.quantize(bases[i][:, :k], lam, delta, 4))
            res.set_basis_q4(i, packed, k, lam, delta)
            if mode == "q4":
                spc.set_basis_host(i, None, k, codes=packed, lam=lam, delta=delta)
            else:
                spc.set_basis_q4(i, packed, k, lam, delta)          # odd layers stay resident (compressed)
        else:
            spc.set_basis_host(i, bases[i], k)                       # full rows of k_full columns, first k used
    bres, bspc = session_batch(res, cfg, arrays), session_batch(spc, cfg, arrays)
    for step in range(3):
        r = res.step(step, bres); s = spc.step(step, bspc)
        assert r == s, (step, r, s)
        res.apply_update(step, r[2], 10 * cfg.lr); spc.apply_update(step, s[2], 10 * cfg.lr)
        for i in range(len(specs)):
            assert np.array_equal(res.get_theta(i), spc.get_theta(i)), (step, specs[i].name)
    res.apply_updates([7, 8, 9], [0.5, -0.25, 1.0], cfg.lr); spc.apply_updates([7, 8, 9], [0.5, -0.25, 1.0], cfg.lr)
    for i in range(len(specs)):
        assert np.array_equal(res.get_theta(i), spc.get_theta(i)), specs[i].name
    g = _guided(specs, bases)
    assert len({specs[i].layer for i in g}) >= 4
    i = g[len(g) // 2]
    assert np.array_equal(res.fill_z(i, 3), spc.fill_z(i, 3))
    res.close(); spc.close()


@pytest.mark.parametrize("cfg", [DEEP_F32, DEEP_BF16], ids=lambda c: c.name)
@pytest.mark.parametrize("mode,stage_tiles", [("f32", 1), ("q4", 1), ("mixed", 20)])
def test_streamed_session_matches_oracle(cfg, mode, stage_tiles):
    """The streamed path against the oracle itself: the oracle is given the basis each tensor really uses (the
    first k columns as sent, or what the 4-bit codes restore to) and runs the same steps; losses within the
    per-pass tolerance, parameters after the restoring pass and after the update (both sides apply the oracle's
    g) within the parameter tolerance, and Z of a streamed tensor within the Gaussian / dot-product bound."""
    specs, values, bases = inputs_of(cfg)
    arrays = make_batch_arrays(cfg)
    spc = make_session(cfg, specs, values, bases)
    spc.set_stage_tiles(stage_tiles)
    used = list(bases)                     # per tensor: the basis the kernels end up contracting with
    for i in _guided(specs, bases):
        k = cfg.k
        if mode == "q4" or (mode == "mixed" and specs[i].layer % 2 == 1):
            lam, delta = D.affine_params(bases[i][:, :k], 4)
            codes = D.quantize(bases[i][:, :k], lam, delta, 4)
            spc.set_basis_host(i, None, k, codes=D.pack_nibbles(codes), lam=lam, delta=delta)
            used[i] = D.dequantize(codes, lam, delta)
        else:
            spc.set_basis_host(i, bases[i], k)
    o = make_oracle(cfg, specs, values, used, oracle_loss_fn(cfg, arrays))
    batch = session_batch(spc, cfg, arrays)
    lr = cfg.lr if cfg.dtype == "f32" else 1e-4
    for step in range(3):
        lp, lm, g = spc.step(step, batch)
        olp, olm, og = o.step(step)
        assert abs(lp - olp) <= LOSS_RTOL[cfg.dtype] * abs(olp), (step, lp, olp)
        assert abs(lm - olm) <= LOSS_RTOL[cfg.dtype] * abs(olm), (step, lm, olm)
        eps_z = [np.float32(cfg.eps) * np.abs(o.z_of(t, step)) for t in o.tensors]
        for i, t in enumerate(o.tensors):
            assert _close_params(spc.get_theta(i), t.theta, cfg.dtype, eps_z[i]), (step, t.name)
        spc.apply_update(step, float(og), lr)
        o.apply_update(step, og, lr)
        for i, t in enumerate(o.tensors):
            got = spc.get_theta(i)
            assert _close_params(got, t.theta, cfg.dtype, eps_z[i]), (step, t.name)
            t.theta = got.copy()           # same trajectory on both sides (bf16 roundings may differ by an ulp)
    g_idx = _guided(specs, bases)
    assert len({specs[i].layer for i in g_idx}) >= 4
    for i in (g_idx[0], g_idx[len(g_idx) // 2], g_idx[-1]):
        s_ = specs[i]
        G, R, Z = P.hybrid_z(cfg.seed, 9, s_.tensor_id, s_.rows, s_.cols, used[i], cfg.k, cfg.alpha, cfg.scale_mode, 32, parts=True)
        got = spc.fill_z(i, 9)
        assert np.all(np.abs(got.astype(np.float64) - Z) <= _z_bound(cfg, G, R, used[i], cfg.k, s_.rows, s_.cols, cfg.scale_mode)), s_.name
    spc.close()


@pytest.mark.parametrize("codes", [False, True])
def test_layer_blocks_travel_as_one_transfer_and_give_identical_steps(codes):
    """A layer's bases packed in one pinned block in staging-slot layout (the single-transfer path)."""
    cfg = DEEP_BF16
    specs, values, bases = inputs_of(cfg)
    arrays = make_batch_arrays(cfg)
    res = make_session(cfg, specs, values, bases)
    spc = make_session(cfg, specs, values, bases)
    spc.set_stage_tiles(1)
    layers = {}
    for i in _guided(specs, bases):
        layers.setdefault(specs[i].layer, []).append(i)
    for layer, idx in layers.items():
        if codes:
            q = []
            for i in idx:
                lam, delta = D.affine_params(bases[i][:, :cfg.k], 4)
                packed = D.pack_nibbles(D.quantize(bases[i][:, :cfg.k], lam, delta, 4))
                res.set_basis_q4(i, packed, cfg.k, lam, delta)
                q.append((packed, lam, delta))
            spc.set_layer_bases_host(idx, [x[0] for x in q], cfg.k, codes=True, lams=[x[1] for x in q], deltas=[x[2] for x in q])
        else:
            spc.set_layer_bases_host(idx, [bases[i] for i in idx], cfg.k)
    bres, bspc = session_batch(res, cfg, arrays), session_batch(spc, cfg, arrays)
    for step in range(3):
        r = res.step(step, bres); s = spc.step(step, bspc)
        assert r == s
        res.apply_update(step, r[2], 10 * cfg.lr); spc.apply_update(step, s[2], 10 * cfg.lr)
    for i in range(len(specs)):
        assert np.array_equal(res.get_theta(i), spc.get_theta(i)), specs[i].name
    res.close(); spc.close()


def test_streamed_basis_can_be_replaced_and_is_bounded_by_the_workspace():
    cfg = DEEP_F32
    specs, values, bases = inputs_of(cfg)
    sess = make_session(cfg, specs, values, bases)
    sess.set_stage_tiles(1)
    g = _guided(specs, bases)
    i = g[0]
    z_res = sess.fill_z(i, 5)
    sess.set_basis_host(i, bases[i], cfg.k)
    assert np.array_equal(sess.fill_z(i, 5), z_res)
    sess.set_basis(i, bases[i], cfg.k)                               # back to a resident basis
    assert np.array_equal(sess.fill_z(i, 5), z_res)
    # the staging slots were sized for rank cfg.k: a layer streamed at eight times that rank does not fit
    refused = False
    for j in g:
        if specs[j].layer == specs[i].layer:
            rows = bases[j].shape[0]
            wide = np.linalg.qr(np.random.default_rng(j).standard_normal((rows, 8 * cfg.k)))[0].astype(np.float32)
            try:
                sess.set_basis_host(j, wide, 8 * cfg.k)
            except Exception:
                refused = True
                break
    assert refused
    for j in g:
        if specs[j].layer == specs[i].layer:
            sess.set_basis(j, bases[j], cfg.k)
    assert np.array_equal(sess.fill_z(i, 5), z_res)                  # back on resident bases, nothing else changed
    # pageable host memory is refused (the kernels read the bases themselves: they must be pinned and mapped)
    from paper_2601_12917_amd import binding as B
    pageable = np.ascontiguousarray(bases[i][:, :cfg.k])
    st = sess.lib.zgr_set_basis_host(sess.ctx, i, pageable.ctypes.data, cfg.k, 32, 0.0, 0.0)
    assert st == B.ZGR_ERR_CONFIG
    assert np.array_equal(sess.fill_z(i, 5), z_res)
    sess.close()
