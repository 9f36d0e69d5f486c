"""HIP path vs CPU oracle for the cloud's backward pass (cloud block of Algorithm 1: back-propagation on the public
dataset, whose gradients build the basis): zgr_cloud_backward against oracle.cloud on the same seeded parameters and batches, tensor by tensor.

Tolerances.  fp32 models: every intermediate result is fp32 on the device and fp64 in the oracle, sums run over at
most a few thousand terms, so a gradient entry differs by a few 1e-6 of the tensor's largest entry; the bound is
2e-4 of it (rounding in the softmax and LayerNorm chains is amplified by their 1 / sigma factors).  bf16 models: the
forward half keeps what the client's forward keeps, bf16-rounded activations (2^-9 relative each), and the weights
are bf16 values the oracle reads exactly; over two blocks that is a few per cent of a tensor's norm, so the test
asks for the direction (cosine >= 0.995) and the norm (within 5 %) of every matrix's gradient, not its entries."""
import numpy as np
import pytest

import zgr_inputs as I
from oracle import cloud as C

pytestmark = pytest.mark.gpu

LN_GAINS = (I.ROLE_LN1_G, I.ROLE_LN2_G, I.ROLE_LNF_G)


def _setup(cfg, scale=4.0, data_seed=0):
    """Session and oracle parameters: the seeded initial values, matrices scaled up so that attention and GELU leave
    their linear regime (the gradient rules of softmax and LayerNorm then carry weight)."""
    from tests.util import make_session
    specs = I.tensor_specs(cfg)
    values = [v if s.role in LN_GAINS else (v * scale).astype(np.float32) for s, v in zip(specs, I.make_params(cfg, data_seed, specs))]
    if cfg.dtype == "bf16":
        import torch
        values = [torch.from_numpy(v).bfloat16().float().numpy() for v in values]
    sess = make_session(cfg, specs, values, [None] * len(specs))
    P = {s.name: v.astype(np.float64) for s, v in zip(specs, values)}
    return sess, specs, P


def _batch(cfg, data_seed):
    from tests.util import make_batch_arrays
    return make_batch_arrays(cfg, data_seed)


def _oracle(cfg, P, arrays):
    if cfg.arch == I.ARCH_DECODER_LM:
        return C.lm_loss_and_gradients(P, arrays["x"], cfg.n_layer, cfg.n_head, cfg.ln_eps, cfg.act, cfg.post_ln)
    return C.cls_loss_and_gradients(P, arrays["x"], arrays["lengths"], arrays["y"], cfg.n_layer, cfg.n_head, cfg.ln_eps, cfg.act, cfg.post_ln)


def _device(sess, cfg, arrays):
    from tests.util import session_batch
    loss, grads = sess.cloud_backward(session_batch(sess, cfg, arrays))
    return loss, [g.cpu().numpy().astype(np.float64) for g in grads]


TINY_LM = dict(name="bw_lm", n_layer=2, d_model=64, n_head=4, d_ff=192, vocab=211, max_pos=40, batch=3, seq=37, k=8, k_full=8)
TINY_CLS = dict(name="bw_cls", arch=I.ARCH_ENCODER_CLS, n_class=3, n_layer=2, d_model=64, n_head=2, d_ff=128, vocab=157, max_pos=48, batch=5, seq=41, k=8, k_full=8)


VARIANT_KW = {"lm_relu": dict(TINY_LM, name="bw_lm_relu", act="relu"), "cls_postln": dict(TINY_CLS, name="bw_cls_postln", post_ln=True),
              "lm_relu_postln": dict(TINY_LM, name="bw_lm_relu_postln", act="relu", post_ln=True),
              # sequences past 256 tokens: a thread of the row-wise softmax rule holds two entries of a row, the [T, T] buffers span
              # five 64-wide tiles with a ragged last one
              "lm_long": dict(TINY_LM, name="bw_lm_long", n_layer=1, d_model=32, n_head=2, d_ff=64, vocab=101, max_pos=320, batch=2, seq=300),
              "cls_long": dict(TINY_CLS, name="bw_cls_long", n_layer=1, d_model=32, n_head=2, d_ff=64, vocab=101, max_pos=320, batch=3, seq=290)}


@pytest.mark.parametrize("which", ["lm", "cls", "cfg2", "lm_relu", "cls_postln", "lm_relu_postln", "lm_long", "cls_long"])
def test_fp32_gradients_match_the_oracle_entry_by_entry(which, say):
    """The default model (pre-LayerNorm, erf-GELU) and the two switches of the paper's model families."""
    cfg = I.CONFIGS["cfg2"] if which == "cfg2" else I.shrink(I.CONFIGS["cfg2"], **(VARIANT_KW[which] if which in VARIANT_KW else TINY_LM if which == "lm" else TINY_CLS))
    sess, specs, P = _setup(cfg)
    theta_before = [sess.get_theta(i).copy() for i in range(len(specs))]
    arrays = _batch(cfg, 1)
    say(f"cloud backward fp32 {which}: {len(specs)} tensors")
    loss, grads = _device(sess, cfg, arrays)
    loss_or, grads_or = _oracle(cfg, P, arrays)
    assert abs(loss - loss_or) <= 2e-5 * max(1.0, abs(loss_or))
    from tests.util import session_batch
    assert abs(loss - sess.loss(session_batch(sess, cfg, arrays))) <= 1e-6 * max(1.0, abs(loss_or))   # the client's own forward
    # the key bias has an identically zero gradient (softmax does not see it): what the device returns there is the
    # rounding of sums that cancel, bounded against the largest gradient entry of the model instead of its own
    floor = 1e-6 * max(np.abs(g).max() for g in grads_or.values())
    for i, s in enumerate(specs):
        want = grads_or[s.name]
        assert grads[i].shape == want.shape, s.name
        scale = np.abs(want).max()
        err = np.abs(grads[i] - want).max()
        assert err <= 2e-4 * scale + floor, (s.name, err, scale)
        assert np.array_equal(sess.get_theta(i), theta_before[i]), s.name          # parameters untouched
    # something flows everywhere except into the key bias (softmax is invariant to it)
    assert all(np.abs(grads[i]).max() > 0 for i, s in enumerate(specs) if s.role != I.ROLE_BK)


@pytest.mark.parametrize("batch,seq,act,post_ln", [(4, 48, "gelu", False), (3, 37, "gelu", False), (4, 48, "relu", True)])
def test_bf16_gradients_point_where_the_oracle_gradients_point(batch, seq, act, post_ln, say):
    """192 tokens: the backward products run on the matrix cores; 111 tokens (not a multiple of 64): on the fp32 kernel."""
    cfg = I.shrink(I.CONFIGS["cfg3"], name="bw_bf16", n_layer=2, d_model=128, n_head=2, d_ff=256, vocab=389, max_pos=64, batch=batch, seq=seq, k=8, k_full=8,
                   act=act, post_ln=post_ln)
    sess, specs, P = _setup(cfg, scale=3.0)
    arrays = _batch(cfg, 2)
    say("cloud backward bf16 decoder")
    loss, grads = _device(sess, cfg, arrays)
    loss_or, grads_or = _oracle(cfg, P, arrays)
    assert abs(loss - loss_or) <= 2e-2 * max(1.0, abs(loss_or))
    for i, s in enumerate(specs):
        want = grads_or[s.name]
        if min(want.shape) == 1 and s.role == I.ROLE_BK:
            continue
        cos = float((grads[i] * want).sum() / (np.linalg.norm(grads[i]) * np.linalg.norm(want)))
        ratio = float(np.linalg.norm(grads[i]) / np.linalg.norm(want))
        assert cos >= 0.995 and abs(ratio - 1.0) <= 0.05, (s.name, cos, ratio)


@pytest.mark.timeout(900)
@pytest.mark.parametrize("name,batch", [("cfg3", 2), ("cfg5", 1)])
def test_bf16_gradients_at_the_size_of_a_real_model(name, batch, say):
    """cfg3 (12 blocks of d = 768) on two of its sequences and cfg5 (24 blocks of d = 2048, the benchmark's model) on one,
    both with the 50272-word vocabulary: every tensor's gradient against the oracle's.  The blocks' bf16-rounded
    activations leave a few per cent: direction and norm are what is asked."""
    cfg = I.shrink(I.CONFIGS[name], name="bw_" + name, batch=batch)
    sess, specs, P = _setup(cfg, scale=1.0)
    arrays = _batch(cfg, 0)
    say(f"cloud backward at {name}, {batch} sequence(s): device")
    loss, grads = _device(sess, cfg, arrays)
    say(f"cloud backward at {name}, {batch} sequence(s): oracle")
    loss_or, grads_or = _oracle(cfg, P, arrays)
    assert abs(loss - loss_or) <= 1e-2 * abs(loss_or)
    worst = (1.0, None)
    for i, s in enumerate(specs):
        want = grads_or[s.name]
        if s.role == I.ROLE_BK:
            continue
        cos = float((grads[i] * want).sum() / (np.linalg.norm(grads[i]) * np.linalg.norm(want)))
        ratio = float(np.linalg.norm(grads[i]) / np.linalg.norm(want))
        worst = min(worst, (cos, s.name))
        assert cos >= 0.99 and abs(ratio - 1.0) <= 0.05, (s.name, cos, ratio)
    say(f"worst cosine {worst[0]:.5f} at {worst[1]}")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_two_runs_agree_bit_for_bit(dtype):
    """No sum of the backward pass depends on scheduling: the same call twice gives the same bits."""
    from tests.util import session_batch
    cfg = I.shrink(I.CONFIGS["cfg3"], name="bw_det", dtype=dtype, n_layer=2, d_model=128, n_head=2, d_ff=256, vocab=389, max_pos=64, batch=4, seq=64, k=8, k_full=8)
    sess, specs, P = _setup(cfg, scale=3.0)
    batch = session_batch(sess, cfg, _batch(cfg, 5))
    l1, g1 = sess.cloud_backward(batch)
    l2, g2 = sess.cloud_backward(batch)
    assert l1 == l2
    for a, b, s_ in zip(g1, g2, specs):
        assert bool((a == b).all()), s_.name


def test_lsq_gradient_through_the_same_entry_point():
    cfg = I.CONFIGS["cfg1"]
    sess, specs, P = _setup(cfg, scale=1.0)
    arrays = _batch(cfg, 0)
    loss, grads = _device(sess, cfg, arrays)
    want = C.lsq_gradient(P[specs[0].name], arrays["x"], arrays["y"])
    assert np.abs(grads[0] - want).max() <= 1e-5 * np.abs(want).max()
    from tests.util import oracle_loss_fn
    assert abs(loss - oracle_loss_fn(cfg, arrays)({"W": P[specs[0].name]})) <= 1e-5 * abs(loss)


def test_descent_along_the_device_gradient_lowers_the_loss():
    """What a gradient is for: theta - lr dL/dtheta has a lower loss, by about lr |dL/dtheta|^2 for a small step."""
    from tests.util import oracle_loss_fn
    cfg = I.shrink(I.CONFIGS["cfg2"], **TINY_LM)
    sess, specs, P = _setup(cfg)
    arrays = _batch(cfg, 3)
    loss, grads = _device(sess, cfg, arrays)
    g2 = sum(float((g * g).sum()) for g in grads)
    lr = 1e-3 / np.sqrt(g2)
    loss_fn = oracle_loss_fn(cfg, arrays)
    stepped = {s.name: P[s.name] - lr * grads[i] for i, s in enumerate(specs)}
    drop = loss_fn(P) - loss_fn(stepped)
    assert abs(drop - lr * g2) <= 0.05 * lr * g2, (drop, lr * g2)


def test_gradient_agrees_with_the_clients_own_directional_estimate(say):
    """At a size the oracle does not reach: along the client's perturbation Z of a step, the two-point estimate of
    Eq. (11), (L(W + h Z) - L(W - h Z)) / 2h from the client's forward, is the directional derivative <dL/dW, Z> up
    to O(h^2); Z itself is read back as (W + h Z - W) / h."""
    from tests.util import session_batch
    cfg = I.shrink(I.CONFIGS["cfg2"], name="bw_mid", n_layer=4, d_model=256, n_head=4, d_ff=1024, vocab=4096, max_pos=128, batch=4, seq=128, k=8, k_full=8)
    sess, specs, P = _setup(cfg, scale=2.0)
    batch = session_batch(sess, cfg, _batch(cfg, 4))
    say("cloud backward, 4 blocks of d = 256")
    loss, grads = sess.cloud_backward(batch)
    h, step = 2e-3, 7
    before = [sess.get_theta(i).astype(np.float64) for i in range(len(specs))]
    sess.perturb(step, h)
    lp = sess.loss(batch)
    dot = sum(float((g.cpu().numpy().astype(np.float64) * ((sess.get_theta(i).astype(np.float64) - before[i]) / h)).sum()) for i, g in enumerate(grads))
    sess.perturb(step, -2.0 * h)
    lm = sess.loss(batch)
    sess.perturb(step, h)
    est = (lp - lm) / (2.0 * h)
    assert abs(loss - 0.5 * (lp + lm)) <= 1e-3 * loss
    assert abs(est - dot) <= 2e-2 * abs(dot) + 1e-3, (est, dot)


def test_basis_from_device_gradients_captures_what_the_oracle_basis_captures():
    """The cloud block end to end on the device: three backward passes give the snapshots of a matrix, zgr_cloud_basis
    their basis; it must capture as much of the ORACLE's gradients as the oracle's own basis does."""
    from paper_2601_12917_amd.session import cloud_basis
    cfg = I.shrink(I.CONFIGS["cfg2"], **TINY_LM)
    sess, specs, P = _setup(cfg, scale=8.0)
    dev, ora = [], []
    for b in range(3):
        arrays = _batch(cfg, 10 + b)
        dev.append(_device(sess, cfg, arrays)[1])
        ora.append(_oracle(cfg, P, arrays)[1])
    k = cfg.k
    for name in ("l0.wq", "l1.w1", "l1.w2", "l0.wo"):
        i = [s.name for s in specs].index(name)
        snaps_dev = [g[i].astype(np.float32) for g in dev]
        snaps_or = [g[name] for g in ora]
        omega = np.random.default_rng(5).standard_normal((snaps_dev[0].shape[1], k)).astype(np.float32)
        U, dep = cloud_basis(snaps_dev, k, omega, 40)
        assert dep == 0
        U0, _ = C.gradient_basis(snaps_or, k)
        assert C.captured_energy(U[:, :k], snaps_or) >= C.captured_energy(U0, snaps_or) * (1.0 - 1e-3), name


def test_argument_errors_are_reported_not_executed():
    import ctypes as Ct
    from paper_2601_12917_amd import binding as B
    from tests.util import session_batch
    cfg = I.shrink(I.CONFIGS["cfg2"], **TINY_LM)
    sess, specs, P = _setup(cfg)
    lib = sess.lib
    batch = session_batch(sess, cfg, _batch(cfg, 0))
    need = lib.zgr_cloud_backward_workspace(sess.ctx, cfg.batch, cfg.seq)
    assert need > 0 and lib.zgr_cloud_backward_workspace(sess.ctx, 0, cfg.seq) == 0
    import torch
    ws = torch.empty(need, dtype=torch.uint8, device="cuda:0")
    grads = [torch.empty(*v.shape, dtype=torch.float32, device="cuda:0") for v in P.values()]
    ptrs = (Ct.c_void_p * len(grads))(*[g.data_ptr() for g in grads])
    v = Ct.c_double()
    assert lib.zgr_cloud_backward(sess.ctx, Ct.byref(batch), ptrs, len(grads) - 1, Ct.byref(v), ws.data_ptr(), need) == B.ZGR_ERR_SHAPE
    assert lib.zgr_cloud_backward(sess.ctx, Ct.byref(batch), ptrs, len(grads), Ct.byref(v), ws.data_ptr(), need - 256) == B.ZGR_ERR_WORKSPACE
    assert lib.zgr_cloud_backward(sess.ctx, Ct.byref(batch), ptrs, len(grads), Ct.byref(v), ws.data_ptr() + 64, need) == B.ZGR_ERR_WORKSPACE
    ptrs[3] = None
    assert lib.zgr_cloud_backward(sess.ctx, Ct.byref(batch), ptrs, len(grads), Ct.byref(v), ws.data_ptr(), need) == B.ZGR_ERR_NULL
