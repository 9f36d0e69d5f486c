"""zgr_lsq_loss_static (the entry point that allocates nothing: its scratch is a static device array of the
library) against zgr_loss of the least-squares model (scratch in the caller's workspace): same kernels, so the
same double, on two calls in a row, the second on a smaller problem, which must not read what the first left."""
import ctypes as C

import numpy as np
import pytest

import zgr_inputs as I
from tests.util import inputs_of, make_batch_arrays, make_session, session_batch

pytestmark = pytest.mark.gpu


def _both(cfg):
    import torch
    specs, values, bases = inputs_of(cfg)
    arrays = make_batch_arrays(cfg)
    sess = make_session(cfg, specs, values, bases)
    batch = session_batch(sess, cfg, arrays)
    want = sess.loss(batch)
    out = torch.full((1,), -1.0, dtype=torch.float64, device=sess.dev)
    st = sess.lib.zgr_lsq_loss_static(sess.theta[0].data_ptr(), batch.x, batch.y, cfg.batch, cfg.lsq_out, cfg.lsq_in,
                                      out.data_ptr(), sess.stream.cuda_stream)
    assert st == 0, sess.lib.zgr_last_error(None)
    torch.cuda.synchronize()
    got = float(out.cpu()[0])
    sess.close()
    return got, want, (values[0], arrays)


def test_static_scratch_loss_equals_workspace_loss_twice_second_smaller():
    from oracle import forward as F
    big = I.shrink(I.CONFIGS["cfg1"], name="lsq_big", lsq_out=300, lsq_in=520, batch=45)
    small = I.shrink(I.CONFIGS["cfg1"], name="lsq_small", lsq_out=37, lsq_in=64, batch=5)
    for cfg in (big, small, big):
        got, want, (W, arrays) = _both(cfg)
        assert got == want, (cfg.name, got, want)                      # bit-identical: the same three kernels
        ref = F.lsq_loss(W, arrays["x"], arrays["y"])
        assert abs(got - ref) <= 1e-4 * abs(ref), (cfg.name, got, ref)  # and the oracle's loss within the fp32 tolerance


def test_static_scratch_rejects_sizes_beyond_its_array():
    import torch
    from paper_2601_12917_amd import binding as B
    lib = B.lib()
    d = torch.zeros(16, dtype=torch.float32, device="cuda:0")
    out = torch.zeros(1, dtype=torch.float64, device="cuda:0")
    st = torch.cuda.current_stream().cuda_stream
    assert lib.zgr_lsq_loss_static(d.data_ptr(), d.data_ptr(), d.data_ptr(), 4097, 1, 1, out.data_ptr(), st) == B.ZGR_ERR_WORKSPACE
    assert b"static scratch" in lib.zgr_last_error(None)
    assert lib.zgr_lsq_loss_static(d.data_ptr(), d.data_ptr(), d.data_ptr(), 1024, 257, 1, out.data_ptr(), st) == B.ZGR_ERR_WORKSPACE
    assert lib.zgr_lsq_loss_static(None, d.data_ptr(), d.data_ptr(), 1, 1, 1, out.data_ptr(), st) == B.ZGR_ERR_NULL
    assert lib.zgr_lsq_loss_static(d.data_ptr(), d.data_ptr(), d.data_ptr(), 0, 1, 1, out.data_ptr(), st) == B.ZGR_ERR_SHAPE
    torch.cuda.synchronize()
    assert float(out.cpu()[0]) == 0.0                                   # nothing was launched
