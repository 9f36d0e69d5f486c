"""Host-side checks that need no GPU: the library loads, exports every symbol
include/zgr.h declares, and rejects bad arguments before touching the device."""
import ctypes as C
import os
import re

import pytest

from paper_2601_12917_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        from paper_2601_12917_amd.build import build
        build()
    return B.lib()


def test_every_declared_symbol_is_exported_and_bound(lib):
    header = open(os.path.join(ROOT, "include", "zgr.h")).read()
    declared = set(re.findall(r"\b(zgr_[a-z0-9_]+)\s*\(", header))
    assert declared, "no declarations found"
    for name in declared:
        assert hasattr(lib, name), name
    assert declared == set(B.SYMBOLS), declared ^ set(B.SYMBOLS)


def _tensor(rows=4, cols=8, theta=0x1000, k=0, U=None, ldu=0, tid=1, role=0, dtype=0):
    t = B.zgr_tensor()
    t.theta, t.rows, t.cols, t.dtype, t.tensor_id, t.U, t.k, t.ldu, t.role, t.layer = theta, rows, cols, dtype, tid, U, k, ldu, role, -1
    return t


def _init(lib, tensors, model=None, cfg=None, ws=0x10000, ws_bytes=1 << 30):
    ctx = C.c_void_p()
    model = model or B.zgr_model(B.ZGR_ARCH_NONE, 0, 0, 0, 0, 0, 0, 0, 1e-5)
    cfg = cfg or B.zgr_config(42, 1e-3, 0.5, 0, 32)
    arr = (B.zgr_tensor * len(tensors))(*tensors)
    st = lib.zgr_init(C.byref(ctx), C.byref(model), arr, len(tensors), C.byref(cfg), ws, ws_bytes, 1, 2, None)
    return st, lib.zgr_last_error(None).decode(), ctx


def test_init_rejects_bad_arguments_without_touching_the_device(lib):
    ctx = C.c_void_p()
    assert lib.zgr_init(C.byref(ctx), None, None, 0, None, None, 0, 0, 0, None) == B.ZGR_ERR_NULL
    assert lib.zgr_init(None, None, None, 0, None, None, 0, 0, 0, None) == B.ZGR_ERR_NULL
    st, msg, _ = _init(lib, [_tensor(theta=None)])
    assert st == B.ZGR_ERR_NULL and "theta" in msg
    st, msg, _ = _init(lib, [_tensor(theta=0x1004)])
    assert st == B.ZGR_ERR_SHAPE and "aligned" in msg
    st, msg, _ = _init(lib, [_tensor(dtype=7)])
    assert st == B.ZGR_ERR_DTYPE
    st, msg, _ = _init(lib, [_tensor(), _tensor(tid=2, dtype=1)])
    assert st == B.ZGR_ERR_DTYPE and "share" in msg
    st, msg, _ = _init(lib, [_tensor(), _tensor()])
    assert st == B.ZGR_ERR_CONFIG and "tensor_id" in msg
    st, msg, _ = _init(lib, [_tensor(tid=1 << 31)])
    assert st == B.ZGR_ERR_CONFIG
    st, msg, _ = _init(lib, [_tensor(k=5, U=0x2000, ldu=8)])            # k > rows
    assert st == B.ZGR_ERR_SHAPE and "rows" in msg
    st, msg, _ = _init(lib, [_tensor(rows=16, k=4, U=0x2000, ldu=2)])   # ldu < k
    assert st == B.ZGR_ERR_SHAPE and "ldu" in msg
    st, msg, _ = _init(lib, [_tensor(rows=16, cols=6, k=4, U=0x2000, ldu=4)])
    assert st == B.ZGR_ERR_SHAPE and "cols" in msg
    st, msg, _ = _init(lib, [_tensor(rows=128, cols=8, k=65, U=0x2000, ldu=65)])
    assert st == B.ZGR_ERR_SHAPE and "exceeds" in msg
    for cfg in (B.zgr_config(1, 0.0, 0.5, 0, 32), B.zgr_config(1, 1e-3, 1.5, 0, 32), B.zgr_config(1, 1e-3, 0.5, 3, 32),
                B.zgr_config(1, 1e-3, 0.5, 0, 24), B.zgr_config(1, float("nan"), 0.5, 0, 32)):
        st, msg, _ = _init(lib, [_tensor()], cfg=cfg)
        assert st == B.ZGR_ERR_CONFIG, msg
    st, msg, _ = _init(lib, [_tensor()], ws=None)
    assert st == B.ZGR_ERR_NULL and "workspace" in msg
    st, msg, _ = _init(lib, [_tensor()], ws=0x10010)
    assert st == B.ZGR_ERR_WORKSPACE and "aligned" in msg
    st, msg, _ = _init(lib, [_tensor()], ws_bytes=16)
    assert st == B.ZGR_ERR_WORKSPACE and "needed" in msg
    # model / table mismatches
    lm = B.zgr_model(B.ZGR_ARCH_DECODER_LM, 1, 16, 2, 32, 50, 8, 0, 1e-5)
    st, msg, _ = _init(lib, [_tensor()], model=lm)
    assert st == B.ZGR_ERR_SHAPE
    bad_head = B.zgr_model(B.ZGR_ARCH_DECODER_LM, 1, 24, 2, 32, 50, 8, 0, 1e-5)
    st, msg, _ = _init(lib, [_tensor()], model=bad_head)
    assert st == B.ZGR_ERR_SHAPE and "head" in msg
    lsq_bf16 = B.zgr_model(B.ZGR_ARCH_LINEAR_LSQ, 0, 0, 0, 0, 0, 0, 0, 1e-5)
    st, msg, _ = _init(lib, [_tensor(dtype=1)], model=lsq_bf16)
    assert st == B.ZGR_ERR_DTYPE
    # the model-family switches: activation in {GELU, ReLU}, post_ln in {0, 1}
    st, msg, _ = _init(lib, [_tensor()], model=B.zgr_model(B.ZGR_ARCH_DECODER_LM, 1, 16, 2, 32, 50, 8, 0, 1e-5, 7, 0))
    assert st == B.ZGR_ERR_CONFIG and "activation" in msg
    st, msg, _ = _init(lib, [_tensor()], model=B.zgr_model(B.ZGR_ARCH_DECODER_LM, 1, 16, 2, 32, 50, 8, 0, 1e-5, B.ZGR_ACT_RELU, 2))
    assert st == B.ZGR_ERR_CONFIG and "post_ln" in msg


def test_workspace_bytes_and_null_context_calls(lib):
    model = B.zgr_model(B.ZGR_ARCH_DECODER_LM, 2, 128, 4, 512, 1024, 64, 0, 1e-5)
    t = (B.zgr_tensor * 1)(_tensor(rows=1024, cols=128))
    n = lib.zgr_workspace_bytes(C.byref(model), t, 1, 8, 64)
    assert n > 8 * 64 * 1024 * 4 and n % 256 == 0
    assert lib.zgr_workspace_bytes(None, t, 1, 8, 64) == 0
    assert lib.zgr_workspace_bytes(C.byref(model), t, 1, 16, 64) > n
    assert lib.zgr_step(None, 0, None, None) == B.ZGR_ERR_NULL
    assert lib.zgr_apply_update(None, 0, 0.0, 0.0) == B.ZGR_ERR_NULL
    assert lib.zgr_perturb(None, 0, 0.0) == B.ZGR_ERR_NULL
    assert lib.zgr_set_basis(None, 0, None, 0, 0) == B.ZGR_ERR_NULL
    assert lib.zgr_profile_enable(None, 1) == B.ZGR_ERR_NULL
    assert lib.zgr_debug_gauss(1, 0, 1, 0, 24, 0, 4, 0x1000, None) == B.ZGR_ERR_CONFIG
    assert lib.zgr_debug_gauss(1, 0, 1, 0, 32, 0, 4, None, None) == B.ZGR_ERR_NULL
    lib.zgr_destroy(None)


def test_compression_share_matches_the_oracle(lib):
    """zgr_dtc_omega / zgr_dtc_memory_factor are host arithmetic: checked here against the oracle's search."""
    import numpy as np
    from oracle import dtc as D
    rng = np.random.default_rng(5)
    seen = set()
    for _ in range(300):
        D0 = 10 ** rng.uniform(4, 9)
        B0 = 10 ** rng.uniform(5, 11)
        Tcc = 10 ** rng.uniform(-5, -1)
        tau = 0.0 if rng.random() < 0.5 else 10 ** rng.uniform(-13, -9)
        theta = rng.uniform(0.05, 0.9)
        w, ok = B.dtc_omega(D0, B0, Tcc, tau, theta)
        w_o, ok_o = D.choose_omega(D0, B0, Tcc, tau, theta)
        assert ok == ok_o and abs(w - w_o) <= 1e-9, (D0, B0, Tcc, tau, theta, w, w_o)
        seen.add((w == 0.0, w == 1.0, ok))
        L = int(rng.integers(1, 97))
        assert B.dtc_memory_factor(L, w, theta) == pytest.approx(D.memory_factor(L, w, theta), rel=1e-14)
    assert len(seen) == 3                      # already hidden, partly compressed, not reachable: all three occurred
    for bad in [(0, 1e9, 1e-3, 0, 0.125), (1e6, 0, 1e-3, 0, 0.125), (1e6, 1e9, -1, 0, 0.125), (1e6, 1e9, 1e-3, 0, 1.0), (1e6, 1e9, 1e-3, 0, 0.0)]:
        with pytest.raises(B.ZgrError):
            B.dtc_omega(*bad)
    with pytest.raises(B.ZgrError):
        B.dtc_memory_factor(0, 0.5, 0.125)



def test_cloud_entry_points_validate_their_arguments_without_a_gpu():
    import ctypes as C
    from paper_2601_12917_amd import binding as B
    lib = B.lib()
    assert lib.zgr_cloud_basis_workspace(256, 512, 4) >= (2 * 256 * 4 + 512 * 4) * 4
    assert lib.zgr_cloud_basis_workspace(256, 512, 65) == 0 and lib.zgr_cloud_basis_workspace(0, 512, 4) == 0
    one = (C.c_void_p * 1)(0x1000)
    dep = C.c_int32(0)
    # NULL pieces, rank above the rows / above 64, row stride below the rank, workspace too small or misaligned
    assert lib.zgr_cloud_basis(None, 1, 8, 8, 2, 0x1000, 1, 0x1000, 2, C.byref(dep), 0x1000, 1 << 20, None) == B.ZGR_ERR_NULL
    assert lib.zgr_cloud_basis((C.c_void_p * 1)(None), 1, 8, 8, 2, 0x1000, 1, 0x1000, 2, C.byref(dep), 0x1000, 1 << 20, None) == B.ZGR_ERR_NULL
    assert lib.zgr_cloud_basis(one, 1, 8, 8, 9, 0x1000, 1, 0x1000, 9, C.byref(dep), 0x1000, 1 << 20, None) == B.ZGR_ERR_SHAPE
    assert lib.zgr_cloud_basis(one, 1, 100, 8, 65, 0x1000, 1, 0x1000, 65, C.byref(dep), 0x1000, 1 << 20, None) == B.ZGR_ERR_SHAPE
    assert lib.zgr_cloud_basis(one, 1, 8, 8, 4, 0x1000, 1, 0x1000, 3, C.byref(dep), 0x1000, 1 << 20, None) == B.ZGR_ERR_SHAPE
    assert lib.zgr_cloud_basis(one, 1, 8, 8, 4, 0x1000, 1, 0x1000, 4, C.byref(dep), 0x1000, 16, None) == B.ZGR_ERR_WORKSPACE
    assert lib.zgr_cloud_basis(one, 1, 8, 8, 4, 0x1000, 1, 0x1000, 4, C.byref(dep), 0x1010, 1 << 20, None) == B.ZGR_ERR_WORKSPACE
    assert lib.zgr_cloud_lsq_gradient(None, 0x1000, 0x1000, 1, 1, 1, 0x1000, 0x1000, 64, None) == B.ZGR_ERR_NULL
    assert lib.zgr_cloud_lsq_gradient(0x1000, 0x1000, 0x1000, 4, 4, 4, 0x1000, 0x1000, 8, None) == B.ZGR_ERR_WORKSPACE
    # the backward pass needs a context: without one it reports that and sizes nothing
    assert lib.zgr_cloud_backward_workspace(None, 4, 16) == 0
    v = C.c_double()
    assert lib.zgr_cloud_backward(None, None, None, 0, C.byref(v), None, 0) == B.ZGR_ERR_NULL


def test_bench_refuses_more_than_one_gpu():
    """One GPU is all the library runs on: the benchmark says so instead of starting ranks."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout.strip() == ""
