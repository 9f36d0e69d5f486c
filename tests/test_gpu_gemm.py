"""The bf16 projection kernels against the oracle's definition of a linear layer, out = act(A W^T + b), in fp64.
Shapes are chosen to reach every block-tile variant and main loop of the launcher (256 x 256 and 128 x 256 with the
ping-pong pipeline, 256 x 192 with one wave per SIMD, 128 x 128 with the ping-pong loop on a long and on a short ring, 64 x 64 with the plain loop), with ragged last tiles in M and in N, a single k-tile,
an odd number of k-tiles, and the depth of the real layers (K = 2048).  Inputs are bf16-representable, so the only
differences are fp32 accumulation order and the bf16 rounding of stored results."""
import numpy as np
import pytest

from oracle import forward as F

pytestmark = pytest.mark.gpu

EPI_STORE, EPI_GELU, EPI_RESID, EPI_F32 = 0, 1, 2, 3

#         M     N     K   what it reaches
SHAPES = [
    (4096, 4160, 64, "256x256 tiles, ragged N, one k-tile"),
    (4000, 4352, 192, "256x256 tiles, ragged M, three k-tiles"),
    (4096, 6144, 128, "256x192 tiles, two k-tiles"),
    (4000, 6144, 320, "256x192 tiles, ragged M, five k-tiles"),
    (4096, 6144, 2048, "256x192 tiles at the QKV shape"),
    (3300, 2048, 320, "128x256 tiles, ragged M, five k-tiles"),
    (4096, 2000, 2048, "128x256 tiles, ragged N, full depth"),
    (1000, 600, 128, "64x64 tiles, plain loop, ragged both"),
    (1990, 1500, 192, "128x128 tiles, ping-pong loop on the long ring (at most one tile per CU), ragged both"),
    (2048, 1536, 1024, "128x128 tiles, ping-pong loop on the long ring, 16 k-tiles"),
    (2000, 2200, 320, "128x128 tiles, ping-pong loop on the short ring (more tiles than CUs), ragged both, five k-tiles"),
    (2048, 2304, 768, "128x128 tiles, ping-pong loop, the QKV shape of the 125M model"),
    (4096, 8192, 2048, "256x256 tiles at the FC1 shape"),
]


def _bf16_round(x):
    import torch
    return torch.from_numpy(x.astype(np.float32)).bfloat16()


@pytest.mark.parametrize("M,N,K,what", SHAPES)
@pytest.mark.parametrize("epi", [EPI_STORE, EPI_GELU, EPI_RESID, EPI_F32])
def test_gemm_matches_linear_layer(M, N, K, what, epi):
    import torch
    from paper_2601_12917_amd import binding as B
    lib = B.lib()
    dev = "cuda:0"
    rng = np.random.default_rng(1000 * epi + M + N + K)
    A = _bf16_round(rng.standard_normal((M, K)) * 0.5)
    W = _bf16_round(rng.standard_normal((N, K)) * 0.05)
    bias = _bf16_round(rng.standard_normal(N) * 0.1)
    res = (rng.standard_normal((M, N)) * 0.3).astype(np.float32) if epi == EPI_RESID else None
    Ad, Wd, bd = A.to(dev), W.to(dev), bias.to(dev)
    if epi in (EPI_STORE, EPI_GELU):
        out = torch.zeros(M, N, device=dev, dtype=torch.bfloat16)
    elif epi == EPI_RESID:
        out = torch.from_numpy(res).to(dev)
    else:
        out = torch.full((M, N), 7.0, device=dev, dtype=torch.float32)
    st = torch.cuda.current_stream().cuda_stream
    B.check(lib.zgr_debug_gemm(1, Ad.data_ptr(), Wd.data_ptr(), bd.data_ptr(), out.data_ptr(), epi, M, N, K, st))
    torch.cuda.synchronize()
    got = out.float().cpu().numpy().astype(np.float64)
    # the oracle checks sampled rows in full (all columns, so every column tile and the ragged tail), plus the
    # first and last rows of every row tile boundary
    rows = np.unique(np.concatenate([rng.integers(0, M, 48), [0, 1, 127, 128, 255, 256, M - 257, M - 256, M - 129, M - 128, M - 2, M - 1]]))
    rows = rows[(rows >= 0) & (rows < M)]
    A64 = A.float().numpy().astype(np.float64)[rows]
    W64 = W.float().numpy().astype(np.float64)
    want = A64 @ W64.T + bias.float().numpy().astype(np.float64)
    if epi == EPI_GELU:
        want = F.gelu(want)
    if epi == EPI_RESID:
        want = want + res[rows].astype(np.float64)
    g = got[rows]
    # fp32 accumulation of K products of magnitude ~ |a||w|: error ~ sqrt(K) * 2^-24 * sum|a w|, far below the
    # tolerances here; stored bf16 results carry half an ulp (2^-9 relative)
    scale = np.abs(A64) @ np.abs(W64).T + 0.1
    if epi in (EPI_STORE, EPI_GELU):
        tol = 2.0 ** -8 * np.abs(want) + 1e-5 * scale
    else:
        tol = 2e-6 * scale + 1e-6 * np.abs(want)
    bad = np.abs(g - want) > tol
    assert not bad.any(), (what, int(bad.sum()), float(np.abs(g - want).max()))


#            M     N     K   what it reaches
F32_SHAPES = [
    (2048, 2100, 72, "128x128 matrix-core tiles, ragged N, a k-tile of 8 at the end"),
    (2000, 2304, 768, "128x128 matrix-core tiles, ragged M, the depth of a real layer"),
    (300, 200, 40, "64x64 matrix-core tiles, ragged both, k-tail"),
    (64, 64, 4, "one tile, a single quarter-filled k-tile"),
    (130, 70, 37, "K no multiple of 4: the vector-ALU kernel"),
]


@pytest.mark.parametrize("M,N,K,what", F32_SHAPES)
@pytest.mark.parametrize("epi", [EPI_STORE, EPI_GELU, EPI_RESID, EPI_F32])
def test_fp32_gemm_matches_linear_layer(M, N, K, what, epi):
    """The fp32 projection kernels (v_mfma_f32_32x32x2_f32 tiles, and the plain kernel for what they do not take)
    against out = act(A W^T + b) in fp64, every output entry."""
    import torch
    from paper_2601_12917_amd import binding as B
    lib = B.lib()
    dev = "cuda:0"
    rng = np.random.default_rng(5000 + 1000 * epi + M + N + K)
    A = (rng.standard_normal((M, K)) * 0.5).astype(np.float32)
    W = (rng.standard_normal((N, K)) * 0.05).astype(np.float32)
    bias = (rng.standard_normal(N) * 0.1).astype(np.float32)
    res = (rng.standard_normal((M, N)) * 0.3).astype(np.float32)
    Ad, Wd, bd = torch.from_numpy(A).to(dev), torch.from_numpy(W).to(dev), torch.from_numpy(bias).to(dev)
    out = torch.from_numpy(res).to(dev) if epi == EPI_RESID else torch.full((M, N), 7.0, device=dev, dtype=torch.float32)
    st = torch.cuda.current_stream().cuda_stream
    B.check(lib.zgr_debug_gemm(0, Ad.data_ptr(), Wd.data_ptr(), bd.data_ptr(), out.data_ptr(), epi, M, N, K, st))
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    A64, W64 = A.astype(np.float64), W.astype(np.float64)
    want = A64 @ W64.T + bias.astype(np.float64)
    if epi == EPI_GELU:
        want = F.gelu(want)
    if epi == EPI_RESID:
        want = want + res.astype(np.float64)
    # fp32 products and sums of K terms: a few 2^-24 of sum |a w|; the result's own rounding: 2^-24 |want|
    scale = np.abs(A64) @ np.abs(W64).T + 0.1
    tol = 2e-6 * scale + 2e-7 * np.abs(want)
    bad = np.abs(got - want) > tol
    assert not bad.any(), (what, int(bad.sum()), float(np.abs(got - want).max()))
