"""Seeded synthetic inputs for the ZGR client step.

This module only *makes data*: model shapes, random-init weights, token ids,
padding lengths, labels and orthonormal bases.  It contains none of the
method's arithmetic (no Philox, no Box-Muller, no perturbation, no loss) and
is the only code that the CPU oracle's tests and the GPU path's tests both
call.  All randomness comes from numpy's PCG64 generator under fixed seeds,
one child stream per array, so every array is reproducible from
(config name, data seed, array name) alone.

The paper evaluates on SST-2, AGNews, 20News and LongAlign with pretrained
checkpoints (Sec. 4, "Models and Datasets"); those are not available, so the
workloads here are stand-ins of the same shape: random-init weights,
uniform or Zipf(1.1) token ids (the rank-frequency law of natural text) and,
for the classifier, padding lengths uniform in [32, 256].
"""
from __future__ import annotations

import dataclasses
import zlib
from typing import Dict, List, Optional

import numpy as np

# ----------------------------------------------------------------------------
# Roles of parameter tensors (values are part of the C ABI: zgr_role in zgr.h)
# ----------------------------------------------------------------------------
ROLE_LSQ_W = 0
ROLE_TOK_EMB = 1
ROLE_POS_EMB = 2
ROLE_LN1_G = 3
ROLE_LN1_B = 4
ROLE_WQ = 5
ROLE_BQ = 6
ROLE_WK = 7
ROLE_BK = 8
ROLE_WV = 9
ROLE_BV = 10
ROLE_WO = 11
ROLE_BO = 12
ROLE_LN2_G = 13
ROLE_LN2_B = 14
ROLE_W1 = 15
ROLE_B1 = 16
ROLE_W2 = 17
ROLE_B2 = 18
ROLE_LNF_G = 19
ROLE_LNF_B = 20
ROLE_CLS_W = 21
ROLE_CLS_B = 22

ARCH_LINEAR_LSQ = 0
ARCH_DECODER_LM = 1
ARCH_ENCODER_CLS = 2

GUIDED_ROLES = (ROLE_LSQ_W, ROLE_WQ, ROLE_WK, ROLE_WV, ROLE_WO, ROLE_W1, ROLE_W2, ROLE_CLS_W)


@dataclasses.dataclass(frozen=True)
class Config:
    """One workload: model shape, batch shape and ZGR hyper-parameters."""
    name: str
    arch: int
    dtype: str                # "f32" | "bf16"  (storage type of the parameters)
    n_layer: int = 0
    d_model: int = 0
    n_head: int = 0
    d_ff: int = 0
    vocab: int = 0
    max_pos: int = 0
    n_class: int = 0
    batch: int = 0
    seq: int = 0
    # LSQ only
    lsq_out: int = 0
    lsq_in: int = 0
    # ZGR
    k: int = 0                # rank the kernel samples in (k' when truncated)
    k_full: int = 0           # columns of the basis as transmitted (ldu)
    alpha: float = 0.5
    eps: float = 1e-3
    lr: float = 1e-6
    steps: int = 1
    seed: int = 42            # Philox seed of the method
    scale_mode: int = 0       # 0: unit-variance scaling of Eq. (10); 1: Eq. (10) as printed
    tokens: str = "uniform"   # "uniform" | "zipf"
    ln_eps: float = 1e-5
    act: str = "gelu"         # feed-forward activation: "gelu" (erf form) | "relu"
    post_ln: bool = False     # LayerNorm after each residual sum (and on the embeddings) instead of before each sublayer


CONFIGS: Dict[str, Config] = {
    # Single linear layer, least-squares loss.  lr = 1e-2 is only stable with the perturbation
    # scaled as Eq. (10) prints it (||z_h||^2 ~ 1); with unit-variance scaling it diverges.
    "cfg1": Config("cfg1", ARCH_LINEAR_LSQ, "f32", lsq_out=256, lsq_in=512, batch=32,
                   k=4, k_full=4, lr=1e-2, steps=10, scale_mode=1),
    # Tiny decoder-only transformer.
    "cfg2": Config("cfg2", ARCH_DECODER_LM, "f32", n_layer=2, d_model=128, n_head=4, d_ff=512,
                   vocab=1024, max_pos=64, batch=8, seq=64, k=8, k_full=8, lr=1e-4, steps=20),
    # OPT-125m-shaped decoder.
    "cfg3": Config("cfg3", ARCH_DECODER_LM, "bf16", n_layer=12, d_model=768, n_head=12, d_ff=3072,
                   vocab=50272, max_pos=2048, batch=16, seq=128, k=16, k_full=16, lr=1e-6,
                   tokens="zipf"),
    # RoBERTa-large-shaped encoder classifier.
    "cfg4": Config("cfg4", ARCH_ENCODER_CLS, "bf16", n_layer=24, d_model=1024, n_head=16, d_ff=4096,
                   vocab=50265, max_pos=512, n_class=2, batch=16, seq=256, k=32, k_full=32, lr=1e-6,
                   tokens="zipf"),
    # OPT-1.3B-shaped decoder; basis sent with 64 columns, first 16 kept.
    "cfg5": Config("cfg5", ARCH_DECODER_LM, "bf16", n_layer=24, d_model=2048, n_head=32, d_ff=8192,
                   vocab=50272, max_pos=2048, batch=16, seq=256, k=16, k_full=64, lr=1e-6,
                   tokens="zipf"),
}


def shrink(cfg: Config, **kw) -> Config:
    """A copy of cfg with some fields replaced (used for small test shapes)."""
    return dataclasses.replace(cfg, **kw)


@dataclasses.dataclass
class TensorSpec:
    name: str
    role: int
    layer: int
    rows: int
    cols: int
    tensor_id: int
    guided: bool

    @property
    def numel(self) -> int:
        return self.rows * self.cols


def tensor_specs(cfg: Config) -> List[TensorSpec]:
    """Parameter tensors of the model, in storage order.  2-D tensors are
    [out, in] row-major; 1-D tensors have rows = 1.  Wq, Wk, Wv (and their
    biases) are adjacent so that an implementation may treat them as one
    [3d, d] matrix."""
    specs: List[TensorSpec] = []

    def add(name, role, layer, rows, cols):
        guided = role in GUIDED_ROLES and cfg.k > 0 and rows >= cfg.k
        specs.append(TensorSpec(name, role, layer, rows, cols, len(specs), guided))

    if cfg.arch == ARCH_LINEAR_LSQ:
        add("W", ROLE_LSQ_W, -1, cfg.lsq_out, cfg.lsq_in)
        return specs
    d, ff = cfg.d_model, cfg.d_ff
    add("tok_emb", ROLE_TOK_EMB, -1, cfg.vocab, d)
    add("pos_emb", ROLE_POS_EMB, -1, cfg.max_pos, d)
    for l in range(cfg.n_layer):
        add(f"l{l}.ln1_g", ROLE_LN1_G, l, 1, d)
        add(f"l{l}.ln1_b", ROLE_LN1_B, l, 1, d)
        add(f"l{l}.wq", ROLE_WQ, l, d, d)
        add(f"l{l}.wk", ROLE_WK, l, d, d)
        add(f"l{l}.wv", ROLE_WV, l, d, d)
        add(f"l{l}.bq", ROLE_BQ, l, 1, d)
        add(f"l{l}.bk", ROLE_BK, l, 1, d)
        add(f"l{l}.bv", ROLE_BV, l, 1, d)
        add(f"l{l}.wo", ROLE_WO, l, d, d)
        add(f"l{l}.bo", ROLE_BO, l, 1, d)
        add(f"l{l}.ln2_g", ROLE_LN2_G, l, 1, d)
        add(f"l{l}.ln2_b", ROLE_LN2_B, l, 1, d)
        add(f"l{l}.w1", ROLE_W1, l, ff, d)
        add(f"l{l}.b1", ROLE_B1, l, 1, ff)
        add(f"l{l}.w2", ROLE_W2, l, d, ff)
        add(f"l{l}.b2", ROLE_B2, l, 1, d)
    add("lnf_g", ROLE_LNF_G, -1, 1, d)
    add("lnf_b", ROLE_LNF_B, -1, 1, d)
    if cfg.arch == ARCH_ENCODER_CLS:
        add("cls_w", ROLE_CLS_W, -1, cfg.n_class, d)
        add("cls_b", ROLE_CLS_B, -1, 1, cfg.n_class)
    return specs


def _rng(cfg_name: str, data_seed: int, array_name: str) -> np.random.Generator:
    tag = zlib.crc32(f"{cfg_name}/{array_name}".encode())
    return np.random.default_rng([data_seed, tag])


def _clear_low_mantissa(x: np.ndarray) -> np.ndarray:
    """Zero the low 16 bits of each fp32 so the value is exactly a bf16 value
    (a property of the generated data, not a rounding rule of the method)."""
    b = x.view(np.uint32) & np.uint32(0xFFFF0000)
    return b.view(np.float32)


def make_params(cfg: Config, data_seed: int = 0, specs: Optional[List[TensorSpec]] = None
                ) -> List[np.ndarray]:
    """Random-init parameter values as fp32 arrays [rows, cols].
    Matrices, embeddings and biases ~ N(0, 0.02^2); LayerNorm gains
    1 + N(0, 0.02^2).  For bf16 configs every value is exactly
    representable in bf16."""
    specs = specs if specs is not None else tensor_specs(cfg)
    out = []
    for s in specs:
        g = _rng(cfg.name, data_seed, "param/" + s.name)
        x = g.standard_normal((s.rows, s.cols), dtype=np.float32) * np.float32(0.02)
        if s.role in (ROLE_LN1_G, ROLE_LN2_G, ROLE_LNF_G):
            x = x + np.float32(1.0)
        if cfg.dtype == "bf16":
            x = _clear_low_mantissa(np.ascontiguousarray(x))
        out.append(np.ascontiguousarray(x, dtype=np.float32))
    return out


def make_basis(cfg: Config, spec: TensorSpec, data_seed: int = 0) -> Optional[np.ndarray]:
    """Orthonormal basis U [rows, k_full] fp32 for a guided tensor: the Q
    factor of a seeded Gaussian matrix, signs fixed so that R has a positive
    diagonal.  None for tensors that are perturbed isotropically."""
    if not spec.guided:
        return None
    g = _rng(cfg.name, data_seed, "basis/" + spec.name)
    a = g.standard_normal((spec.rows, cfg.k_full))
    q, r = np.linalg.qr(a)
    q = q * np.sign(np.diag(r))[None, :]
    return np.ascontiguousarray(q, dtype=np.float32)


def zipf_cdf(vocab: int, s: float = 1.1) -> np.ndarray:
    p = np.arange(1, vocab + 1, dtype=np.float64) ** (-s)
    c = np.cumsum(p)
    return c / c[-1]


def make_tokens(cfg: Config, data_seed: int = 0) -> np.ndarray:
    """int32 token ids [batch, seq]: uniform, or bounded Zipf(1.1) by
    inverse CDF (id = rank - 1)."""
    g = _rng(cfg.name, data_seed, "tokens")
    if cfg.tokens == "uniform":
        return g.integers(0, cfg.vocab, size=(cfg.batch, cfg.seq), dtype=np.int64).astype(np.int32)
    u = g.random((cfg.batch, cfg.seq))
    ids = np.searchsorted(zipf_cdf(cfg.vocab), u, side="left")
    return np.minimum(ids, cfg.vocab - 1).astype(np.int32)


def make_lengths(cfg: Config, data_seed: int = 0, lo: int = 32) -> np.ndarray:
    """int32 valid lengths [batch], uniform in [min(lo, seq), seq]."""
    g = _rng(cfg.name, data_seed, "lengths")
    lo = min(lo, cfg.seq)
    return g.integers(lo, cfg.seq + 1, size=(cfg.batch,), dtype=np.int64).astype(np.int32)


def make_labels(cfg: Config, data_seed: int = 0) -> np.ndarray:
    g = _rng(cfg.name, data_seed, "labels")
    return g.integers(0, cfg.n_class, size=(cfg.batch,), dtype=np.int64).astype(np.int32)


def make_lsq_data(cfg: Config, data_seed: int = 0):
    """X [batch, in] ~ N(0,1), Y = X W*^T + N(0, 0.01^2) with a second seeded
    W* ~ N(0, 0.02^2); both fp32."""
    g = _rng(cfg.name, data_seed, "lsq")
    wstar = g.standard_normal((cfg.lsq_out, cfg.lsq_in)) * 0.02
    x = g.standard_normal((cfg.batch, cfg.lsq_in))
    y = x @ wstar.T + g.standard_normal((cfg.batch, cfg.lsq_out)) * 0.01
    return (np.ascontiguousarray(x, dtype=np.float32), np.ascontiguousarray(y, dtype=np.float32))
