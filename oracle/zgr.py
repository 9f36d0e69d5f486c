"""TEST INFRASTRUCTURE ONLY: CPU oracle, never imported by the product path.

One client-side ZGR step and the edge server's update, in the order of
Algorithm 1 (client block, edge-server block) with the estimator of Eq. (11):

    Delta = L(W + eps z_h; x) - L(W - eps z_h; x)          (client, sends the scalar)
    g_hat = Delta / (2 eps) * z_h,  z_h regenerated from the seed   (edge server)
    W <- W - eta g_hat

The parameters are perturbed in place and restored, as the workflow of
Sec. 3.1 (step 5) describes, in three passes W += eps Z, W -= 2 eps Z,
W += eps Z, each pass regenerating Z from (seed, step).  Storage types:
'f32' (one fp32 fused multiply-add per element and pass) or 'bf16' (the same,
followed by round-to-nearest-even; no fp32 master copy, since the method's
memory claim rests on holding only the model itself, Sec. 3.3).
"""
import numpy as np

from . import forward as F
from .perturbation import SCALE_UNIT, axpy_inplace_value, bf16_round, hybrid_z


class Tensor:
    """One parameter tensor: fp32 array `theta` [rows, cols] (holding bf16
    values when the storage type is bf16), id, optional basis."""

    def __init__(self, name, theta, tensor_id, U=None, k=0):
        self.name = name
        self.theta = np.array(theta, dtype=np.float32, copy=True)
        self.rows, self.cols = self.theta.shape
        self.tensor_id = int(tensor_id)
        self.U = None if U is None else np.asarray(U, dtype=np.float32)
        self.k = int(k) if U is not None else 0


class ZgrOracle:
    def __init__(self, tensors, loss_fn, seed, eps, alpha, dtype="f32", scale_mode=SCALE_UNIT,
                 gauss_bits=32, keep_z=False):
        """loss_fn(dict name -> fp64 array) -> python float.  keep_z: remember every Z(seed, step) of
        every tensor once computed (Z is a pure function of them, so the passes of a step, which all
        regenerate it, get the same array; only worth the memory on large models)."""
        self.z_kept = {} if keep_z else None
        self.tensors = list(tensors)
        self.loss_fn = loss_fn
        self.seed, self.eps, self.alpha = int(seed), np.float32(eps), float(alpha)
        self.dtype, self.scale_mode, self.bits = dtype, scale_mode, gauss_bits

    # -- building blocks -----------------------------------------------------
    def z_of(self, t: Tensor, step: int):
        if self.z_kept is not None and (t.tensor_id, step) in self.z_kept:
            return self.z_kept[(t.tensor_id, step)]
        z = hybrid_z(self.seed, step, t.tensor_id, t.rows, t.cols, t.U, t.k, self.alpha,
                     self.scale_mode, self.bits)
        if self.z_kept is not None:
            self.z_kept[(t.tensor_id, step)] = z
        return z

    def axpy_all(self, step: int, c):
        """theta <- rnd(theta + c Z(seed, step)) for every tensor."""
        for t in self.tensors:
            t.theta = axpy_inplace_value(t.theta, c, self.z_of(t, step), self.dtype)

    def loss(self):
        return self.loss_fn({t.name: t.theta.astype(np.float64) for t in self.tensors})

    # -- Algorithm 1 ----------------------------------------------------------
    def step(self, step: int, fuse_lr=None):
        """Client block.  Returns (L+, L-, g) with g = (L+ - L-)/(2 eps) as fp32;
        leaves theta restored (to rounding).  With a learning rate fuse_lr the
        restoring pass and the update of Algorithm 1 (theta - lr g Z) are one
        pass with the fp32 coefficient eps - lr g, each product rounded to fp32."""
        eps = self.eps
        self.axpy_all(step, eps)
        lp = self.loss()
        self.axpy_all(step, np.float32(-2.0) * eps)
        lm = self.loss()
        g = np.float32((lp - lm) / (2.0 * np.float64(eps)))
        if fuse_lr is None:
            self.axpy_all(step, eps)
        else:
            self.axpy_all(step, np.float32(eps - np.float32(np.float32(fuse_lr) * g)))
        return lp, lm, g

    def apply_update(self, step: int, g, lr):
        """Edge-server block for one client with weight 1:
        theta <- theta - lr g Z(seed, step); the product lr*g is formed in fp32."""
        c = np.float32(-(np.float32(lr) * np.float32(g)))
        self.axpy_all(step, c)


    def apply_updates(self, steps, gs, lr):
        """Edge-server block with its sum over local steps (Algorithm 1, aggregation
        line): theta <- theta - lr * sum_q g_q Z(seed, step_q), the sum taken
        exactly (fp64 over the fp32 perturbations, each coefficient -(lr g_q) an
        fp32 product), rounded to fp32 and then to the storage type once."""
        coefs = [np.float64(np.float32(-(np.float32(lr) * np.float32(g)))) for g in gs]
        for t in self.tensors:
            acc = t.theta.astype(np.float64)
            for step, c in zip(steps, coefs):
                acc = acc + c * self.z_of(t, int(step)).astype(np.float64)
            v = acc.astype(np.float32)
            t.theta = bf16_round(v) if self.dtype == "bf16" else v


# ---------------------------------------------------------------- loss adapters

def make_lsq_loss(X, Y):
    return lambda P: F.lsq_loss(P["W"], X, Y)


def make_lm_loss(tokens, n_layer, n_head, ln_eps=1e-5, act="gelu", post_ln=False):
    return lambda P: F.lm_loss(P, tokens, n_layer, n_head, ln_eps, act, post_ln)


def make_cls_loss(tokens, lengths, labels, n_layer, n_head, ln_eps=1e-5, act="gelu", post_ln=False):
    return lambda P: F.cls_loss(P, tokens, lengths, labels, n_layer, n_head, ln_eps, act, post_ln)
