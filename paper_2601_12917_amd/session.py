"""Device-memory plumbing around the C ABI: allocates parameters, bases, batch
and workspace with torch, builds the tensor table and forwards every call to
libzgr.so.  No arithmetic of the method happens here."""
import ctypes as C
from typing import List, Optional, Sequence

import numpy as np
import torch

from . import binding as B


class ParamSpec:
    """One tensor handed to the session: host values fp32 [rows, cols]
    (bf16-representable when dtype is 'bf16'), optional basis fp32 [rows, ldu]."""

    def __init__(self, name, role, layer, tensor_id, values, U=None, k=0):
        self.name, self.role, self.layer, self.tensor_id = name, int(role), int(layer), int(tensor_id)
        self.values = np.ascontiguousarray(values, dtype=np.float32)
        self.U = None if U is None else np.ascontiguousarray(U, dtype=np.float32)
        self.k = int(k) if U is not None else 0


def _align(x, a=256):
    return (x + a - 1) // a * a


class Session:
    def __init__(self, arch, dtype, params: Sequence[ParamSpec], seed, eps, alpha, scale_mode=B.ZGR_SCALE_UNIT,
                 gauss_bits=32, n_layer=0, d_model=0, n_head=0, d_ff=0, vocab=0, max_pos=0, n_class=0, ln_eps=1e-5,
                 max_batch=1, max_seq=2, device="cuda:0", pack_after=(), fuse_lr=None, act="gelu", post_ln=False):
        """pack_after: names of tensors that must start right where the previous one ends
        (Wk, Wv after Wq; bk, bv after bq).  fuse_lr: a learning rate makes step() end with the fused
        restore + update pass (apply_update is then not to be called)."""
        self.lib = B.lib()
        self.dev = torch.device(device)
        torch.cuda.set_device(self.dev)
        self.dtype = dtype
        self.tdtype = torch.float32 if dtype == "f32" else torch.bfloat16
        es = 4 if dtype == "f32" else 2
        self.params = list(params)
        # one slab for all parameters
        offs, off = [], 0
        for p in self.params:
            if p.name not in pack_after:
                off = _align(off)
            offs.append(off)
            off += p.values.size * es
        self.slab = torch.zeros(_align(off) // es, dtype=self.tdtype, device=self.dev)
        self.theta: List[torch.Tensor] = []
        for p, o in zip(self.params, offs):
            t = self.slab[o // es: o // es + p.values.size].view(p.values.shape)
            t.copy_(torch.from_numpy(p.values).to(self.tdtype))
            self.theta.append(t)
        self.U = [None if p.U is None else torch.from_numpy(p.U).to(self.dev) for p in self.params]
        self.table = (B.zgr_tensor * len(self.params))()
        for i, p in enumerate(self.params):
            e = self.table[i]
            e.theta = self.theta[i].data_ptr()
            e.rows, e.cols = p.values.shape
            e.dtype = B.ZGR_F32 if dtype == "f32" else B.ZGR_BF16
            e.tensor_id = p.tensor_id
            e.U = self.U[i].data_ptr() if self.U[i] is not None else None
            e.k = p.k
            e.ldu = p.U.shape[1] if p.U is not None else 0
            e.role, e.layer = p.role, p.layer
        self.model = B.zgr_model(arch, n_layer, d_model, n_head, d_ff, vocab, max_pos, n_class, ln_eps,
                                 {"gelu": B.ZGR_ACT_GELU, "relu": B.ZGR_ACT_RELU}[act], 1 if post_ln else 0)
        self.config = B.zgr_config(seed, eps, alpha, scale_mode, gauss_bits, 0 if fuse_lr is None else 1,
                                     0.0 if fuse_lr is None else fuse_lr)
        nbytes = self.lib.zgr_workspace_bytes(C.byref(self.model), self.table, len(self.params), max_batch, max_seq)
        if nbytes == 0:
            raise B.ZgrError(B.ZGR_ERR_SHAPE, "zgr_workspace_bytes rejected the arguments")
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=self.dev)
        self.stream = torch.cuda.current_stream(self.dev)
        self.ctx = C.c_void_p()
        st = self.lib.zgr_init(C.byref(self.ctx), C.byref(self.model), self.table, len(self.params), C.byref(self.config),
                               self.workspace.data_ptr(), nbytes, max_batch, max_seq, self.stream.cuda_stream)
        B.check(st, None)
        self._batch_keep = None

    # ---- batches --------------------------------------------------------------
    def make_batch(self, x, y=None, lengths=None, seq=0):
        keep = []

        def up(a):
            if a is None:
                return None
            t = torch.from_numpy(np.ascontiguousarray(a)).to(self.dev)
            keep.append(t)
            return t.data_ptr()
        b = B.zgr_batch(up(x), up(y), up(lengths), int(np.asarray(x).shape[0]), int(seq))
        self._batch_keep = keep
        return b

    # ---- calls of the C ABI ---------------------------------------------------
    def step(self, step, batch):
        r = B.zgr_result()
        B.check(self.lib.zgr_step(self.ctx, step, C.byref(batch), C.byref(r)), self.ctx)
        return r.loss_plus, r.loss_minus, r.g

    def apply_update(self, step, g, lr):
        B.check(self.lib.zgr_apply_update(self.ctx, step, g, lr), self.ctx)

    def apply_updates(self, steps, gs, lr):
        n = len(steps)
        sa = (C.c_uint64 * max(n, 1))(*[int(x) for x in steps])
        ga = (C.c_float * max(n, 1))(*[float(x) for x in gs])
        B.check(self.lib.zgr_apply_updates(self.ctx, n, sa, ga, lr), self.ctx)

    def perturb(self, step, c):
        B.check(self.lib.zgr_perturb(self.ctx, step, c), self.ctx)

    def loss(self, batch):
        v = C.c_double()
        B.check(self.lib.zgr_loss(self.ctx, C.byref(batch), C.byref(v)), self.ctx)
        return v.value

    def cloud_backward(self, batch, seq=0):
        """(loss, [dL/dtheta_i as a device fp32 tensor [rows, cols] per parameter]) by zgr_cloud_backward."""
        n_b = int(batch.batch)
        nbytes = self.lib.zgr_cloud_backward_workspace(self.ctx, n_b, int(batch.seq) if batch.seq else int(seq))
        if nbytes == 0:
            raise RuntimeError("zgr_cloud_backward_workspace returned 0 (a context without a model, or a bad batch)")
        ws = torch.empty(nbytes, dtype=torch.uint8, device=self.dev)
        grads = [torch.empty(*p.values.shape, dtype=torch.float32, device=self.dev) for p in self.params]
        ptrs = (C.c_void_p * len(grads))(*[g.data_ptr() for g in grads])
        v = C.c_double()
        B.check(self.lib.zgr_cloud_backward(self.ctx, C.byref(batch), ptrs, len(grads), C.byref(v), ws.data_ptr(), nbytes), self.ctx)
        return v.value, grads

    def set_basis(self, index, U: Optional[np.ndarray], k):
        if U is None:
            B.check(self.lib.zgr_set_basis(self.ctx, index, None, 0, 0), self.ctx)
            return
        t = torch.from_numpy(np.ascontiguousarray(U, dtype=np.float32)).to(self.dev)
        self.U[index] = t
        B.check(self.lib.zgr_set_basis(self.ctx, index, t.data_ptr(), k, U.shape[1]), self.ctx)

    def set_basis_q4(self, index, codes_packed: np.ndarray, k, lam, delta):
        """codes_packed: uint8 [rows, ldq] (two 4-bit codes per byte)."""
        t = torch.from_numpy(np.ascontiguousarray(codes_packed, dtype=np.uint8)).to(self.dev)
        self.Uq = getattr(self, "Uq", {})
        self.Uq[index] = t
        B.check(self.lib.zgr_set_basis_q4(self.ctx, index, t.data_ptr(), k, codes_packed.shape[1], float(lam), float(delta)), self.ctx)

    def quantize_basis(self, U: np.ndarray, k):
        """Device quantiser: returns (packed codes uint8 [rows, (k+1)//2], lambda, delta)."""
        u = torch.from_numpy(np.ascontiguousarray(U, dtype=np.float32)).to(self.dev)
        rows, ldu = u.shape
        ldq = (k + 1) // 2
        q = torch.zeros(rows, ldq, dtype=torch.uint8, device=self.dev)
        mm = torch.zeros(2, dtype=torch.float32, device=self.dev)
        lam, delta = C.c_float(0), C.c_float(0)
        B.check(self.lib.zgr_quantize_basis(u.data_ptr(), rows, k, ldu, q.data_ptr(), ldq, mm.data_ptr(), C.byref(lam), C.byref(delta),
                                            self.stream.cuda_stream), None)
        torch.cuda.synchronize(self.dev)
        return q.cpu().numpy(), lam.value, delta.value

    def set_basis_host(self, index, U: np.ndarray, k, codes=None, lam=0.0, delta=0.0):
        """Keep the basis of one tensor in pinned host memory (compact rows of its first k columns) and let the
        kernels stream it per layer during the passes.  codes: packed 4-bit codes [rows, (k+1)//2] instead of U
        (then lam, delta are their scale and zero point)."""
        src = (np.ascontiguousarray(codes[:, :(k + 1) // 2], dtype=np.uint8) if codes is not None
               else np.ascontiguousarray(U[:, :k], dtype=np.float32))
        t = torch.from_numpy(src).pin_memory()
        self.Uhost = getattr(self, "Uhost", {})
        self.Uhost[index] = t
        B.check(self.lib.zgr_set_basis_host(self.ctx, index, t.data_ptr(), k, 4 if codes is not None else 32,
                                            float(lam), float(delta)), self.ctx)

    def set_layer_bases_host(self, indices, arrays, k, codes=False, lams=None, deltas=None):
        """Stream the bases of one layer from ONE pinned block laid out like the staging slot (tensor order, compact
        rows, each tensor padded to 256 bytes), so that the whole layer travels as a single transfer.
        arrays: fp32 [rows, >= k] per tensor, or packed 4-bit codes [rows, (k+1)//2] when codes=True."""
        width = (k + 1) // 2 if codes else 4 * k
        offs, off = [], 0
        for a in arrays:
            offs.append(off)
            off += _align(a.shape[0] * width)
        block = torch.zeros(off, dtype=torch.uint8).pin_memory()
        view = block.numpy()
        for a, o in zip(arrays, offs):
            src = np.ascontiguousarray(a[:, :(k + 1) // 2], dtype=np.uint8) if codes else np.ascontiguousarray(a[:, :k], dtype=np.float32)
            view[o:o + src.nbytes] = src.view(np.uint8).reshape(-1)
        self.Uhost = getattr(self, "Uhost", {})
        for j, (i, o) in enumerate(zip(indices, offs)):
            self.Uhost[i] = block
            B.check(self.lib.zgr_set_basis_host(self.ctx, i, block.data_ptr() + o, k, 4 if codes else 32,
                                                float(lams[j]) if codes else 0.0, float(deltas[j]) if codes else 0.0), self.ctx)

    def set_stage_tiles(self, min_tiles):
        B.check(self.lib.zgr_debug_set_stage_tiles(self.ctx, int(min_tiles)), self.ctx)

    def compress_basis(self, index):
        """Quantise the installed fp32 basis of one tensor to 4 bits on the device and install the codes in its place."""
        u, k = self.U[index], self.params[index].k
        rows, ldu = u.shape
        ldq = (k + 1) // 2
        q = torch.zeros(rows, ldq, dtype=torch.uint8, device=self.dev)
        mm = torch.zeros(2, dtype=torch.float32, device=self.dev)
        lam, delta = C.c_float(0), C.c_float(0)
        B.check(self.lib.zgr_quantize_basis(u.data_ptr(), rows, k, ldu, q.data_ptr(), ldq, mm.data_ptr(), C.byref(lam), C.byref(delta),
                                            self.stream.cuda_stream), None)
        self.Uq = getattr(self, "Uq", {})
        self.Uq[index] = q
        B.check(self.lib.zgr_set_basis_q4(self.ctx, index, q.data_ptr(), k, ldq, lam.value, delta.value), self.ctx)
        return lam.value, delta.value

    def fill_z(self, index, step):
        rows, cols = self.params[index].values.shape
        z = torch.empty(rows, cols, dtype=torch.float32, device=self.dev)
        B.check(self.lib.zgr_debug_fill_z(self.ctx, index, step, z.data_ptr()), self.ctx)
        torch.cuda.synchronize(self.dev)
        return z.cpu().numpy()

    def last_row_losses(self, n):
        out = np.empty(n, dtype=np.float32)
        B.check(self.lib.zgr_debug_last_row_losses(self.ctx, out.ctypes.data, n), self.ctx)
        return out

    def step_row_losses(self, which, n):
        """Row losses of the last step's forward at W + eps Z (which = 0) or W - eps Z (which = 1)."""
        out = np.empty(n, dtype=np.float32)
        B.check(self.lib.zgr_debug_step_row_losses(self.ctx, which, out.ctypes.data, n), self.ctx)
        return out

    def profile_enable(self, on=True):
        B.check(self.lib.zgr_profile_enable(self.ctx, 1 if on else 0), self.ctx)

    def profile_read(self):
        ms = (C.c_double * B.ZGR_K_COUNT)()
        n = (C.c_int64 * B.ZGR_K_COUNT)()
        B.check(self.lib.zgr_profile_read(self.ctx, ms, n), self.ctx)
        return {name: (ms[i], n[i]) for i, name in enumerate(B.KERNEL_CLASS_NAMES)}

    def get_theta(self, index):
        torch.cuda.synchronize(self.dev)
        return self.theta[index].float().cpu().numpy()

    def set_theta(self, index, values):
        self.theta[index].copy_(torch.from_numpy(np.ascontiguousarray(values, dtype=np.float32)).to(self.tdtype))

    def close(self):
        if self.ctx:
            self.lib.zgr_destroy(self.ctx)
            self.ctx = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


# ---- context-free debug exports ------------------------------------------------
def debug_philox(ctr: np.ndarray, key, device="cuda:0"):
    lib = B.lib()
    c = torch.from_numpy(np.ascontiguousarray(ctr, dtype=np.uint32).view(np.int32)).to(device)
    out = torch.empty_like(c)
    k = (C.c_uint32 * 2)(int(key[0]), int(key[1]))
    B.check(lib.zgr_debug_philox(c.data_ptr(), k, out.data_ptr(), c.shape[0], torch.cuda.current_stream().cuda_stream))
    torch.cuda.synchronize()
    return out.cpu().numpy().view(np.uint32)


def debug_gauss(seed, step, tensor_id, stream, bits, first, n, device="cuda:0"):
    lib = B.lib()
    out = torch.empty(n, dtype=torch.float32, device=device)
    B.check(lib.zgr_debug_gauss(seed, step, tensor_id, stream, bits, first, n, out.data_ptr(), torch.cuda.current_stream().cuda_stream))
    torch.cuda.synchronize()
    return out.cpu().numpy()


def debug_radius_table(bits, device="cuda:0"):
    lib = B.lib()
    out = torch.empty(1 << (23 if bits == 32 else 16), dtype=torch.float32, device=device)
    B.check(lib.zgr_debug_radius_table(bits, out.data_ptr(), torch.cuda.current_stream().cuda_stream))
    torch.cuda.synchronize()
    return out.cpu().numpy()


def debug_cossin_table(bits, device="cuda:0"):
    lib = B.lib()
    n = 1 << (24 if bits == 32 else 16)
    c = torch.empty(n, dtype=torch.float32, device=device)
    s = torch.empty(n, dtype=torch.float32, device=device)
    B.check(lib.zgr_debug_cossin_table(bits, c.data_ptr(), s.data_ptr(), torch.cuda.current_stream().cuda_stream))
    torch.cuda.synchronize()
    return c.cpu().numpy(), s.cpu().numpy()


# ---- cloud block of Algorithm 1 (context-free) ----------------------------------
def cloud_basis_device(snaps, k, omega, n_iter, ldu=None):
    """(U [rows, ldu] device tensor, dependent columns) from device fp32 snapshots [rows, cols] and a device start omega [cols, k]."""
    lib = B.lib()
    snaps = [g.contiguous() for g in snaps]
    rows, cols = snaps[0].shape
    ldu = ldu or k
    om = omega.contiguous()
    U = torch.zeros(rows, ldu, dtype=torch.float32, device=snaps[0].device)
    nbytes = lib.zgr_cloud_basis_workspace(rows, cols, k)
    ws = torch.empty(nbytes, dtype=torch.uint8, device=snaps[0].device)
    ptrs = (C.c_void_p * len(snaps))(*[t.data_ptr() for t in snaps])
    dep = C.c_int32(-1)
    B.check(lib.zgr_cloud_basis(ptrs, len(snaps), rows, cols, k, om.data_ptr(), n_iter, U.data_ptr(), ldu, C.byref(dep), ws.data_ptr(), nbytes,
                                torch.cuda.current_stream().cuda_stream))
    torch.cuda.synchronize()
    return U, dep.value


def cloud_basis(snapshots, k, omega, n_iter, ldu=None, device="cuda:0"):
    """U [rows, ldu] and the number of dependent columns: zgr_cloud_basis on host arrays (marshalling only)."""
    snaps = [torch.from_numpy(np.ascontiguousarray(g, dtype=np.float32)).to(device) for g in snapshots]
    om = torch.from_numpy(np.ascontiguousarray(omega, dtype=np.float32)).to(device)
    U, dep = cloud_basis_device(snaps, k, om, n_iter, ldu)
    return U.cpu().numpy(), dep


def cloud_lsq_gradient(W, X, Y, device="cuda:0"):
    lib = B.lib()
    w, x, y = (torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device) for a in (W, X, Y))
    G = torch.zeros_like(w)
    ws = torch.empty(x.shape[0] * w.shape[0] * 4, dtype=torch.uint8, device=device)
    B.check(lib.zgr_cloud_lsq_gradient(w.data_ptr(), x.data_ptr(), y.data_ptr(), x.shape[0], w.shape[0], w.shape[1], G.data_ptr(), ws.data_ptr(), ws.numel(),
                                       torch.cuda.current_stream().cuda_stream))
    torch.cuda.synchronize()
    return G.cpu().numpy()
