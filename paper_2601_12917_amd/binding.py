"""ctypes binding of libzgr.so: the same names and arguments as include/zgr.h.

Argument marshalling only; every step of the path runs in the library's HIP
kernels.  There is no fallback: if the shared library is missing, importing
this module's `lib()` raises.
"""
import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libzgr.so")

# enums of zgr.h
ZGR_ACT_GELU, ZGR_ACT_RELU = 0, 1
ZGR_OK, ZGR_ERR_NULL, ZGR_ERR_SHAPE, ZGR_ERR_DTYPE, ZGR_ERR_CONFIG = 0, 1, 2, 3, 4
ZGR_ERR_WORKSPACE, ZGR_ERR_DEVICE, ZGR_ERR_NONFINITE, ZGR_ERR_STATE = 5, 6, 7, 8
ZGR_F32, ZGR_BF16 = 0, 1
ZGR_SCALE_UNIT, ZGR_SCALE_PAPER = 0, 1
ZGR_MAX_BATCH = 8
ZGR_ARCH_NONE, ZGR_ARCH_LINEAR_LSQ, ZGR_ARCH_DECODER_LM, ZGR_ARCH_ENCODER_CLS = -1, 0, 1, 2
ZGR_K_PERTURB_TILE, ZGR_K_PERTURB_FLAT, ZGR_K_GEMM, ZGR_K_ATTN, ZGR_K_NORM, ZGR_K_EMBED, ZGR_K_LOSS, ZGR_K_COUNT = range(8)
KERNEL_CLASS_NAMES = ("perturb_tile", "perturb_flat", "gemm", "attention", "norm", "embed", "loss")


class zgr_tensor(C.Structure):
    _fields_ = [("theta", C.c_void_p), ("rows", C.c_int64), ("cols", C.c_int64), ("dtype", C.c_int32),
                ("tensor_id", C.c_uint32), ("U", C.c_void_p), ("k", C.c_int32), ("ldu", C.c_int32),
                ("role", C.c_int32), ("layer", C.c_int32)]


class zgr_model(C.Structure):
    _fields_ = [("arch", C.c_int32), ("n_layer", C.c_int32), ("d_model", C.c_int32), ("n_head", C.c_int32),
                ("d_ff", C.c_int32), ("vocab", C.c_int32), ("max_pos", C.c_int32), ("n_class", C.c_int32),
                ("ln_eps", C.c_float), ("act", C.c_int32), ("post_ln", C.c_int32)]


class zgr_config(C.Structure):
    _fields_ = [("seed", C.c_uint64), ("eps", C.c_float), ("alpha", C.c_float), ("scale_mode", C.c_int32),
                ("gauss_bits", C.c_int32), ("fuse_restore_update", C.c_int32), ("lr", C.c_float)]


class zgr_batch(C.Structure):
    _fields_ = [("x", C.c_void_p), ("y", C.c_void_p), ("lengths", C.c_void_p), ("batch", C.c_int32), ("seq", C.c_int32)]


class zgr_result(C.Structure):
    _fields_ = [("loss_plus", C.c_double), ("loss_minus", C.c_double), ("g", C.c_float)]


# every symbol include/zgr.h declares: name -> (restype, argtypes)
SYMBOLS = {
    "zgr_workspace_bytes": (C.c_size_t, [C.POINTER(zgr_model), C.POINTER(zgr_tensor), C.c_int32, C.c_int32, C.c_int32]),
    "zgr_init": (C.c_int, [C.POINTER(C.c_void_p), C.POINTER(zgr_model), C.POINTER(zgr_tensor), C.c_int32, C.POINTER(zgr_config),
                           C.c_void_p, C.c_size_t, C.c_int32, C.c_int32, C.c_void_p]),
    "zgr_set_basis": (C.c_int, [C.c_void_p, C.c_int32, C.c_void_p, C.c_int32, C.c_int32]),
    "zgr_set_basis_q4": (C.c_int, [C.c_void_p, C.c_int32, C.c_void_p, C.c_int32, C.c_int32, C.c_float, C.c_float]),
    "zgr_set_basis_host": (C.c_int, [C.c_void_p, C.c_int32, C.c_void_p, C.c_int32, C.c_int32, C.c_float, C.c_float]),
    "zgr_quantize_basis": (C.c_int, [C.c_void_p, C.c_int64, C.c_int32, C.c_int32, C.c_void_p, C.c_int32, C.c_void_p,
                                     C.POINTER(C.c_float), C.POINTER(C.c_float), C.c_void_p]),
    "zgr_dtc_omega": (C.c_int, [C.c_double, C.c_double, C.c_double, C.c_double, C.c_double, C.POINTER(C.c_double), C.POINTER(C.c_int32)]),
    "zgr_dtc_memory_factor": (C.c_int, [C.c_int32, C.c_double, C.c_double, C.POINTER(C.c_double)]),
    "zgr_cloud_basis_workspace": (C.c_size_t, [C.c_int64, C.c_int64, C.c_int32]),
    "zgr_cloud_basis": (C.c_int, [C.POINTER(C.c_void_p), C.c_int32, C.c_int64, C.c_int64, C.c_int32, C.c_void_p, C.c_int32, C.c_void_p, C.c_int32,
                                  C.POINTER(C.c_int32), C.c_void_p, C.c_size_t, C.c_void_p]),
    "zgr_cloud_backward_workspace": (C.c_size_t, [C.c_void_p, C.c_int32, C.c_int32]),
    "zgr_cloud_backward": (C.c_int, [C.c_void_p, C.c_void_p, C.POINTER(C.c_void_p), C.c_int32, C.POINTER(C.c_double), C.c_void_p, C.c_size_t]),
    "zgr_cloud_lsq_gradient": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "zgr_step": (C.c_int, [C.c_void_p, C.c_uint64, C.POINTER(zgr_batch), C.POINTER(zgr_result)]),
    "zgr_apply_update": (C.c_int, [C.c_void_p, C.c_uint64, C.c_float, C.c_float]),
    "zgr_apply_updates": (C.c_int, [C.c_void_p, C.c_int32, C.POINTER(C.c_uint64), C.POINTER(C.c_float), C.c_float]),
    "zgr_perturb": (C.c_int, [C.c_void_p, C.c_uint64, C.c_float]),
    "zgr_loss": (C.c_int, [C.c_void_p, C.POINTER(zgr_batch), C.POINTER(C.c_double)]),
    "zgr_lsq_loss_static": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]),
    "zgr_destroy": (None, [C.c_void_p]),
    "zgr_last_error": (C.c_char_p, [C.c_void_p]),
    "zgr_profile_enable": (C.c_int, [C.c_void_p, C.c_int32]),
    "zgr_profile_pause": (C.c_int, [C.c_void_p, C.c_int32]),
    "zgr_profile_read": (C.c_int, [C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_int64)]),
    "zgr_debug_philox": (C.c_int, [C.c_void_p, C.POINTER(C.c_uint32), C.c_void_p, C.c_int64, C.c_void_p]),
    "zgr_debug_gauss": (C.c_int, [C.c_uint64, C.c_uint64, C.c_uint32, C.c_int32, C.c_int32, C.c_int64, C.c_int64, C.c_void_p, C.c_void_p]),
    "zgr_debug_fill_z": (C.c_int, [C.c_void_p, C.c_int32, C.c_uint64, C.c_void_p]),
    "zgr_debug_set_stage_tiles": (C.c_int, [C.c_void_p, C.c_int64]),
    "zgr_debug_last_row_losses": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int64]),
    "zgr_debug_step_row_losses": (C.c_int, [C.c_void_p, C.c_int32, C.c_void_p, C.c_int64]),
    "zgr_debug_radius_table": (C.c_int, [C.c_int32, C.c_void_p, C.c_void_p]),
    "zgr_debug_cossin_table": (C.c_int, [C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]),
    "zgr_debug_copy": (C.c_int, [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "zgr_debug_rmw": (C.c_int, [C.c_void_p, C.c_size_t, C.c_int32, C.c_float, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]),
    "zgr_debug_issue_rate": (C.c_int, [C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]),
    "zgr_debug_generator_rate": (C.c_int, [C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]),
    "zgr_debug_gemm": (C.c_int, [C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p]),
}

_lib = None


def lib():
    """The loaded library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2601_12917_amd.build` first "
                               "(there is no CPU fallback)")
        l = C.CDLL(LIB_PATH)
        for name, (res, args) in SYMBOLS.items():
            f = getattr(l, name)
            f.restype, f.argtypes = res, args
        _lib = l
    return _lib


class ZgrError(RuntimeError):
    def __init__(self, status, message):
        super().__init__(f"zgr status {status}: {message}")
        self.status = status


def check(status, ctx=None):
    if status != ZGR_OK:
        msg = lib().zgr_last_error(ctx)
        raise ZgrError(status, msg.decode() if msg else "")


def dtc_omega(data_bytes, bandwidth_bytes_per_s, t_cc_s, restore_s_per_byte, theta):
    """(omega, hidden) of zgr_dtc_omega: argument marshalling only."""
    w, ok = C.c_double(0), C.c_int32(0)
    check(lib().zgr_dtc_omega(float(data_bytes), float(bandwidth_bytes_per_s), float(t_cc_s), float(restore_s_per_byte), float(theta),
                              C.byref(w), C.byref(ok)))
    return w.value, bool(ok.value)


def dtc_memory_factor(n_layers, omega, theta):
    f = C.c_double(0)
    check(lib().zgr_dtc_memory_factor(int(n_layers), float(omega), float(theta), C.byref(f)))
    return f.value

