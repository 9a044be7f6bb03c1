"""ctypes binding of libols.so: the same entry points as include/ols.h, argument marshalling only.

Every step of the Overlap Local-SGD iteration runs inside the library's HIP kernels.  There is no
fallback: if the library has not been built this module raises at import of the symbols.
"""
import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("OLS_LIBRARY", os.path.join(HERE, "libols.so"))   # override: an alternative build

OLS_OK, OLS_EINVAL, OLS_ESTATE, OLS_EHIP, OLS_ENOMEM = 0, -1, -2, -3, -4
(OLS_OPT_NESTEROV, OLS_OPT_FUSE_PULL, OLS_OPT_SERIALIZE, OLS_OPT_DRY_RUN, OLS_OPT_KERNEL_TIMING, OLS_OPT_TRACE,
 OLS_OPT_MEAN_SPLIT, OLS_OPT_FUSE_MEAN, OLS_OPT_TUNING) = range(1, 10)
(OLS_OPT_GEMM_SPLITK, OLS_OPT_FUSE_GEMM_UPDATE, OLS_OPT_GEMM_FORCE_GENERAL, OLS_OPT_ANCHOR_DELAY_US,
 OLS_OPT_HEAD_DW_GUEST) = range(12, 17)
TUNE_FWD, TUNE_DW, TUNE_DA = 0, 256, 512    # OLS_OPT_TUNING value = one of these + the variant number
(OLS_K_INIT, OLS_K_STEP, OLS_K_STEP_PULL, OLS_K_PULL, OLS_K_MEAN, OLS_K_STEP_PULL_MEAN, OLS_K_LSQ_RESID,
 OLS_K_LSQ_GRAD, OLS_K_GEMM_FWD, OLS_K_GEMM_DW, OLS_K_GEMM_DA, OLS_K_HEAD_FWD, OLS_K_HEAD_BWD, OLS_K_MIX,
 OLS_K_CAST, OLS_K_DELAY, OLS_K_LSQ_STEP, OLS_K_STALE_SYNC, OLS_K_CONV_FWD, OLS_K_CONV_DX, OLS_K_CONV_DW, OLS_K_POOL,
 OLS_K_POOL_BWD, OLS_K_BN_FWD, OLS_K_BN_BWD, OLS_K_COUNT) = range(26)


class ols_trace_entry(C.Structure):
    _fields_ = [("kind", C.c_int32), ("stream", C.c_int32), ("src_buf", C.c_int32), ("dst_buf", C.c_int32),
                ("waited", C.c_int32), ("k", C.c_int32)]


class OlsError(RuntimeError):
    def __init__(self, code, message):
        super().__init__("ols error %d: %s" % (code, message))
        self.code = code


_H = C.c_void_p
_P = C.c_void_p
_SIGNATURES = {
    "ols_create": (_H, [C.c_int, C.c_int64, C.c_int, C.c_float, C.c_float, C.c_float]),
    "ols_destroy": (C.c_int, [_H]),
    "ols_row_stride": (C.c_int64, [C.c_int64]),
    "ols_bind": (C.c_int, [_H, _P, _P, _P, _P, _P, C.c_int64, _P, _P]),
    "ols_init_params": (C.c_int, [_H, _P]),
    "ols_set_anchor_momentum": (C.c_int, [_H, C.c_float, _P]),
    "ols_set_mixing": (C.c_int, [_H, _P]),
    "ols_set_stale_average": (C.c_int, [_H, _P]),
    "ols_set_lr": (C.c_int, [_H, C.c_float]),
    "ols_attach_lsq": (C.c_int, [_H, C.c_int]),
    "ols_attach_mlp": (C.c_int, [_H, C.c_int, C.POINTER(C.c_int), C.c_int, C.c_int]),
    "ols_attach_convblock": (C.c_int, [_H, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int]),
    "ols_attach_convblock_bn": (C.c_int, [_H, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_float]),
    "ols_attach_convblock_bf16": (C.c_int, [_H, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int]),
    "ols_attach_convblock_bn_bf16": (C.c_int, [_H, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_float]),
    "ols_workspace_bytes": (C.c_int64, [_H]),
    "ols_bind_workspace": (C.c_int, [_H, _P, C.c_int64]),
    "ols_set_batch": (C.c_int, [_H, _P, C.c_int64, _P, C.c_int64]),
    "ols_run_steps": (C.c_int, [_H, C.c_int64, _P, _P, C.c_int]),
    "ols_run_steps_static": (C.c_int, [_H, C.c_int64, _P, _P, C.c_int]),
    "ols_static_workspace_bytes": (C.c_int64, []),
    "ols_set_gradient": (C.c_int, [_H, _P]),
    "ols_local_step": (C.c_int, [_H]),
    "ols_sync_pull": (C.c_int, [_H]),
    "ols_anchor_update_async": (C.c_int, [_H]),
    "ols_get_params": (C.c_int, [_H, C.c_int, _P, C.c_int]),
    "ols_get_loss": (C.c_int, [_H, C.POINTER(C.c_float)]),
    "ols_sync": (C.c_int, [_H]),
    "ols_set_option": (C.c_int, [_H, C.c_int, C.c_int64]),
    "ols_iteration": (C.c_int64, [_H]),
    "ols_kernel_stats": (C.c_int, [_H, C.c_int, C.POINTER(C.c_int64), C.POINTER(C.c_double)]),
    "ols_kernel_name": (C.c_char_p, [C.c_int]),
    "ols_trace_count": (C.c_int64, [_H]),
    "ols_trace_get": (C.c_int, [_H, C.c_int64, C.POINTER(ols_trace_entry)]),
    "ols_last_error": (C.c_char_p, []),
    "ols_version": (C.c_char_p, []),
}

_lib = None


def load():
    """Loads libols.so (built beforehand with `python -m paper_2002_09539_amd.build`)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise OlsError(OLS_EHIP, "libols.so is not built (%s); run python -m paper_2002_09539_amd.build" % LIB_PATH)
    lib = C.CDLL(LIB_PATH)
    for name, (res, args) in _SIGNATURES.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    _lib = lib
    return lib


def last_error():
    return load().ols_last_error().decode()


def _check(rc):
    if rc != OLS_OK:
        raise OlsError(rc, last_error())


def ols_version():
    return load().ols_version().decode()


def ols_row_stride(d):
    return load().ols_row_stride(d)


def ols_kernel_name(kind):
    return load().ols_kernel_name(kind).decode()


def ols_create(m, d, tau, alpha, gamma, beta):
    h = load().ols_create(m, d, tau, alpha, gamma, beta)
    if not h:
        raise OlsError(OLS_EINVAL, last_error())
    return h


def ols_destroy(h):
    _check(load().ols_destroy(h))


def ols_bind(h, x, x_alt, buf, g, z, ld, main_stream, side_stream):
    _check(load().ols_bind(h, x, x_alt, buf, g, z, ld, main_stream, side_stream))


def ols_init_params(h, x0):
    _check(load().ols_init_params(h, x0))


def ols_set_anchor_momentum(h, beta_z, v):
    _check(load().ols_set_anchor_momentum(h, beta_z, v))


def ols_set_mixing(h, w):
    _check(load().ols_set_mixing(h, w))


def ols_set_stale_average(h, snap):
    _check(load().ols_set_stale_average(h, snap))


def ols_set_lr(h, gamma):
    _check(load().ols_set_lr(h, gamma))


def ols_attach_lsq(h, batch):
    _check(load().ols_attach_lsq(h, batch))


def ols_attach_mlp(h, dims, batch, gemm_dtype):
    arr = (C.c_int * len(dims))(*dims)
    _check(load().ols_attach_mlp(h, len(dims) - 1, arr, batch, gemm_dtype))


def ols_attach_convblock(h, channels, height, width, classes, batch):
    _check(load().ols_attach_convblock(h, channels, height, width, classes, batch))


def ols_attach_convblock_bf16(h, channels, height, width, classes, batch):
    _check(load().ols_attach_convblock_bf16(h, channels, height, width, classes, batch))


def ols_attach_convblock_bn(h, channels, height, width, classes, batch, eps=1e-5):
    _check(load().ols_attach_convblock_bn(h, channels, height, width, classes, batch, eps))


def ols_attach_convblock_bn_bf16(h, channels, height, width, classes, batch, eps=1e-5):
    _check(load().ols_attach_convblock_bn_bf16(h, channels, height, width, classes, batch, eps))


def ols_workspace_bytes(h):
    return load().ols_workspace_bytes(h)


def ols_bind_workspace(h, ws, nbytes):
    _check(load().ols_bind_workspace(h, ws, nbytes))


def ols_set_batch(h, X, x_worker_stride, y, y_worker_stride):
    _check(load().ols_set_batch(h, X, x_worker_stride, y, y_worker_stride))


def ols_run_steps(h, steps, X, y, nb):
    _check(load().ols_run_steps(h, steps, X, y, nb))


def ols_run_steps_static(h, steps, X, y, nb):
    _check(load().ols_run_steps_static(h, steps, X, y, nb))


def ols_static_workspace_bytes():
    return load().ols_static_workspace_bytes()


def ols_set_gradient(h, g):
    _check(load().ols_set_gradient(h, g))


def ols_local_step(h):
    _check(load().ols_local_step(h))


def ols_sync_pull(h):
    _check(load().ols_sync_pull(h))


def ols_anchor_update_async(h):
    _check(load().ols_anchor_update_async(h))


def ols_get_params(h, which, dst, dst_is_device):
    _check(load().ols_get_params(h, which, dst, dst_is_device))


def ols_get_loss(h, m):
    out = (C.c_float * m)()
    _check(load().ols_get_loss(h, out))
    return list(out)


def ols_sync(h):
    _check(load().ols_sync(h))


def ols_set_option(h, key, value):
    _check(load().ols_set_option(h, key, value))


def ols_iteration(h):
    return load().ols_iteration(h)


def ols_kernel_stats(h, kind):
    n, ms = C.c_int64(0), C.c_double(0.0)
    _check(load().ols_kernel_stats(h, kind, C.byref(n), C.byref(ms)))
    return n.value, ms.value


def ols_trace(h):
    lib = load()
    out = []
    for i in range(lib.ols_trace_count(h)):
        e = ols_trace_entry()
        _check(lib.ols_trace_get(h, i, C.byref(e)))
        out.append(dict(kind=e.kind, stream=e.stream, src_buf=e.src_buf, dst_buf=e.dst_buf, waited=e.waited, k=e.k))
    return out
