"""ctypes binding of the C ABI in include/br.h -- argument marshalling only.

Function names and argument order follow the header.  PyTorch is used by callers for
device memory and the stream handle; this module only passes raw pointers through.
Importing this module raises if the HIP library has not been built: there is no
fallback path.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libbr_hip.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it with `python -m paper_2602_03515_amd.build` "
        "(hipcc, gfx950). The optimizer has no CPU or PyTorch fallback.")

_lib = C.CDLL(LIB_PATH)

# ---- enums (values as in br.h) --------------------------------------------------------
BR_OK, BR_ERR_INVALID_ARG, BR_ERR_SHAPE, BR_ERR_DTYPE, BR_ERR_STATE, BR_ERR_WORKSPACE, BR_ERR_HIP, \
    BR_ERR_UNSUPPORTED = range(8)
BR_F32, BR_BF16 = 0, 1
BR_BILATERAL, BR_UNILATERAL = 0, 1
BR_SRC_SECOND, BR_SRC_FIRST = 0, 1
BR_MATH_F32, BR_MATH_BF16, BR_MATH_BF16X3 = 0, 1, 2
BR_REFRESH_AUTO, BR_REFRESH_F32, BR_REFRESH_F16X3 = 0, 1, 2
BR_STATE_M, BR_STATE_S, BR_STATE_L, BR_STATE_R, BR_STATE_QL, BR_STATE_QR, BR_STATE_MASTER, BR_STATE_NORMS, \
    BR_STATE_MROT = range(9)

STATUS_NAMES = ["BR_OK", "BR_ERR_INVALID_ARG", "BR_ERR_SHAPE", "BR_ERR_DTYPE", "BR_ERR_STATE",
                "BR_ERR_WORKSPACE", "BR_ERR_HIP", "BR_ERR_UNSUPPORTED"]


class br_matrix_desc(C.Structure):
    _fields_ = [("m", C.c_int64), ("n", C.c_int64), ("param_dtype", C.c_int32), ("grad_dtype", C.c_int32),
                ("rotate", C.c_int32), ("reserved", C.c_int32)]


class br_hparams(C.Structure):
    _fields_ = [("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float), ("weight_decay", C.c_float),
                ("stat_beta", C.c_float), ("geometry", C.c_int32), ("source", C.c_int32),
                ("power_iters", C.c_int32), ("bias_correction", C.c_int32), ("eps_outside_sqrt", C.c_int32),
                ("math", C.c_int32), ("compute_norms", C.c_int32), ("stats_on_refresh_only", C.c_int32),
                ("refresh_math", C.c_int32), ("cache_rotated_moment", C.c_int32)]


class br_profile_entry(C.Structure):
    _fields_ = [("kernel", C.c_char * 64), ("launches", C.c_int64), ("ms", C.c_double), ("flops", C.c_double),
                ("bytes", C.c_double)]


_ctx_p = C.c_void_p

_lib.br_workspace_bytes.argtypes = [C.POINTER(br_matrix_desc), C.c_int32, C.POINTER(br_hparams),
                                    C.POINTER(C.c_size_t), C.POINTER(C.c_size_t)]
_lib.br_workspace_bytes.restype = C.c_int
_lib.br_init.argtypes = [C.POINTER(_ctx_p), C.POINTER(br_matrix_desc), C.c_int32, C.POINTER(br_hparams),
                         C.c_void_p, C.c_size_t, C.c_void_p]
_lib.br_init.restype = C.c_int
_lib.br_accumulate_stats.argtypes = [_ctx_p, C.POINTER(C.c_void_p), C.c_int32]
_lib.br_accumulate_stats.restype = C.c_int
_lib.br_clip_gradients.argtypes = [_ctx_p, C.POINTER(C.c_void_p), C.c_int32, C.c_float]
_lib.br_clip_gradients.restype = C.c_int
_lib.br_delay_compensate.argtypes = [_ctx_p, C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), C.c_int32,
                                     C.c_float]
_lib.br_delay_compensate.restype = C.c_int
_lib.br_get_clip_result.argtypes = [_ctx_p, C.POINTER(C.c_void_p)]
_lib.br_get_clip_result.restype = C.c_int
_lib.br_clip_gradients_static.argtypes = [C.POINTER(br_matrix_desc), C.POINTER(C.c_void_p), C.c_int32, C.c_float, C.c_void_p,
                                          C.c_void_p]
_lib.br_clip_gradients_static.restype = C.c_int
_lib.br_refresh_basis.argtypes = [_ctx_p]
_lib.br_refresh_basis.restype = C.c_int
_lib.br_step.argtypes = [_ctx_p, C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), C.c_int32, C.c_float]
_lib.br_step.restype = C.c_int
_lib.br_get_state.argtypes = [_ctx_p, C.c_int32, C.c_int32, C.POINTER(C.c_void_p), C.POINTER(C.c_int64),
                              C.POINTER(C.c_int64)]
_lib.br_get_state.restype = C.c_int
_lib.br_get_health.argtypes = [_ctx_p, C.POINTER(C.c_void_p)]
_lib.br_get_health.restype = C.c_int
_lib.br_check_health.argtypes = [_ctx_p, C.POINTER(C.c_int32)]
_lib.br_check_health.restype = C.c_int
_lib.br_set_qr_wait_limit.argtypes = [_ctx_p, C.c_int64]
_lib.br_set_qr_wait_limit.restype = C.c_int
_lib.br_notify_state_written.argtypes = [_ctx_p]
_lib.br_notify_state_written.restype = C.c_int
_lib.br_get_step_count.argtypes = [_ctx_p, C.POINTER(C.c_int64)]
_lib.br_get_step_count.restype = C.c_int
_lib.br_set_step_count.argtypes = [_ctx_p, C.c_int64]
_lib.br_set_step_count.restype = C.c_int
_lib.br_profile_begin.argtypes = [_ctx_p]
_lib.br_profile_begin.restype = C.c_int
_lib.br_profile_end.argtypes = [_ctx_p, C.POINTER(br_profile_entry), C.c_int32, C.POINTER(C.c_int32)]
_lib.br_profile_end.restype = C.c_int
_lib.br_last_error.argtypes = [_ctx_p]
_lib.br_last_error.restype = C.c_char_p
_lib.br_version.argtypes = []
_lib.br_version.restype = C.c_char_p
_lib.br_destroy.argtypes = [_ctx_p]
_lib.br_destroy.restype = None

BR_STATIC_CLIP_MAX_MATS = 4096

EXPORTED = ["br_workspace_bytes", "br_init", "br_delay_compensate", "br_clip_gradients", "br_clip_gradients_static", "br_get_clip_result", "br_accumulate_stats", "br_refresh_basis", "br_step", "br_get_state",
            "br_get_health", "br_check_health", "br_set_qr_wait_limit", "br_notify_state_written", "br_get_step_count", "br_set_step_count", "br_profile_begin", "br_profile_end", "br_last_error",
            "br_version", "br_destroy"]


class BrError(RuntimeError):
    def __init__(self, status: int, where: str, text: str):
        self.status = status
        name = STATUS_NAMES[status] if 0 <= status < len(STATUS_NAMES) else str(status)
        super().__init__(f"{where}: {name}: {text}")


def _check(status: int, where: str, ctx=None):
    if status != BR_OK:
        raise BrError(status, where, br_last_error(ctx))


def make_descs(shapes: Sequence, param_dtype=BR_F32, grad_dtype=BR_F32, rotate=1):
    """shapes: iterable of (m, n) or (m, n, param_dtype, grad_dtype, rotate)."""
    arr = (br_matrix_desc * len(shapes))()
    for i, s in enumerate(shapes):
        m, n = int(s[0]), int(s[1])
        pd, gd, ro = (s[2], s[3], s[4]) if len(s) >= 5 else (param_dtype, grad_dtype, rotate)
        arr[i] = br_matrix_desc(m, n, int(pd), int(gd), int(ro), 0)
    return arr


def make_hparams(beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.0, stat_beta=-1.0, geometry=BR_BILATERAL,
                 source=BR_SRC_SECOND, power_iters=1, bias_correction=0, eps_outside_sqrt=0, math=BR_MATH_F32,
                 compute_norms=0, cache_rotated_moment=1, stats_on_refresh_only=0, refresh_math=0) -> br_hparams:
    return br_hparams(beta1, beta2, eps, weight_decay, stat_beta, geometry, source, power_iters,
                      int(bias_correction), int(eps_outside_sqrt), math, int(compute_norms),
                      int(stats_on_refresh_only), int(refresh_math), int(cache_rotated_moment))


def _ptr_array(ptrs: Sequence[int]):
    arr = (C.c_void_p * len(ptrs))()
    for i, p in enumerate(ptrs):
        arr[i] = C.c_void_p(int(p) if p else None)
    return arr


# ---- the calls, same names as the header ------------------------------------------------
def br_version() -> str:
    return _lib.br_version().decode()


def br_last_error(ctx=None) -> str:
    return _lib.br_last_error(ctx).decode()


def br_workspace_bytes(descs, hp: br_hparams):
    st, sc = C.c_size_t(0), C.c_size_t(0)
    n = len(descs) if descs is not None else 0
    _check(_lib.br_workspace_bytes(descs, n, C.byref(hp) if hp is not None else None, C.byref(st), C.byref(sc)),
           "br_workspace_bytes")
    return st.value, sc.value


def br_init(descs, hp: br_hparams, dev_workspace: int, workspace_bytes: int, hip_stream: int = 0):
    ctx = _ctx_p()
    n = len(descs) if descs is not None else 0
    _check(_lib.br_init(C.byref(ctx), descs, n, C.byref(hp) if hp is not None else None,
                        C.c_void_p(dev_workspace or None), workspace_bytes, C.c_void_p(hip_stream or None)),
           "br_init")
    return ctx


def br_accumulate_stats(ctx, grads: Sequence[int]):
    _check(_lib.br_accumulate_stats(ctx, _ptr_array(grads), len(grads)), "br_accumulate_stats", ctx)


def br_clip_gradients(ctx, grads: Sequence[int], max_norm: float):
    _check(_lib.br_clip_gradients(ctx, _ptr_array(grads), len(grads), max_norm), "br_clip_gradients", ctx)


def br_clip_gradients_static(descs, grads: Sequence[int], max_norm: float, dev_result: int, hip_stream: int = 0):
    n = len(descs) if descs is not None else 0
    _check(_lib.br_clip_gradients_static(descs, _ptr_array(grads), n, max_norm, C.c_void_p(dev_result or None),
                                         C.c_void_p(hip_stream or None)), "br_clip_gradients_static")


def br_delay_compensate(ctx, grads: Sequence[int], params_now: Sequence[int], params_stale: Sequence[int], lam: float):
    _check(_lib.br_delay_compensate(ctx, _ptr_array(grads), _ptr_array(params_now), _ptr_array(params_stale), len(grads), lam),
           "br_delay_compensate", ctx)


def br_get_clip_result(ctx) -> int:
    p = C.c_void_p()
    _check(_lib.br_get_clip_result(ctx, C.byref(p)), "br_get_clip_result", ctx)
    return p.value


def br_refresh_basis(ctx):
    _check(_lib.br_refresh_basis(ctx), "br_refresh_basis", ctx)


def br_step(ctx, params: Sequence[int], grads: Sequence[int], lr: float):
    if len(params) != len(grads):
        raise BrError(BR_ERR_SHAPE, "br_step", "params and grads differ in length")
    _check(_lib.br_step(ctx, _ptr_array(params), _ptr_array(grads), len(grads), lr), "br_step", ctx)


def br_get_state(ctx, mat: int, which: int):
    """Returns (device pointer, rows, cols)."""
    p, r, c = C.c_void_p(), C.c_int64(), C.c_int64()
    _check(_lib.br_get_state(ctx, mat, which, C.byref(p), C.byref(r), C.byref(c)), "br_get_state", ctx)
    return p.value, r.value, c.value


BR_HEALTH_QR_GAVE_UP, BR_HEALTH_NONFINITE_WEIGHT, BR_HEALTH_WORDS = 0, 1, 4


def br_get_health(ctx) -> int:
    """Device pointer to the BR_HEALTH_WORDS int32 health counters (no synchronisation)."""
    p = C.c_void_p()
    _check(_lib.br_get_health(ctx, C.byref(p)), "br_get_health", ctx)
    return p.value


def br_check_health(ctx):
    """Synchronises; returns the four counters, raises BrError(BR_ERR_STATE) when any is non-zero."""
    counts = (C.c_int32 * BR_HEALTH_WORDS)()
    _check(_lib.br_check_health(ctx, counts), "br_check_health", ctx)
    return list(counts)


def br_set_qr_wait_limit(ctx, polls: int):
    _check(_lib.br_set_qr_wait_limit(ctx, polls), "br_set_qr_wait_limit", ctx)


def br_notify_state_written(ctx):
    _check(_lib.br_notify_state_written(ctx), "br_notify_state_written", ctx)


def br_get_step_count(ctx) -> int:
    t = C.c_int64()
    _check(_lib.br_get_step_count(ctx, C.byref(t)), "br_get_step_count", ctx)
    return t.value


def br_set_step_count(ctx, t: int):
    _check(_lib.br_set_step_count(ctx, t), "br_set_step_count", ctx)


def br_profile_begin(ctx):
    _check(_lib.br_profile_begin(ctx), "br_profile_begin", ctx)


def br_profile_end(ctx, cap: int = 64):
    out = (br_profile_entry * cap)()
    n = C.c_int32(0)
    _check(_lib.br_profile_end(ctx, out, cap, C.byref(n)), "br_profile_end", ctx)
    return [dict(kernel=out[i].kernel.decode(), launches=out[i].launches, ms=out[i].ms, flops=out[i].flops,
                 bytes=out[i].bytes) for i in range(n.value)]


def br_destroy(ctx):
    _lib.br_destroy(ctx)
