"""ctypes binding of ``libjigsaw.so`` (declared in ``include/jigsaw.h``).

Argument marshalling only: every step of the layer runs in the library's HIP
kernels.  The functions carry the C names.  Device pointers are plain integers
(e.g. ``torch.Tensor.data_ptr()``); shard arguments are sequences of ``ways``
such integers.  A negative status raises :class:`JigsawError`.

There is no CPU fallback: importing this module fails if the library has not
been built (``python -m paper_2507_05753_amd.build`` or ``__graft_entry__.build()``).
"""
from __future__ import annotations

import ctypes
import os

import torch  # noqa: F401  imported first so that the library binds to the HIP runtime torch loaded

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libjigsaw.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build the HIP library first "
        "(python paper_2507_05753_amd/build.py); there is no CPU fallback")

_lib = ctypes.CDLL(LIB_PATH)

# ---- constants (mirror include/jigsaw.h) ------------------------------------
JG_OK = 0
JG_E_NULL, JG_E_SHAPE, JG_E_WAYS, JG_E_DTYPE = -1, -2, -3, -4
JG_E_WORKSPACE, JG_E_ALIGN, JG_E_HIP, JG_E_ARCH = -5, -6, -7, -8
JG_OP_XWT, JG_OP_XTW, JG_OP_XW = 0, 1, 2
JG_F32, JG_BF16, JG_BF16X3 = 0, 1, 2
JG_COMBINE_FUSED, JG_COMBINE_SEPARATE = 0, 1
JG_WEIGHTS_COPY, JG_WEIGHTS_DIRECT = 0, 1
JG_TAIL_SPLIT, JG_TAIL_WHOLE = 0, 1
JG_ACC_LEVELS, JG_ACC_SINGLE = 0, 1
JG_STATIC_WORKSPACE_BYTES = 64 << 20
JG_ACT_NONE, JG_ACT_GELU = 0, 1
JG_T_X, JG_T_W, JG_T_B, JG_T_Y, JG_T_X_F32, JG_T_W_F32 = 0, 1, 2, 3, 4, 5
(JG_Q_WORKSPACE_BYTES, JG_Q_FLOPS_TOTAL, JG_Q_FLOPS_RANK, JG_Q_HBM_BYTES_ALGO,
 JG_Q_EXCHANGE_BYTES_RANK, JG_Q_X_ROWS, JG_Q_X_COLS, JG_Q_W_ROWS, JG_Q_W_COLS,
 JG_Q_Y_ROWS, JG_Q_Y_COLS, JG_Q_B_LEN, JG_Q_RESIDENT_BYTES_RANK, JG_Q_GEMM_LAUNCHES,
 JG_Q_BACKWARD_WORKSPACE_BYTES, JG_Q_BACKWARD_FLOPS_TOTAL, JG_Q_BACKWARD_GEMM_LAUNCHES,
 JG_Q_TAIL_SCRATCH_BYTES, JG_Q_BACKWARD_TAIL_SCRATCH_BYTES, JG_Q_X_SHARD_BYTES, JG_Q_W_SHARD_BYTES,
 JG_Q_CHAIN_WORKSPACE_BYTES, JG_Q_X_F32_SHARDS_BYTES, JG_Q_NORM_BACKWARD_WORKSPACE_BYTES,
 JG_Q_BIAS_BACKWARD_WORKSPACE_BYTES) = range(25)
(JG_KERNEL_GEMM, JG_KERNEL_WEIGHT_COPY, JG_KERNEL_COMBINE, JG_KERNEL_SHARD,
 JG_KERNEL_GATHER, JG_KERNEL_GEMM_DX, JG_KERNEL_GEMM_DW, JG_KERNEL_JOIN, JG_KERNEL_NORM, JG_KERNEL_REDUCE,
 JG_KERNEL_COUNT) = range(11)

EXPORTS = ("jg_init", "jg_free", "jg_plan_create", "jg_plan_destroy", "jg_plan_query", "jg_shard",
           "jg_shard_patches", "jg_gather_patches",
           "jg_linear_forward", "jg_linear_forward_ex", "jg_linear_forward_static", "jg_mlp_forward", "jg_layernorm_forward",
           "jg_mixing_forward", "jg_token_mixing_forward", "jg_linear_backward", "jg_bias_backward", "jg_layernorm_backward", "jg_mlp_backward", "jg_mixing_backward", "jg_token_mixing_backward", "jg_gather", "jg_gather_as", "jg_profile",
           "jg_profile_read", "jg_strerror",
           "jg_last_hip_error")


class jg_linear_desc(ctypes.Structure):
    _fields_ = [("M", ctypes.c_int64), ("K", ctypes.c_int64), ("N", ctypes.c_int64),
                ("ways", ctypes.c_int32), ("op", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("has_bias", ctypes.c_int32), ("combine", ctypes.c_int32), ("weights", ctypes.c_int32),
                ("tail", ctypes.c_int32), ("accumulate", ctypes.c_int32)]


class JigsawError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = f"{where}: {_lib.jg_strerror(status).decode()} ({status})"
        if status == JG_E_HIP:
            msg += f" [{_lib.jg_last_hip_error().decode()}]"
        super().__init__(msg)


_vp = ctypes.c_void_p
_vpp = ctypes.POINTER(ctypes.c_void_p)
_lib.jg_strerror.argtypes = [ctypes.c_int]
_lib.jg_strerror.restype = ctypes.c_char_p
_lib.jg_last_hip_error.argtypes = []
_lib.jg_last_hip_error.restype = ctypes.c_char_p
_lib.jg_init.argtypes = [_vpp, ctypes.c_int, _vp]
_lib.jg_free.argtypes = [_vp]
_lib.jg_free.restype = None
_lib.jg_plan_create.argtypes = [_vp, ctypes.POINTER(jg_linear_desc), _vpp]
_lib.jg_plan_destroy.argtypes = [_vp]
_lib.jg_plan_destroy.restype = None
_lib.jg_plan_query.argtypes = [_vp, ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_int64)]
_lib.jg_shard.argtypes = [_vp, ctypes.c_int, _vp, ctypes.c_int64, _vpp]
_lib.jg_shard_patches.argtypes = [_vp, _vp, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, _vpp]
_lib.jg_gather_patches.argtypes = [_vp, _vpp, _vp, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64]
_lib.jg_shard_patches.restype = ctypes.c_int
_lib.jg_gather_patches.restype = ctypes.c_int
_lib.jg_linear_forward.argtypes = [_vp, _vpp, _vpp, _vpp, _vpp, _vp, ctypes.c_size_t]
_lib.jg_linear_forward_static.argtypes = [_vp, _vpp, _vpp, _vpp, _vpp]
_lib.jg_linear_forward_static.restype = ctypes.c_int
_lib.jg_linear_forward_ex.argtypes = [_vp, _vpp, _vpp, _vpp, _vpp, ctypes.c_int, _vpp, _vp, ctypes.c_size_t]
_lib.jg_mlp_forward.argtypes = [_vp, _vp, _vpp, _vpp, _vpp, _vpp, _vpp, _vpp, _vpp, _vp, ctypes.c_size_t]
_lib.jg_layernorm_forward.argtypes = [_vp, _vpp, _vp, _vp, ctypes.c_double, _vpp]
_lib.jg_mixing_forward.argtypes = [_vp, _vp, _vpp, _vp, _vp, ctypes.c_double, _vpp, _vpp, _vpp, _vpp, _vpp, _vpp, _vpp,
                                   _vp, ctypes.c_size_t]
_lib.jg_token_mixing_forward.argtypes = [_vp, _vp, _vpp, _vp, _vp, ctypes.c_double, _vpp, _vpp, _vpp, _vp, _vpp, _vpp,
                                         _vpp, _vp, ctypes.c_size_t]
_lib.jg_linear_backward.argtypes = [_vp, _vpp, _vpp, _vpp, _vpp, _vpp, _vp, ctypes.c_size_t]
_lib.jg_layernorm_backward.argtypes = [_vp, _vpp, _vp, ctypes.c_double, _vpp, _vpp, _vp, _vp, _vp, ctypes.c_size_t]
_lib.jg_layernorm_backward.restype = ctypes.c_int
_lib.jg_mlp_backward.argtypes = [_vp, _vp] + [_vpp] * 14 + [_vp, ctypes.c_size_t]
_lib.jg_mlp_backward.restype = ctypes.c_int
_lib.jg_mixing_backward.argtypes = ([_vp, _vp, _vpp, _vp, ctypes.c_double] + [_vpp] * 15 +
                                    [_vp, _vp, _vp, ctypes.c_size_t])
_lib.jg_mixing_backward.restype = ctypes.c_int
_lib.jg_token_mixing_backward.argtypes = ([_vp, _vp, _vpp, _vp, ctypes.c_double] + [_vpp] * 14 +
                                          [_vp, _vp, _vp, _vp, ctypes.c_size_t])
_lib.jg_token_mixing_backward.restype = ctypes.c_int
_lib.jg_bias_backward.argtypes = [_vp, _vpp, _vpp, _vp, ctypes.c_size_t]
_lib.jg_bias_backward.restype = ctypes.c_int
_lib.jg_gather.argtypes = [_vp, _vpp, _vp, ctypes.c_int64]
_lib.jg_gather_as.argtypes = [_vp, ctypes.c_int, _vpp, _vp, ctypes.c_int64]
_lib.jg_profile.argtypes = [_vp, ctypes.c_int]
_lib.jg_profile_read.argtypes = [_vp, ctypes.c_int, ctypes.POINTER(ctypes.c_double),
                                 ctypes.POINTER(ctypes.c_int64)]
for _n in ("jg_init", "jg_plan_create", "jg_plan_query", "jg_shard", "jg_linear_forward", "jg_linear_forward_ex",
           "jg_mlp_forward", "jg_layernorm_forward", "jg_mixing_forward", "jg_token_mixing_forward",
           "jg_linear_backward", "jg_gather", "jg_gather_as", "jg_profile", "jg_profile_read"):
    getattr(_lib, _n).restype = ctypes.c_int


def _ptr_array(ptrs):
    if ptrs is None or isinstance(ptrs, _vpp):
        return ptrs
    arr = (ctypes.c_void_p * len(ptrs))(*[int(p) if p else None for p in ptrs])
    out = ctypes.cast(arr, _vpp)
    out._keep = arr         # the array lives as long as the pointer to it
    return out


def ptr_array(ptrs):
    """A host array of device pointers, marshalled once: every shard argument accepts the result in place of a
    sequence, which saves the conversion in a loop that passes the same buffers again and again."""
    return _ptr_array(ptrs)


def _raise(status: int, where: str):
    if status != JG_OK:
        raise JigsawError(status, where)


def jg_strerror(status: int) -> str:
    return _lib.jg_strerror(status).decode()


def jg_last_hip_error() -> str:
    return _lib.jg_last_hip_error().decode()


def jg_init(device: int = 0, hip_stream: int | None = None) -> int:
    out = ctypes.c_void_p()
    _raise(_lib.jg_init(ctypes.byref(out), device, hip_stream or None), "jg_init")
    return out.value


def jg_free(ctx) -> None:
    _lib.jg_free(ctx)


def jg_plan_create(ctx, M: int, K: int, N: int, ways: int, has_bias: bool = False,
                   combine: int = JG_COMBINE_FUSED, weights: int = JG_WEIGHTS_COPY,
                   op: int = JG_OP_XWT, dtype: int = JG_F32, tail: int = JG_TAIL_SPLIT,
                   accumulate: int = JG_ACC_LEVELS) -> int:
    d = jg_linear_desc(M, K, N, ways, op, dtype, int(has_bias), combine, weights, tail, accumulate)
    out = ctypes.c_void_p()
    _raise(_lib.jg_plan_create(ctx, ctypes.byref(d), ctypes.byref(out)), "jg_plan_create")
    return out.value


def jg_plan_destroy(plan) -> None:
    _lib.jg_plan_destroy(plan)


def jg_plan_query(plan, what: int, rank: int = 0) -> int:
    out = ctypes.c_int64()
    _raise(_lib.jg_plan_query(plan, what, rank, ctypes.byref(out)), "jg_plan_query")
    return out.value


def jg_shard(plan, which: int, global_ptr: int, ld: int, shard_ptrs) -> None:
    _raise(_lib.jg_shard(plan, which, global_ptr, ld, _ptr_array(shard_ptrs)), "jg_shard")


def jg_shard_patches(plan, field_ptr: int, C: int, H: int, W: int, p: int, x_ptrs) -> None:
    _raise(_lib.jg_shard_patches(plan, field_ptr, C, H, W, p, _ptr_array(x_ptrs)), "jg_shard_patches")


def jg_gather_patches(plan, y_ptrs, field_ptr: int, C: int, H: int, W: int, p: int) -> None:
    _raise(_lib.jg_gather_patches(plan, _ptr_array(y_ptrs), field_ptr, C, H, W, p), "jg_gather_patches")


def jg_linear_forward(plan, x_ptrs, w_ptrs, b_ptrs, y_ptrs, workspace_ptr, workspace_bytes: int) -> None:
    _raise(_lib.jg_linear_forward(plan, _ptr_array(x_ptrs), _ptr_array(w_ptrs), _ptr_array(b_ptrs),
                                  _ptr_array(y_ptrs), workspace_ptr or None, workspace_bytes),
           "jg_linear_forward")


def jg_linear_forward_static(plan, x_ptrs, w_ptrs, b_ptrs, y_ptrs) -> None:
    _raise(_lib.jg_linear_forward_static(plan, _ptr_array(x_ptrs), _ptr_array(w_ptrs), _ptr_array(b_ptrs),
                                         _ptr_array(y_ptrs)), "jg_linear_forward_static")


def jg_linear_forward_ex(plan, x_ptrs, w_ptrs, b_ptrs, r_ptrs, activation: int, y_ptrs, workspace_ptr,
                         workspace_bytes: int) -> None:
    _raise(_lib.jg_linear_forward_ex(plan, _ptr_array(x_ptrs), _ptr_array(w_ptrs), _ptr_array(b_ptrs),
                                     _ptr_array(r_ptrs), activation, _ptr_array(y_ptrs), workspace_ptr or None,
                                     workspace_bytes), "jg_linear_forward_ex")


def jg_mlp_forward(first, second, x_ptrs, w1_ptrs, b1_ptrs, w2_ptrs, b2_ptrs, h_ptrs, y_ptrs, workspace_ptr,
                   workspace_bytes: int) -> None:
    _raise(_lib.jg_mlp_forward(first, second, _ptr_array(x_ptrs), _ptr_array(w1_ptrs), _ptr_array(b1_ptrs),
                               _ptr_array(w2_ptrs), _ptr_array(b2_ptrs), _ptr_array(h_ptrs), _ptr_array(y_ptrs),
                               workspace_ptr or None, workspace_bytes), "jg_mlp_forward")


def jg_layernorm_forward(plan, x_ptrs, gamma_ptr, beta_ptr, eps: float, out_ptrs) -> None:
    _raise(_lib.jg_layernorm_forward(plan, _ptr_array(x_ptrs), gamma_ptr or None, beta_ptr or None, float(eps),
                                     _ptr_array(out_ptrs)), "jg_layernorm_forward")


def jg_mixing_forward(first, second, x_ptrs, gamma_ptr, beta_ptr, eps: float, w1_ptrs, b1_ptrs, w2_ptrs, b2_ptrs,
                      xn_ptrs, h_ptrs, y_ptrs, workspace_ptr, workspace_bytes: int) -> None:
    _raise(_lib.jg_mixing_forward(first, second, _ptr_array(x_ptrs), gamma_ptr or None, beta_ptr or None, float(eps),
                                  _ptr_array(w1_ptrs), _ptr_array(b1_ptrs), _ptr_array(w2_ptrs), _ptr_array(b2_ptrs),
                                  _ptr_array(xn_ptrs), _ptr_array(h_ptrs), _ptr_array(y_ptrs),
                                  workspace_ptr or None, workspace_bytes), "jg_mixing_forward")


def jg_token_mixing_forward(first, second, x_ptrs, gamma_ptr, beta_ptr, eps: float, w1_ptrs, b1_ptrs, w2_ptrs, b2_ptr,
                            xn_ptrs, h_ptrs, y_ptrs, workspace_ptr, workspace_bytes: int) -> None:
    _raise(_lib.jg_token_mixing_forward(first, second, _ptr_array(x_ptrs), gamma_ptr or None, beta_ptr or None,
                                        float(eps), _ptr_array(w1_ptrs), _ptr_array(b1_ptrs), _ptr_array(w2_ptrs),
                                        b2_ptr or None, _ptr_array(xn_ptrs), _ptr_array(h_ptrs), _ptr_array(y_ptrs),
                                        workspace_ptr or None, workspace_bytes), "jg_token_mixing_forward")


def jg_linear_backward(plan, x_ptrs, w_ptrs, dy_ptrs, dx_ptrs, dw_ptrs, workspace_ptr, workspace_bytes: int) -> None:
    _raise(_lib.jg_linear_backward(plan, _ptr_array(x_ptrs), _ptr_array(w_ptrs), _ptr_array(dy_ptrs),
                                   _ptr_array(dx_ptrs), _ptr_array(dw_ptrs), workspace_ptr or None,
                                   workspace_bytes), "jg_linear_backward")


def jg_layernorm_backward(plan, x_ptrs, gamma_ptr, eps: float, dy_ptrs, dx_ptrs, dgamma_ptr, dbeta_ptr, workspace_ptr,
                          workspace_bytes: int) -> None:
    _raise(_lib.jg_layernorm_backward(plan, _ptr_array(x_ptrs), gamma_ptr or None, float(eps), _ptr_array(dy_ptrs),
                                      _ptr_array(dx_ptrs), dgamma_ptr or None, dbeta_ptr or None,
                                      workspace_ptr or None, workspace_bytes), "jg_layernorm_backward")


def jg_mlp_backward(first, second, x_ptrs, w1_ptrs, b1_ptrs, w2_ptrs, h_ptrs, dy_ptrs, a_ptrs, dh_ptrs, da_ptrs, dx_ptrs,
                    dw1_ptrs, db1_ptrs, dw2_ptrs, db2_ptrs, workspace_ptr, workspace_bytes: int) -> None:
    arrays = [_ptr_array(v) for v in (x_ptrs, w1_ptrs, b1_ptrs, w2_ptrs, h_ptrs, dy_ptrs, a_ptrs, dh_ptrs, da_ptrs, dx_ptrs,
                                      dw1_ptrs, db1_ptrs, dw2_ptrs, db2_ptrs)]
    _raise(_lib.jg_mlp_backward(first, second, *arrays, workspace_ptr or None, workspace_bytes), "jg_mlp_backward")


def jg_mixing_backward(first, second, x_ptrs, gamma_ptr, eps: float, xn_ptrs, w1_ptrs, b1_ptrs, w2_ptrs, h_ptrs, dy_ptrs,
                       a_ptrs, dh_ptrs, da_ptrs, dxn_ptrs, dx_ptrs, dw1_ptrs, db1_ptrs, dw2_ptrs, db2_ptrs, dgamma_ptr,
                       dbeta_ptr, workspace_ptr, workspace_bytes: int) -> None:
    arrays = [_ptr_array(v) for v in (xn_ptrs, w1_ptrs, b1_ptrs, w2_ptrs, h_ptrs, dy_ptrs, a_ptrs, dh_ptrs, da_ptrs,
                                      dxn_ptrs, dx_ptrs, dw1_ptrs, db1_ptrs, dw2_ptrs, db2_ptrs)]
    _raise(_lib.jg_mixing_backward(first, second, _ptr_array(x_ptrs), gamma_ptr or None, float(eps), *arrays,
                                   dgamma_ptr or None, dbeta_ptr or None, workspace_ptr or None, workspace_bytes),
           "jg_mixing_backward")


def jg_token_mixing_backward(first, second, x_ptrs, gamma_ptr, eps: float, xn_ptrs, w1_ptrs, b1_ptrs, w2_ptrs, h_ptrs,
                             dy_ptrs, a_ptrs, dh_ptrs, da_ptrs, dxn_ptrs, dx_ptrs, dw1_ptrs, db1_ptrs, dw2_ptrs, db2_ptr,
                             dgamma_ptr, dbeta_ptr, workspace_ptr, workspace_bytes: int) -> None:
    arrays = [_ptr_array(v) for v in (xn_ptrs, w1_ptrs, b1_ptrs, w2_ptrs, h_ptrs, dy_ptrs, a_ptrs, dh_ptrs, da_ptrs,
                                      dxn_ptrs, dx_ptrs, dw1_ptrs, db1_ptrs, dw2_ptrs)]
    _raise(_lib.jg_token_mixing_backward(first, second, _ptr_array(x_ptrs), gamma_ptr or None, float(eps), *arrays,
                                         db2_ptr or None, dgamma_ptr or None, dbeta_ptr or None, workspace_ptr or None,
                                         workspace_bytes), "jg_token_mixing_backward")


def jg_bias_backward(plan, dy_ptrs, db_ptrs, workspace_ptr=None, workspace_bytes: int = 0) -> None:
    _raise(_lib.jg_bias_backward(plan, _ptr_array(dy_ptrs), _ptr_array(db_ptrs), workspace_ptr or None, workspace_bytes),
           "jg_bias_backward")


def jg_gather(plan, y_ptrs, global_y_ptr: int, ld: int) -> None:
    _raise(_lib.jg_gather(plan, _ptr_array(y_ptrs), global_y_ptr, ld), "jg_gather")


def jg_gather_as(plan, which: int, shard_ptrs, global_ptr: int, ld: int) -> None:
    _raise(_lib.jg_gather_as(plan, which, _ptr_array(shard_ptrs), global_ptr, ld), "jg_gather_as")


def jg_profile(ctx, enable: bool) -> None:
    _raise(_lib.jg_profile(ctx, int(enable)), "jg_profile")


def jg_profile_read(ctx, kernel: int):
    ms = ctypes.c_double()
    n = ctypes.c_int64()
    _raise(_lib.jg_profile_read(ctx, kernel, ctypes.byref(ms), ctypes.byref(n)), "jg_profile_read")
    return ms.value, n.value


def raw():
    """The loaded ``ctypes.CDLL`` (for tests that drive the C ABI with hand-made arguments)."""
    return _lib
