"""ctypes binding of include/adapm.h: argument marshalling only.

Every step of the optimizer runs inside libadapm.so (hand-written HIP for gfx950).
There is no Python or CPU fallback: if the library has not been built, importing
this module raises.  PyTorch is used by callers for device memory and streams only.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

# PyTorch ships its own HIP runtime.  It must be the one already loaded when libadapm.so
# is opened, so that the library, the tensors and the streams share a single runtime.
import torch  # noqa: F401

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libadapm.so")

ADAPM_OK, ADAPM_EINVAL, ADAPM_ENOMEM, ADAPM_EHIP, ADAPM_ESTATE = 0, -1, -2, -3, -4
ADAPM_F32, ADAPM_BF16 = 0, 1
ADAPM_MOM_NONE, ADAPM_MOM_FULL, ADAPM_MOM_LOWRANK = 0, 1, 2
ADAPM_V_ELEMENT, ADAPM_V_ROWGROUP, ADAPM_V_WHOLE = 0, 1, 2
ADAPM_CONTRACT_AUTO, ADAPM_CONTRACT_F64, ADAPM_CONTRACT_BF16X2 = 0, 1, 2


class adapm_block_t(C.Structure):
    _fields_ = [("rows", C.c_int64), ("cols", C.c_int64),
                ("param_dtype", C.c_int32), ("grad_dtype", C.c_int32),
                ("mom_mode", C.c_int32), ("rank", C.c_int32),
                ("v_mode", C.c_int32), ("v_group_rows", C.c_int32),
                ("lr_scale", C.c_float), ("weight_decay", C.c_float)]


class adapm_hparams_t(C.Structure):
    _fields_ = [("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float), ("clip", C.c_float),
                ("adam_debias", C.c_int32), ("refresh_iters_K", C.c_int32),
                ("refresh_period_T", C.c_int32), ("bias_correction", C.c_int32),
                ("contraction", C.c_int32), ("refresh_normalise", C.c_int32),
                ("seed", C.c_uint64)]


EXPORTS = ["adapm_init", "adapm_state_bytes", "adapm_workspace_bytes", "adapm_state_offsets",
           "adapm_state_init", "adapm_state_loaded", "adapm_step", "adapm_block_contraction", "adapm_last_launch_count",
           "adapm_algorithmic_bytes",
           "adapm_algorithmic_flops", "adapm_profile_enable", "adapm_profile_read", "adapm_last_error",
           "adapm_set_grad_clip", "adapm_last_grad_norm", "adapm_lr_cosine_warmup", "adapm_destroy",
           "adapm_step_static", "adapm_static_scratch_bytes"]


def _load() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()'). "
            "There is no fallback path.")
    lib = C.CDLL(LIB_PATH)
    P = C.c_void_p
    lib.adapm_init.restype = C.c_int
    lib.adapm_init.argtypes = [C.POINTER(P), C.POINTER(adapm_block_t), C.c_int64, C.POINTER(adapm_hparams_t)]
    lib.adapm_state_bytes.restype = C.c_size_t
    lib.adapm_state_bytes.argtypes = [P]
    lib.adapm_workspace_bytes.restype = C.c_size_t
    lib.adapm_workspace_bytes.argtypes = [P]
    lib.adapm_state_offsets.restype = C.c_int
    lib.adapm_state_offsets.argtypes = [P, C.c_int64] + [C.POINTER(C.c_size_t)] * 4
    lib.adapm_state_init.restype = C.c_int
    lib.adapm_state_init.argtypes = [P, P, P]
    lib.adapm_set_grad_clip.restype = C.c_int
    lib.adapm_set_grad_clip.argtypes = [P, C.c_float]
    lib.adapm_last_grad_norm.restype = C.c_int
    lib.adapm_last_grad_norm.argtypes = [P, P, P, C.POINTER(C.c_float), C.POINTER(C.c_float)]
    lib.adapm_lr_cosine_warmup.restype = C.c_float
    lib.adapm_lr_cosine_warmup.argtypes = [C.c_int64, C.c_float, C.c_float, C.c_int64, C.c_int64]
    lib.adapm_state_loaded.restype = C.c_int
    lib.adapm_state_loaded.argtypes = [P]
    lib.adapm_step.restype = C.c_int
    lib.adapm_step.argtypes = [P, C.POINTER(P), C.POINTER(P), P, P, C.c_int64, C.c_float, P]
    lib.adapm_step_static.restype = C.c_int
    lib.adapm_step_static.argtypes = [P, C.POINTER(P), C.POINTER(P), P, C.c_int64, C.c_float, P]
    lib.adapm_static_scratch_bytes.restype = C.c_size_t
    lib.adapm_static_scratch_bytes.argtypes = []
    lib.adapm_block_contraction.restype = C.c_int32
    lib.adapm_block_contraction.argtypes = [P, C.c_int64]
    lib.adapm_last_launch_count.restype = C.c_int64
    lib.adapm_last_launch_count.argtypes = [P]
    lib.adapm_algorithmic_bytes.restype = C.c_double
    lib.adapm_algorithmic_bytes.argtypes = [P, C.c_int32]
    lib.adapm_algorithmic_flops.restype = C.c_double
    lib.adapm_algorithmic_flops.argtypes = [P, C.c_int32]
    lib.adapm_profile_enable.restype = C.c_int
    lib.adapm_profile_enable.argtypes = [P, C.c_int32]
    lib.adapm_profile_read.restype = C.c_int64
    lib.adapm_profile_read.argtypes = [P, C.c_int64, C.c_char_p, C.c_size_t, C.POINTER(C.c_double),
                                       C.POINTER(C.c_int64)]
    lib.adapm_last_error.restype = C.c_char_p
    lib.adapm_last_error.argtypes = []
    lib.adapm_destroy.restype = None
    lib.adapm_destroy.argtypes = [P]
    return lib


lib = _load()


class AdapmError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        super().__init__(f"adapm status {status}: {adapm_last_error()}")


def adapm_last_error() -> str:
    return lib.adapm_last_error().decode()


def _check(st: int):
    if st != ADAPM_OK:
        raise AdapmError(st)


def adapm_init(table: Sequence[adapm_block_t], hp: adapm_hparams_t) -> C.c_void_p:
    arr = (adapm_block_t * max(len(table), 1))(*table)
    ctx = C.c_void_p()
    _check(lib.adapm_init(C.byref(ctx), arr, len(table), C.byref(hp)))
    return ctx


def adapm_state_bytes(ctx) -> int:
    return lib.adapm_state_bytes(ctx)


def adapm_workspace_bytes(ctx) -> int:
    return lib.adapm_workspace_bytes(ctx)


def adapm_state_offsets(ctx, block: int):
    """(L, R, m, v) byte offsets; None for an absent sub-buffer."""
    o = [C.c_size_t() for _ in range(4)]
    _check(lib.adapm_state_offsets(ctx, block, *[C.byref(x) for x in o]))
    absent = C.c_size_t(-1).value
    return tuple(None if x.value == absent else x.value for x in o)


def adapm_state_init(ctx, state_ptr: int, stream: int = 0):
    _check(lib.adapm_state_init(ctx, C.c_void_p(state_ptr), C.c_void_p(stream)))


def adapm_state_loaded(ctx):
    _check(lib.adapm_state_loaded(ctx))


def adapm_step(ctx, params_ptrs, grads_ptrs, state_ptr: int, workspace_ptr: int, step: int, lr: float,
               stream: int = 0):
    """params_ptrs / grads_ptrs: ctypes arrays of c_void_p (see ptr_array)."""
    _check(lib.adapm_step(ctx, params_ptrs, grads_ptrs, C.c_void_p(state_ptr), C.c_void_p(workspace_ptr),
                          step, lr, C.c_void_p(stream)))


def adapm_step_static(ctx, params_ptrs, grads_ptrs, state_ptr: int, step: int, lr: float, stream: int = 0):
    """adapm_step on the library's own scratch array (allocates nothing)."""
    _check(lib.adapm_step_static(ctx, params_ptrs, grads_ptrs, C.c_void_p(state_ptr), step, lr, C.c_void_p(stream)))


def adapm_static_scratch_bytes() -> int:
    return lib.adapm_static_scratch_bytes()


def adapm_block_contraction(ctx, block: int) -> int:
    return lib.adapm_block_contraction(ctx, block)


def adapm_last_launch_count(ctx) -> int:
    return lib.adapm_last_launch_count(ctx)


def adapm_algorithmic_bytes(ctx, refresh_step: bool) -> float:
    return lib.adapm_algorithmic_bytes(ctx, 1 if refresh_step else 0)


def adapm_algorithmic_flops(ctx, refresh_step: bool) -> float:
    return lib.adapm_algorithmic_flops(ctx, 1 if refresh_step else 0)


def adapm_set_grad_clip(ctx, max_norm: float):
    _check(lib.adapm_set_grad_clip(ctx, C.c_float(max_norm)))


def adapm_last_grad_norm(ctx, workspace_ptr: int, stream: int = 0):
    """(norm, factor) of the last clipped step; synchronises the stream."""
    norm, scale = C.c_float(), C.c_float()
    _check(lib.adapm_last_grad_norm(ctx, C.c_void_p(workspace_ptr), C.c_void_p(stream), C.byref(norm), C.byref(scale)))
    return norm.value, scale.value


def adapm_lr_cosine_warmup(step: int, peak_lr: float, min_lr: float, warmup_steps: int, total_steps: int) -> float:
    return float(lib.adapm_lr_cosine_warmup(step, peak_lr, min_lr, warmup_steps, total_steps))


def adapm_profile_enable(ctx, on: bool):
    _check(lib.adapm_profile_enable(ctx, 1 if on else 0))


def adapm_profile_read(ctx):
    """{label: (total_ms, launches)} accumulated since the last read; synchronise the stream first."""
    out = {}
    name = C.create_string_buffer(64)
    ms, cnt = C.c_double(), C.c_int64()
    n = lib.adapm_profile_read(ctx, 0, name, 64, C.byref(ms), C.byref(cnt))
    for i in range(n):
        if i:
            lib.adapm_profile_read(ctx, i, name, 64, C.byref(ms), C.byref(cnt))
        out[name.value.decode()] = (ms.value, cnt.value)
    return out


def adapm_destroy(ctx):
    lib.adapm_destroy(ctx)


def ptr_array(ptrs: Sequence[int]):
    return (C.c_void_p * max(len(ptrs), 1))(*ptrs)
