"""ctypes binding of liblga.so: same names as include/lga.h and include/lga_ops.h.

Argument marshalling only - every step of the path runs in the library's HIP kernels.
PyTorch is used by callers for device memory and streams; tensors cross this boundary as raw
device pointers (`tensor.data_ptr()`).  There is no CPU fallback: if the library has not been
built, importing this module raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

# PyTorch ships its own HIP runtime (soname libamdhip64.so.7).  Importing it first makes the
# loader bind liblga.so to that same runtime, so the process holds ONE runtime and pointers from
# torch allocations are known to the runtime that launches this library's kernels.
import torch  # noqa: F401  (device memory and streams for the callers)

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblga.so")

LGA_FP32, LGA_BF16, LGA_FP16 = 0, 1, 2
LGA_OK, LGA_ERR_ARG, LGA_ERR_SHAPE, LGA_ERR_OOM, LGA_ERR_STATE, LGA_ERR_HIP = 0, -1, -2, -3, -4, -5
LGA_OVERLAP_NONE, LGA_OVERLAP_RESTORE, LGA_OVERLAP_ADAM = 0, 1, 2
LGA_ATTN_CAUSAL, LGA_ATTN_FULL = 0, 1
LGA_ORDER_LAYERED, LGA_ORDER_MICROBATCH_MAJOR = 0, 1
(LGA_EPI_STORE, LGA_EPI_BIAS, LGA_EPI_BIAS_RESID, LGA_EPI_BIAS_GELU, LGA_EPI_MUL_DGELU,
 LGA_EPI_ACCUM_F32) = range(6)

_STATUS_NAMES = {0: "LGA_OK", -1: "LGA_ERR_ARG", -2: "LGA_ERR_SHAPE", -3: "LGA_ERR_OOM", -4: "LGA_ERR_STATE",
                 -5: "LGA_ERR_HIP"}


class lga_config(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_heads", C.c_int32), ("d_ff", C.c_int32),
                ("seq_len", C.c_int32), ("micro_batch", C.c_int32), ("n_micro", C.c_int32), ("dtype", C.c_int32),
                ("group", C.c_int32), ("retain_grads", C.c_int32), ("wgrad_groups", C.c_int32), ("param_buffers", C.c_int32),
                ("overlap", C.c_int32), ("attention", C.c_int32), ("offload_checkpoints", C.c_int32),
                ("ln_eps", C.c_float),
                ("stream", C.c_void_p)]


class lga_adam(C.Structure):
    _fields_ = [("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float),
                ("step", C.c_int32), ("loss_scale", C.c_float), ("skip_nonfinite", C.c_int32)]


class lga_loss_scaler(C.Structure):
    _fields_ = [("scale", C.c_float), ("growth", C.c_float), ("backoff", C.c_float), ("min_scale", C.c_float),
                ("max_scale", C.c_float), ("growth_interval", C.c_int32), ("good_steps", C.c_int32)]


class lga_kernel_stat(C.Structure):
    _fields_ = [("name", C.c_char * 112), ("launches", C.c_uint64), ("ms", C.c_double), ("flops", C.c_double),
                ("bytes", C.c_double)]


class LgaError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"{_STATUS_NAMES.get(code, code)}: {message}")
        self.code = code


if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2106_02679_amd.build` "
                      "(there is no fallback path)")

lib = C.CDLL(LIB_PATH)

_vp, _i32, _u64, _f32 = C.c_void_p, C.c_int32, C.c_uint64, C.c_float
_P = C.POINTER

# name -> (restype, argtypes); every symbol include/*.h declares
SIGNATURES = {
    "lga_init_stack": (C.c_int, [_P(lga_config), _vp, _P(_vp)]),
    "lga_destroy_stack": (None, [_vp]),
    "lga_forward_layered": (C.c_int, [_vp, _vp, _vp]),
    "lga_backward_layered": (C.c_int, [_vp, _vp, _vp, _P(lga_adam)]),
    "lga_adam_step_layer": (C.c_int, [_vp, _i32, _P(lga_adam)]),
    "lga_grads": (C.c_int, [_vp, _i32, _P(_vp), _P(C.c_size_t)]),
    "lga_params": (C.c_int, [_vp, _i32, _P(_vp), _P(C.c_size_t)]),
    "lga_moments": (C.c_int, [_vp, _i32, _P(_vp), _P(_vp), _P(C.c_size_t)]),
    "lga_checkpoint": (C.c_int, [_vp, _i32, _P(_vp), _P(C.c_size_t)]),
    "lga_step_mbmajor": (C.c_int, [_vp, _vp, _vp, _vp, _vp, _P(lga_adam)]),
    "lga_forward_layer": (C.c_int, [_vp, _i32, _vp, _vp]),
    "lga_backward_layer": (C.c_int, [_vp, _i32, _vp, _vp, _P(lga_adam)]),
    "lga_traffic_model": (C.c_int, [_P(lga_config), _i32, _P(_u64), _P(_u64), _P(C.c_double)]),
    "lga_arena_bytes": (C.c_int, [_P(lga_config), _P(_u64)]),
    "lga_host_bytes": (C.c_int, [_P(lga_config), _P(_u64)]),
    "lga_restore_count": (C.c_int, [_vp, _P(_u64)]),
    "lga_params_per_layer": (C.c_int, [_P(lga_config), _P(_u64)]),
    "lga_last_error": (C.c_char_p, []),
    "lga_profile_begin": (C.c_int, [_vp]),
    "lga_profile_begin_only": (C.c_int, [_vp, C.c_char_p]),
    "lga_profile_end": (C.c_int, [_vp, _P(lga_kernel_stat), _i32, _P(_i32)]),
    "lga_op_gemm": (C.c_int, [_i32, _i32, _i32, _i32, _i32, _i32, _i32, _vp, _i32, _vp, _i32, _vp, _vp, _vp, _i32,
                              _vp, _vp, _f32, _vp]),
    "lga_op_gemm_splitk": (C.c_int, [_i32, _i32, _i32, _i32, _vp, _i32, _vp, _i32, _vp, _i32, _f32, _vp, _u64, _vp]),
    "lga_op_gemm_splitk_slices": (_i32, [_i32, _i32, _i32]),
    "lga_op_mfma_rate": (C.c_int, [_i32, _i32, _vp, _P(C.c_double), _vp]),
    "lga_op_layernorm_fwd": (C.c_int, [_i32, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _f32, _vp]),
    "lga_op_layernorm_bwd": (C.c_int, [_i32, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _f32, _vp, _i32, _i32,
                                       _vp]),
    "lga_op_layernorm_bwd_scratch_floats": (_u64, [_i32, _i32]),
    "lga_op_transpose": (C.c_int, [_vp, _vp, _i32, _i32, C.c_int64, C.c_int64, _vp]),
    "lga_op_transpose_colsum": (C.c_int, [_i32, _vp, _vp, _i32, _i32, C.c_int64, C.c_int64, _f32, _vp, _vp, _vp]),
    "lga_op_colsum": (C.c_int, [_i32, _vp, _i32, _i32, _i32, _f32, _vp, _vp, _vp]),
    "lga_op_colsum_scratch_floats": (_u64, [_i32, _i32]),
    "lga_op_colsum_static": (C.c_int, [_i32, _vp, _i32, _i32, _i32, _f32, _vp, _vp]),
    "lga_op_colsum_static_max_floats": (_u64, []),
    "lga_op_attention_fwd": (C.c_int, [_i32, _i32, _vp, _vp, _vp, _i32, _i32, _i32, _i32, _i32, _vp]),
    "lga_op_attention_bwd": (C.c_int, [_i32, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _i32, _i32, _i32, _vp]),
    "lga_op_attention_gemm_workspace_bytes": (_u64, [_i32, _i32]),
    "lga_op_attention_gemm_fwd": (C.c_int, [_i32, _vp, _vp, _vp, _i32, _i32, _i32, _i32, _i32, _vp, _u64, _vp]),
    "lga_op_attention_gemm_bwd": (C.c_int, [_i32, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _i32, _i32, _i32, _vp, _u64,
                                            _vp]),
    "lga_op_adam": (C.c_int, [_vp, _vp, _vp, _vp, _vp, _i32, _u64, _P(lga_adam), _vp, _vp]),
    "lga_nonfinite_layers": (C.c_int, [_vp, _P(_i32), _P(_i32)]),
    "lga_grads_nonfinite": (C.c_int, [_vp, _P(_i32), _P(_i32)]),
    "lga_loss_scaler_update": (C.c_int, [_P(lga_loss_scaler), _i32]),
}
for _name, (_res, _args) in SIGNATURES.items():
    _fn = getattr(lib, _name)
    _fn.restype = _res
    _fn.argtypes = _args


_hip = C.CDLL("libamdhip64.so.7")      # already loaded (by torch); resolved by soname
_hip.hipMemcpy.restype = C.c_int
_hip.hipMemcpy.argtypes = [_vp, _vp, C.c_size_t, C.c_int]


def read_device(ptr: int, count: int, dtype="float32"):
    """Blocking copy of `count` elements at device (or pinned host) address `ptr` into a new numpy array.
    Synchronise the stream that produced the data first."""
    import numpy as np
    out = np.empty(count, dtype=dtype)
    rc = _hip.hipMemcpy(out.ctypes.data_as(_vp), ptr, out.nbytes, 4)   # hipMemcpyDefault: the runtime tells from ptr
    if rc != 0:
        raise RuntimeError(f"hipMemcpy device->host failed with HIP error {rc}")
    return out


def copy_device(dst_ptr: int, src_ptr: int, nbytes: int) -> None:
    """Blocking copy of nbytes between two addresses the runtime knows (device or pinned host)."""
    rc = _hip.hipMemcpy(dst_ptr, src_ptr, nbytes, 4)                   # hipMemcpyDefault
    if rc != 0:
        raise RuntimeError(f"hipMemcpy failed with HIP error {rc}")


def write_device(ptr: int, array) -> None:
    """Blocking copy of a contiguous numpy array to device address `ptr`."""
    import numpy as np
    a = np.ascontiguousarray(array)
    rc = _hip.hipMemcpy(ptr, a.ctypes.data_as(_vp), a.nbytes, 1)       # hipMemcpyHostToDevice
    if rc != 0:
        raise RuntimeError(f"hipMemcpy host->device failed with HIP error {rc}")


def last_error() -> str:
    return (lib.lga_last_error() or b"").decode()


def check(code: int) -> None:
    if code != LGA_OK:
        raise LgaError(code, last_error())


def make_config(n_layers, d_model, n_heads, d_ff, seq_len, micro_batch, n_micro, dtype, group=1, retain_grads=0,
                ln_eps=1e-5, stream: Optional[int] = None, wgrad_groups=0, param_buffers=0, overlap=0,
                attention=0, offload_checkpoints=0) -> lga_config:
    return lga_config(n_layers, d_model, n_heads, d_ff, seq_len, micro_batch, n_micro, dtype, group, retain_grads,
                      wgrad_groups, param_buffers, overlap, attention, offload_checkpoints, ln_eps, stream)


def params_per_layer(cfg: lga_config) -> int:
    out = _u64()
    check(lib.lga_params_per_layer(C.byref(cfg), C.byref(out)))
    return out.value


def arena_bytes(cfg: lga_config) -> int:
    out = _u64()
    check(lib.lga_arena_bytes(C.byref(cfg), C.byref(out)))
    return out.value


def host_bytes(cfg: lga_config) -> int:
    out = _u64()
    check(lib.lga_host_bytes(C.byref(cfg), C.byref(out)))
    return out.value


def traffic_model(cfg: lga_config, order: int):
    pb, gb, fl = _u64(), _u64(), C.c_double()
    check(lib.lga_traffic_model(C.byref(cfg), order, C.byref(pb), C.byref(gb), C.byref(fl)))
    return pb.value, gb.value, fl.value


class Stack:
    """Owns an lga_stack handle.  Methods map one-to-one onto the C entry points."""

    def __init__(self, cfg: lga_config, host_params=None):
        self.cfg = cfg
        self._h = _vp()
        ptr = None
        if host_params is not None:
            import numpy as np
            self._keep = np.ascontiguousarray(host_params, dtype=np.float32)
            n = cfg.n_layers * params_per_layer(cfg)
            if self._keep.size != n:
                raise ValueError(f"host_params has {self._keep.size} floats, expected {n}")
            ptr = self._keep.ctypes.data_as(_vp)
        check(lib.lga_init_stack(C.byref(cfg), ptr, C.byref(self._h)))
        self._keep = None

    def close(self):
        if self._h:
            lib.lga_destroy_stack(self._h)
            self._h = _vp()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def forward_layered(self, x_ptr: int, y_ptr: Optional[int]):
        check(lib.lga_forward_layered(self._h, x_ptr, y_ptr))

    def backward_layered(self, dy_ptr: int, dx_ptr: Optional[int], adam: Optional[lga_adam]):
        check(lib.lga_backward_layered(self._h, dy_ptr, dx_ptr, C.byref(adam) if adam is not None else None))

    def step_mbmajor(self, x_ptr, dy_ptr, y_ptr, dx_ptr, adam: Optional[lga_adam]):
        check(lib.lga_step_mbmajor(self._h, x_ptr, dy_ptr, y_ptr, dx_ptr, C.byref(adam) if adam is not None else None))

    def forward_layer(self, layer: int, x_in_ptr: int, x_out_ptr: Optional[int]):
        check(lib.lga_forward_layer(self._h, layer, x_in_ptr, x_out_ptr))

    def backward_layer(self, layer: int, dy_ptr: int, dx_ptr: Optional[int], adam: Optional[lga_adam]):
        check(lib.lga_backward_layer(self._h, layer, dy_ptr, dx_ptr, C.byref(adam) if adam is not None else None))

    def adam_step_layer(self, layer: int, adam: lga_adam):
        check(lib.lga_adam_step_layer(self._h, layer, C.byref(adam)))

    def _borrow(self, fn, index):
        p, n = _vp(), C.c_size_t()
        check(fn(self._h, index, C.byref(p), C.byref(n)))
        return p.value, n.value

    def grads(self, layer: int):
        return self._borrow(lib.lga_grads, layer)

    def params(self, layer: int):
        return self._borrow(lib.lga_params, layer)

    def checkpoint(self, boundary: int):
        return self._borrow(lib.lga_checkpoint, boundary)

    def _layer_flags(self, fn):
        flags = (C.c_int32 * self.cfg.n_layers)()
        count = C.c_int32()
        check(fn(self._h, flags, C.byref(count)))
        assert count.value == sum(flags)
        return list(flags)

    def nonfinite_layers(self):
        """Per layer: 1 if its last Adam step with skip_nonfinite was left out."""
        return self._layer_flags(lib.lga_nonfinite_layers)

    def grads_nonfinite(self):
        """Per layer: 1 if the gradient it currently holds has a non-finite value."""
        return self._layer_flags(lib.lga_grads_nonfinite)

    def restore_count(self) -> int:
        out = _u64()
        check(lib.lga_restore_count(self._h, C.byref(out)))
        return out.value

    def profile_begin(self, only: str | None = None):
        """Bracket every launch with an event pair, or only those of the kernel whose name starts with `only`."""
        if only:
            check(lib.lga_profile_begin_only(self._h, only.encode()))
        else:
            check(lib.lga_profile_begin(self._h))

    def profile_end(self, capacity: int = 64):
        arr = (lga_kernel_stat * capacity)()
        n = _i32()
        check(lib.lga_profile_end(self._h, arr, capacity, C.byref(n)))
        return [dict(name=arr[i].name.decode(), launches=arr[i].launches, ms=arr[i].ms, flops=arr[i].flops,
                     bytes=arr[i].bytes) for i in range(min(n.value, capacity))]

    def moments(self, layer: int):
        m, v, n = _vp(), _vp(), C.c_size_t()
        check(lib.lga_moments(self._h, layer, C.byref(m), C.byref(v), C.byref(n)))
        return m.value, v.value, n.value
