"""Thin ctypes binding of the C-ABI library declared in ``include/lp.h``.

Argument marshalling only: every step of the path runs in the library's HIP
kernels.  Function names are the C names.  Device buffers are passed as raw
addresses (``tensor.data_ptr()``) or as torch tensors, from which the address
is taken; the stream is a raw ``hipStream_t`` value (``torch.cuda.current_stream().cuda_stream``)
or 0/None for the default stream.

There is no fallback: if ``liblp_mi355x.so`` has not been built (``python -m
paper_2512_07350_amd.build``) loading raises, and any non-zero status from the
library raises :class:`LPError`.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblp_mi355x.so")

LP_OK = 0
LP_ERR_INVALID_ARG = -1
LP_ERR_SHAPE = -2
LP_ERR_UNSUPPORTED = -3
LP_ERR_HIP = -4
LP_ERR_NOMEM = -5
LP_ERR_LIMIT = -6
LP_MAX_PARTS = 64

# every symbol include/lp.h declares
EXPORTS = (
    "lp_rotation_dim", "lp_plan_create", "lp_plan_destroy", "lp_plan_num_parts", "lp_plan_dim",
    "lp_plan_total_elems", "lp_plan_latent_elems", "lp_plan_query", "lp_partition", "lp_reconstruct",
    "lp_reconstruct_guided_step", "lp_reconstruct_guided_step_partition",
    "lp_attention", "lp_attention_batch", "lp_attention_workspace_size", "lp_attention_static",
    "lp_attention_static_scratch_bytes", "lp_qkv_projection", "lp_linear", "lp_qk_norm_rope",
    "lp_strerror", "lp_last_hip_error", "lp_version",
)


class lp_config(C.Structure):
    _fields_ = [("C", C.c_int32), ("T", C.c_int32), ("H", C.c_int32), ("W", C.c_int32),
                ("pT", C.c_int32), ("pH", C.c_int32), ("pW", C.c_int32),
                ("K", C.c_int32), ("overlap_patches", C.c_int32), ("overlap_ratio", C.c_double)]


class lp_part_info(C.Structure):
    _fields_ = [("alpha", C.c_int32), ("beta", C.c_int32), ("alpha_ext", C.c_int32), ("beta_ext", C.c_int32),
                ("s", C.c_int32), ("e", C.c_int32), ("len", C.c_int32),
                ("delta_start", C.c_int32), ("delta_end", C.c_int32), ("shape", C.c_int32 * 4),
                ("elem_offset", C.c_int64), ("n_elems", C.c_int64), ("n_tokens", C.c_int64)]


class lp_rope(C.Structure):
    _fields_ = [("grid", C.c_int32 * 3), ("offset", C.c_int32 * 3), ("split", C.c_int32 * 3), ("base", C.c_float)]


class LPError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = _lib().lp_strerror(status).decode()
        if status == LP_ERR_HIP:
            msg += " [hipError %d]" % _lib().lp_last_hip_error()
        super().__init__("%s: %s (%d)" % (where, msg, status))


_handle = None


def _lib():
    global _handle
    if _handle is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("%s is missing: build it with `python -m paper_2512_07350_amd.build` "
                               "(there is no fallback path)" % LIB_PATH)
        # One HIP runtime per process: the PyTorch wheel bundles its own libamdhip64, and
        # device memory and streams come from PyTorch, so it has to be the runtime this
        # library binds to.  Importing torch first makes the loader resolve the library's
        # libamdhip64 dependency to the copy that is already mapped.
        import torch  # noqa: F401
        lib = C.CDLL(LIB_PATH)
        vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
        lib.lp_rotation_dim.argtypes = [i64]
        lib.lp_rotation_dim.restype = C.c_int
        lib.lp_plan_create.argtypes = [C.POINTER(lp_config), i32, C.POINTER(vp)]
        lib.lp_plan_create.restype = C.c_int
        lib.lp_plan_destroy.argtypes = [vp]
        lib.lp_plan_destroy.restype = None
        lib.lp_plan_num_parts.argtypes = [vp]
        lib.lp_plan_num_parts.restype = i32
        lib.lp_plan_dim.argtypes = [vp]
        lib.lp_plan_dim.restype = i32
        lib.lp_plan_total_elems.argtypes = [vp]
        lib.lp_plan_total_elems.restype = i64
        lib.lp_plan_latent_elems.argtypes = [vp]
        lib.lp_plan_latent_elems.restype = i64
        lib.lp_plan_query.argtypes = [vp, i32, C.POINTER(lp_part_info)]
        lib.lp_plan_query.restype = C.c_int
        lib.lp_partition.argtypes = [vp, vp, vp, vp]
        lib.lp_partition.restype = C.c_int
        lib.lp_reconstruct.argtypes = [vp, vp, vp, vp]
        lib.lp_reconstruct.restype = C.c_int
        lib.lp_reconstruct_guided_step.argtypes = [vp, vp, vp, C.c_float, vp, C.c_float, C.c_float, vp, vp]
        lib.lp_reconstruct_guided_step.restype = C.c_int
        lib.lp_reconstruct_guided_step_partition.argtypes = [vp, vp, vp, C.c_float, vp, C.c_float, C.c_float, vp, vp, vp, vp]
        lib.lp_reconstruct_guided_step_partition.restype = C.c_int
        lib.lp_attention.argtypes = [vp, vp, vp, vp, i64, i32, i32, i64, i64, C.c_float, vp, i64, vp]
        lib.lp_attention.restype = C.c_int
        lib.lp_attention_batch.argtypes = [vp, vp, vp, vp, i32, i64, i32, i32, i64, i64, i64, C.c_float, vp, i64, vp]
        lib.lp_attention_batch.restype = C.c_int
        lib.lp_attention_static.argtypes = [vp, vp, vp, vp, i64, i32, i32, i64, i64, C.c_float, vp]
        lib.lp_attention_static.restype = C.c_int
        lib.lp_attention_static_scratch_bytes.argtypes = []
        lib.lp_attention_static_scratch_bytes.restype = i64
        lib.lp_qkv_projection.argtypes = [vp, vp, vp, vp, vp, C.c_float, C.POINTER(lp_rope), vp, vp, vp, i64, i32, i32, vp]
        lib.lp_qkv_projection.restype = C.c_int
        lib.lp_linear.argtypes = [vp, vp, vp, vp, i64, i32, i32, vp]
        lib.lp_linear.restype = C.c_int
        lib.lp_qk_norm_rope.argtypes = [vp, vp, C.c_float, C.POINTER(lp_rope), i64, i32, i32, i64, i64, vp]
        lib.lp_qk_norm_rope.restype = C.c_int
        lib.lp_attention_workspace_size.argtypes = [i32]
        lib.lp_attention_workspace_size.restype = i64
        lib.lp_strerror.argtypes = [C.c_int]
        lib.lp_strerror.restype = C.c_char_p
        lib.lp_last_hip_error.argtypes = []
        lib.lp_last_hip_error.restype = C.c_int
        lib.lp_version.argtypes = []
        lib.lp_version.restype = C.c_char_p
        _handle = lib
    return _handle


def _ptr(x) -> int:
    """Raw address of a device buffer: an int, or anything with data_ptr() (a torch tensor)."""
    if x is None:
        return 0
    if isinstance(x, int):
        return x
    return int(x.data_ptr())


def _check(status: int, where: str) -> None:
    if status != LP_OK:
        raise LPError(status, where)


def lp_version() -> str:
    return _lib().lp_version().decode()


def lp_strerror(status: int) -> str:
    return _lib().lp_strerror(int(status)).decode()


def lp_last_hip_error() -> int:
    return int(_lib().lp_last_hip_error())


def lp_rotation_dim(step_1based: int) -> int:
    d = _lib().lp_rotation_dim(int(step_1based))
    if d < 0:
        raise LPError(d, "lp_rotation_dim")
    return d


class Plan:
    """Owns one ``lp_plan*``; destroyed with the object."""

    def __init__(self, handle: int):
        self._h = C.c_void_p(handle)

    def __del__(self):
        h, self._h = getattr(self, "_h", None), None
        if h and _handle is not None:
            _handle.lp_plan_destroy(h)

    @property
    def handle(self):
        return self._h

    @property
    def K(self) -> int:
        return lp_plan_num_parts(self)

    @property
    def dim(self) -> int:
        return lp_plan_dim(self)

    @property
    def total_elems(self) -> int:
        return lp_plan_total_elems(self)

    @property
    def latent_elems(self) -> int:
        return lp_plan_latent_elems(self)

    def parts(self):
        return [lp_plan_query(self, k) for k in range(self.K)]


def lp_plan_create(latent, patch, K: int, dim: int, overlap_patches: int = -1, overlap_ratio: float = 0.0) -> Plan:
    cfg = lp_config(int(latent[0]), int(latent[1]), int(latent[2]), int(latent[3]),
                    int(patch[0]), int(patch[1]), int(patch[2]), int(K), int(overlap_patches), float(overlap_ratio))
    out = C.c_void_p()
    _check(_lib().lp_plan_create(C.byref(cfg), int(dim), C.byref(out)), "lp_plan_create")
    return Plan(out.value)


def lp_plan_num_parts(plan: Plan) -> int:
    return int(_lib().lp_plan_num_parts(plan.handle))


def lp_plan_dim(plan: Plan) -> int:
    return int(_lib().lp_plan_dim(plan.handle))


def lp_plan_total_elems(plan: Plan) -> int:
    return int(_lib().lp_plan_total_elems(plan.handle))


def lp_plan_latent_elems(plan: Plan) -> int:
    return int(_lib().lp_plan_latent_elems(plan.handle))


def lp_plan_query(plan: Plan, k: int) -> lp_part_info:
    info = lp_part_info()
    _check(_lib().lp_plan_query(plan.handle, int(k), C.byref(info)), "lp_plan_query")
    return info


def lp_partition(plan: Plan, z, subs_packed, stream: Optional[int] = None) -> None:
    _check(_lib().lp_partition(plan.handle, _ptr(z), _ptr(subs_packed), stream or None), "lp_partition")


def lp_reconstruct(plan: Plan, preds_packed, out, stream: Optional[int] = None) -> None:
    _check(_lib().lp_reconstruct(plan.handle, _ptr(preds_packed), _ptr(out), stream or None), "lp_reconstruct")


def lp_reconstruct_guided_step(plan: Plan, cond_packed, uncond_packed, guidance: float, z, coef_z: float,
                               coef_pred: float, out, stream: Optional[int] = None) -> None:
    _check(_lib().lp_reconstruct_guided_step(plan.handle, _ptr(cond_packed), _ptr(uncond_packed), float(guidance),
                                             _ptr(z), float(coef_z), float(coef_pred), _ptr(out), stream or None),
           "lp_reconstruct_guided_step")


def lp_reconstruct_guided_step_partition(plan: Plan, cond_packed, uncond_packed, guidance: float, z, coef_z: float,
                                         coef_pred: float, out, next_plan: Plan, next_subs_packed,
                                         stream: Optional[int] = None) -> None:
    _check(_lib().lp_reconstruct_guided_step_partition(plan.handle, _ptr(cond_packed), _ptr(uncond_packed),
                                                       float(guidance), _ptr(z), float(coef_z), float(coef_pred),
                                                       _ptr(out), next_plan.handle, _ptr(next_subs_packed),
                                                       stream or None), "lp_reconstruct_guided_step_partition")


def lp_attention_workspace_size(head_dim: int) -> int:
    n = int(_lib().lp_attention_workspace_size(int(head_dim)))
    if n < 0:
        raise LPError(n, "lp_attention_workspace_size")
    return n


def lp_attention(q, k, v, o, n_tokens: int, heads: int, head_dim: int, stride_tok: int, stride_head: int,
                 scale: float = 0.0, workspace=None, workspace_bytes: int = 0, stream: Optional[int] = None) -> None:
    _check(_lib().lp_attention(_ptr(q), _ptr(k), _ptr(v), _ptr(o), int(n_tokens), int(heads), int(head_dim),
                               int(stride_tok), int(stride_head), float(scale), _ptr(workspace) or None,
                               int(workspace_bytes), stream or None), "lp_attention")


def lp_attention_batch(q, k, v, o, batch: int, n_tokens: int, heads: int, head_dim: int, stride_batch: int,
                       stride_tok: int, stride_head: int, scale: float = 0.0, workspace=None,
                       workspace_bytes: int = 0, stream: Optional[int] = None) -> None:
    _check(_lib().lp_attention_batch(_ptr(q), _ptr(k), _ptr(v), _ptr(o), int(batch), int(n_tokens), int(heads),
                                     int(head_dim), int(stride_batch), int(stride_tok), int(stride_head), float(scale),
                                     _ptr(workspace) or None, int(workspace_bytes), stream or None), "lp_attention_batch")


def lp_attention_static(q, k, v, o, n_tokens: int, heads: int, head_dim: int, stride_tok: int, stride_head: int,
                        scale: float = 0.0, stream: Optional[int] = None) -> None:
    _check(_lib().lp_attention_static(_ptr(q), _ptr(k), _ptr(v), _ptr(o), int(n_tokens), int(heads), int(head_dim),
                                      int(stride_tok), int(stride_head), float(scale), stream or None), "lp_attention_static")


def lp_attention_static_scratch_bytes() -> int:
    return int(_lib().lp_attention_static_scratch_bytes())


def make_rope(grid, offset=(0, 0, 0), split=None, base: float = 10000.0, head_dim: int = 128) -> lp_rope:
    """The rotary description; split defaults to (head_dim - 4 floor(head_dim / 6), 2 floor(head_dim / 6), 2 floor(head_dim / 6))."""
    if split is None:
        hw = 2 * (head_dim // 6)
        split = (head_dim - 2 * hw, hw, hw)
    r = lp_rope()
    for i in range(3):
        r.grid[i], r.offset[i], r.split[i] = int(grid[i]), int(offset[i]), int(split[i])
    r.base = float(base)
    return r


def lp_qkv_projection(x, w_qkv, bias, gain_q, gain_k, eps: float, rope: lp_rope, q, k, v, n_tokens: int, heads: int,
                      head_dim: int, stream: Optional[int] = None) -> None:
    _check(_lib().lp_qkv_projection(_ptr(x), _ptr(w_qkv), _ptr(bias) or None, _ptr(gain_q), _ptr(gain_k), float(eps),
                                    C.byref(rope), _ptr(q), _ptr(k), _ptr(v), int(n_tokens), int(heads), int(head_dim),
                                    stream or None), "lp_qkv_projection")


def lp_linear(x, w, bias, y, n: int, d_in: int, d_out: int, stream: Optional[int] = None) -> None:
    _check(_lib().lp_linear(_ptr(x), _ptr(w), _ptr(bias) or None, _ptr(y), int(n), int(d_in), int(d_out), stream or None),
           "lp_linear")


def lp_qk_norm_rope(x, gain, eps: float, rope: lp_rope, n_tokens: int, heads: int, head_dim: int, stride_tok: int,
                    stride_head: int, stream: Optional[int] = None) -> None:
    _check(_lib().lp_qk_norm_rope(_ptr(x), _ptr(gain), float(eps), C.byref(rope), int(n_tokens), int(heads), int(head_dim),
                                  int(stride_tok), int(stride_head), stream or None), "lp_qk_norm_rope")
