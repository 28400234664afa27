"""ctypes front end of the CPU oracle (``lp_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the
benchmark's CPU-baseline leg.  The HIP library and its Python binding never
import this module, and this module imports nothing from them.

The functions mirror the C ones one to one; numpy is used for buffers only, no
arithmetic of the method happens on this side.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lp_oracle.c")
_SRC_BLOCK = os.path.join(_HERE, "lp_block_oracle.c")
_LIB = os.path.join(_HERE, "liblp_oracle.so")

# -ffp-contract=off and no -ffast-math: the reconstruction's binary32 operation
# order is part of the definition being checked.
_CFLAGS = ["-O2", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared", "-Wall", "-Wextra"]


def build(force: bool = False) -> str:
    """Compile lp_oracle.c and lp_block_oracle.c with gcc into liblp_oracle.so (next to the sources)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < max(os.path.getmtime(_SRC), os.path.getmtime(_SRC_BLOCK))
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.run(["gcc", *_CFLAGS, "-o", tmp, _SRC, _SRC_BLOCK, "-lm"], check=True)
        os.replace(tmp, _LIB)
    return _LIB


class _Part(C.Structure):
    _fields_ = [
        ("alpha", C.c_int32), ("beta", C.c_int32),
        ("alpha_ext", C.c_int32), ("beta_ext", C.c_int32),
        ("s", C.c_int32), ("e", C.c_int32), ("len", C.c_int32),
        ("delta_start", C.c_int32), ("delta_end", C.c_int32),
        ("shape", C.c_int32 * 4),
        ("elem_offset", C.c_int64), ("n_elems", C.c_int64), ("n_tokens", C.c_int64),
    ]


@dataclass(frozen=True)
class Part:
    alpha: int
    beta: int
    alpha_ext: int
    beta_ext: int
    s: int
    e: int
    len: int
    delta_start: int
    delta_end: int
    shape: tuple
    elem_offset: int
    n_elems: int
    n_tokens: int


@dataclass(frozen=True)
class Plan:
    latent: tuple          # (C, T, H, W)
    patch: tuple           # (pT, pH, pW)
    K: int
    dim: int               # 0 = T, 1 = H, 2 = W
    parts: tuple           # of Part
    total_elems: int

    def _c_parts(self):
        arr = (_Part * self.K)()
        for i, p in enumerate(self.parts):
            a = arr[i]
            a.alpha, a.beta, a.alpha_ext, a.beta_ext = p.alpha, p.beta, p.alpha_ext, p.beta_ext
            a.s, a.e, a.len, a.delta_start, a.delta_end = p.s, p.e, p.len, p.delta_start, p.delta_end
            for d in range(4):
                a.shape[d] = p.shape[d]
            a.elem_offset, a.n_elems, a.n_tokens = p.elem_offset, p.n_elems, p.n_tokens
        return arr


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = C.CDLL(build())
        i32p = C.POINTER(C.c_int32)
        lib.lpo_rotation_dim.argtypes = [C.c_int64]
        lib.lpo_rotation_dim.restype = C.c_int
        lib.lpo_plan.argtypes = [i32p, i32p, C.c_int32, C.c_int32, C.c_double, C.c_int32, C.POINTER(_Part)]
        lib.lpo_plan.restype = C.c_int
        lib.lpo_weight.argtypes = [C.c_int32] * 4
        lib.lpo_weight.restype = C.c_float
        lib.lpo_partition.argtypes = [i32p, C.c_int32, C.c_int32, C.POINTER(_Part), C.c_void_p, C.c_void_p]
        lib.lpo_partition.restype = None
        lib.lpo_reconstruct.argtypes = [i32p, C.c_int32, C.c_int32, C.POINTER(_Part), C.c_void_p, C.c_void_p]
        lib.lpo_reconstruct.restype = None
        lib.lpo_guided_step.argtypes = [i32p, C.c_int32, C.c_int32, C.POINTER(_Part), C.c_int64, C.c_void_p, C.c_void_p,
                                        C.c_float, C.c_void_p, C.c_float, C.c_float, C.c_void_p, C.c_void_p]
        lib.lpo_guided_step.restype = None
        lib.lpo_attention.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int32,
                                      C.c_int32, C.c_int64, C.c_int64, C.c_double, C.c_void_p, C.c_int64]
        lib.lpo_attention.restype = C.c_int
        lib.lpo_linear.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_int64, C.c_void_p]
        lib.lpo_linear.restype = None
        lib.lpo_rms_norm_heads.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, C.c_int32, C.c_double]
        lib.lpo_rms_norm_heads.restype = None
        lib.lpo_rope3d.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_int32, i32p, i32p, i32p, C.c_double]
        lib.lpo_rope3d.restype = C.c_int
        lib.lpo_num_threads.argtypes = []
        lib.lpo_num_threads.restype = C.c_int
        _lib = lib
    return _lib


def _i32(vals):
    return (C.c_int32 * len(vals))(*[int(v) for v in vals])


def rotation_dim(step_1based: int) -> int:
    """Eq. 3: 0 = temporal, 1 = height, 2 = width for the 1-based step index."""
    d = _load().lpo_rotation_dim(int(step_1based))
    if d < 0:
        raise ValueError("step index must be >= 1")
    return d


def plan(latent: Sequence[int], patch: Sequence[int], K: int, dim: int, *,
         overlap_patches: int = -1, r: float = 0.0, overlap_ratio: Optional[float] = None) -> Plan:
    """Eq. 7-9, 11: the K partitions of a [C,T,H,W] latent along ``dim``.
    ``overlap_ratio`` is another name for ``r``."""
    if overlap_ratio is not None:
        r = overlap_ratio
    if K < 1:
        raise ValueError("K must be >= 1")
    parts = (_Part * K)()
    rc = _load().lpo_plan(_i32(latent), _i32(patch), K, int(overlap_patches), float(r), int(dim), parts)
    if rc != 0:
        raise ValueError("arguments outside what the method defines")
    out: List[Part] = []
    for a in parts:
        out.append(Part(a.alpha, a.beta, a.alpha_ext, a.beta_ext, a.s, a.e, a.len, a.delta_start,
                        a.delta_end, tuple(a.shape), a.elem_offset, a.n_elems, a.n_tokens))
    total = sum(p.n_elems for p in out)
    return Plan(tuple(int(v) for v in latent), tuple(int(v) for v in patch), K, int(dim), tuple(out), total)


def weight(j: int, length: int, delta_start: int, delta_end: int) -> np.float32:
    """Eq. 12 at local position j (binary32)."""
    return np.float32(_load().lpo_weight(j, length, delta_start, delta_end))


def partition(pl: Plan, z: np.ndarray) -> np.ndarray:
    """Eq. 10: packed sub-latents (float32, total_elems) of latent z [C,T,H,W]."""
    z = np.ascontiguousarray(z, dtype=np.float32)
    assert z.shape == pl.latent
    subs = np.empty(pl.total_elems, dtype=np.float32)
    _load().lpo_partition(_i32(pl.latent), pl.dim, pl.K, pl._c_parts(), z.ctypes.data, subs.ctypes.data)
    return subs


def reconstruct(pl: Plan, preds: np.ndarray) -> np.ndarray:
    """Eq. 13-17: stitched [C,T,H,W] float32 latent from packed predictions."""
    preds = np.ascontiguousarray(preds, dtype=np.float32)
    assert preds.shape == (pl.total_elems,)
    out = np.empty(pl.latent, dtype=np.float32)
    _load().lpo_reconstruct(_i32(pl.latent), pl.dim, pl.K, pl._c_parts(), preds.ctypes.data, out.ctypes.data)
    return out


def guided_step(pl: Plan, cond: np.ndarray, uncond: np.ndarray, guidance: float, z: np.ndarray,
                coef_z: float, coef_pred: float) -> np.ndarray:
    """Eq. 4-6: z' = coef_z * z + coef_pred * F({u_k + guidance (c_k - u_k)}), float32 [C,T,H,W]."""
    cond = np.ascontiguousarray(cond, dtype=np.float32)
    uncond = np.ascontiguousarray(uncond, dtype=np.float32)
    z = np.ascontiguousarray(z, dtype=np.float32)
    assert cond.shape == uncond.shape == (pl.total_elems,) and z.shape == tuple(pl.latent)
    scratch = np.empty(pl.total_elems, dtype=np.float32)
    out = np.empty(pl.latent, dtype=np.float32)
    _load().lpo_guided_step(_i32(pl.latent), pl.dim, pl.K, pl._c_parts(), pl.total_elems, cond.ctypes.data,
                            uncond.ctypes.data, float(guidance), z.ctypes.data, float(coef_z), float(coef_pred),
                            scratch.ctypes.data, out.ctypes.data)
    return out


def attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, *, scale: Optional[float] = None,
              rows: Optional[Sequence[int]] = None) -> np.ndarray:
    """softmax(scale q k^T) v per head.

    q, k, v: uint16 arrays of bf16 bit patterns, shape [n, heads, head_dim],
    C-contiguous.  ``rows`` selects query rows (each still sees all n keys).
    Returns float32 [n_rows, heads, head_dim].
    """
    for a in (q, k, v):
        assert a.dtype == np.uint16 and a.ndim == 3 and a.flags.c_contiguous
    assert q.shape == k.shape == v.shape
    n, heads, hd = q.shape
    if scale is None:
        scale = 1.0 / float(np.sqrt(np.float64(hd)))
    if rows is None:
        rows_arr, n_rows, rows_ptr = None, n, None
    else:
        rows_arr = np.ascontiguousarray(rows, dtype=np.int64)
        assert rows_arr.ndim == 1
        if rows_arr.size and (rows_arr.min() < 0 or rows_arr.max() >= n):
            raise IndexError("query row out of range")
        n_rows, rows_ptr = rows_arr.size, rows_arr.ctypes.data
    out = np.zeros((n_rows, heads, hd), dtype=np.float32)
    rc = _load().lpo_attention(q.ctypes.data, k.ctypes.data, v.ctypes.data, out.ctypes.data, n, heads, hd,
                               heads * hd, hd, float(scale), rows_ptr, n_rows)
    if rc != 0:
        raise MemoryError("oracle attention could not allocate its work buffers")
    return out


def num_threads() -> int:
    """Threads the oracle's parallel loops use."""
    return int(_load().lpo_num_threads())


# ---- the DiT-block operations next to attention (lp_block_oracle.c)

def rope_split(head_dim: int):
    """The split of head_dim into (temporal, height, width) parts used throughout: height and
    width get 2 * floor(head_dim / 6) each, the temporal part the rest (128 -> 44, 42, 42)."""
    hw = 2 * (head_dim // 6)
    return (head_dim - 2 * hw, hw, hw)


def linear(x: np.ndarray, w: np.ndarray, bias: Optional[np.ndarray] = None) -> np.ndarray:
    """y = x w^T + bias.  x: uint16 bf16 bits [n, d_in]; w: uint16 [d_out, d_in]; bias float32 [d_out] or None.
    Returns float32 [n, d_out]."""
    assert x.dtype == np.uint16 and w.dtype == np.uint16 and x.ndim == 2 and w.ndim == 2 and x.shape[1] == w.shape[1]
    x, w = np.ascontiguousarray(x), np.ascontiguousarray(w)
    n, d_in = x.shape
    d_out = w.shape[0]
    b = None if bias is None else np.ascontiguousarray(bias, dtype=np.float32)
    assert b is None or b.shape == (d_out,)
    y = np.empty((n, d_out), dtype=np.float32)
    _load().lpo_linear(x.ctypes.data, w.ctypes.data, None if b is None else b.ctypes.data, n, d_in, d_out, y.ctypes.data)
    return y


def rms_norm_heads(x: np.ndarray, gain: np.ndarray, eps: float) -> np.ndarray:
    """Per-(token, head) RMS normalisation over head_dim times gain[head, d].  x: float32 [n, heads, head_dim]."""
    out = np.array(x, dtype=np.float32, order="C", copy=True)
    n, heads, hd = out.shape
    g = np.ascontiguousarray(gain, dtype=np.float32)
    assert g.shape == (heads, hd)
    _load().lpo_rms_norm_heads(out.ctypes.data, g.ctypes.data, n, heads, hd, float(eps))
    return out


def rope3d(x: np.ndarray, grid: Sequence[int], offset: Sequence[int] = (0, 0, 0), split: Optional[Sequence[int]] = None,
           base: float = 10000.0) -> np.ndarray:
    """3-D rotary encoding of x float32 [n, heads, head_dim] over the (t, h, w) patch grid `grid` (n = product)."""
    out = np.array(x, dtype=np.float32, order="C", copy=True)
    n, heads, hd = out.shape
    split = rope_split(hd) if split is None else tuple(split)
    rc = _load().lpo_rope3d(out.ctypes.data, n, heads, hd, _i32(grid), _i32(offset), _i32(split), float(base))
    if rc != 0:
        raise ValueError("rotary split must be even parts adding up to head_dim, and the grid must hold n tokens")
    return out


def qkv_block(x: np.ndarray, w_qkv: np.ndarray, bias: Optional[np.ndarray], gain_q: np.ndarray, gain_k: np.ndarray,
              eps: float, heads: int, head_dim: int, grid: Sequence[int], offset: Sequence[int] = (0, 0, 0),
              split: Optional[Sequence[int]] = None, base: float = 10000.0):
    """The block's way into attention: y = x w_qkv^T + bias, cut into the q | k | v sections of d_model
    features each ([n, heads, head_dim]); q and k are normalised per head and rotated, v is left as it is.
    Returns (q, k, v) float32."""
    dm = heads * head_dim
    assert w_qkv.shape == (3 * dm, dm)
    y = linear(x, w_qkv, bias)
    n = y.shape[0]
    q, k, v = (np.ascontiguousarray(y[:, s * dm:(s + 1) * dm]).reshape(n, heads, head_dim) for s in range(3))
    q = rope3d(rms_norm_heads(q, gain_q, eps), grid, offset, split, base)
    k = rope3d(rms_norm_heads(k, gain_k, eps), grid, offset, split, base)
    return q, k, v
