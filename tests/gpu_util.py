"""Helpers for the GPU parity tests: run the HIP path through the C-ABI binding.

torch is used for device memory and the stream only.
"""
import numpy as np
import torch

from paper_2512_07350_amd import binding as lp
from paper_2512_07350_amd import synth


def stream():
    return torch.cuda.current_stream().cuda_stream


def make_plan(latent, patch, K, dim, overlap_patches=-1, overlap_ratio=0.0):
    return lp.lp_plan_create(latent, patch, K, dim, overlap_patches=overlap_patches, overlap_ratio=overlap_ratio)


def hip_partition(plan, z: np.ndarray) -> np.ndarray:
    zd = torch.from_numpy(np.ascontiguousarray(z, dtype=np.float32)).cuda()
    subs = torch.full((max(plan.total_elems, 1),), float("nan"), dtype=torch.float32, device="cuda")
    lp.lp_partition(plan, zd, subs, stream())
    torch.cuda.synchronize()
    return subs.cpu().numpy()[:plan.total_elems]


def hip_reconstruct(plan, preds: np.ndarray, latent) -> np.ndarray:
    pd = torch.from_numpy(np.ascontiguousarray(preds, dtype=np.float32)).cuda()
    out = torch.full(tuple(latent), float("nan"), dtype=torch.float32, device="cuda")
    lp.lp_reconstruct(plan, pd, out, stream())
    torch.cuda.synchronize()
    return out.cpu().numpy()


def hip_guided_step(plan, cond: np.ndarray, uncond: np.ndarray, guidance, z: np.ndarray, coef_z, coef_pred,
                    in_place: bool = False) -> np.ndarray:
    cd = torch.from_numpy(np.ascontiguousarray(cond, dtype=np.float32)).cuda()
    ud = torch.from_numpy(np.ascontiguousarray(uncond, dtype=np.float32)).cuda()
    zd = torch.from_numpy(np.ascontiguousarray(z, dtype=np.float32)).cuda()
    out = zd if in_place else torch.full(tuple(z.shape), float("nan"), dtype=torch.float32, device="cuda")
    lp.lp_reconstruct_guided_step(plan, cd, ud, guidance, zd, coef_z, coef_pred, out, stream())
    torch.cuda.synchronize()
    return out.cpu().numpy()


def hip_guided_step_partition(plan, cond, uncond, guidance, z, coef_z, coef_pred, next_plan, in_place=False):
    """-> (updated latent, packed sub-latents of the next step), one fused launch."""
    cd = torch.from_numpy(np.ascontiguousarray(cond, dtype=np.float32)).cuda()
    ud = torch.from_numpy(np.ascontiguousarray(uncond, dtype=np.float32)).cuda()
    zd = torch.from_numpy(np.ascontiguousarray(z, dtype=np.float32)).cuda()
    out = zd if in_place else torch.full(tuple(z.shape), float("nan"), dtype=torch.float32, device="cuda")
    subs = torch.full((max(next_plan.total_elems, 1),), float("nan"), dtype=torch.float32, device="cuda")
    lp.lp_reconstruct_guided_step_partition(plan, cd, ud, guidance, zd, coef_z, coef_pred, out, next_plan, subs, stream())
    torch.cuda.synchronize()
    return out.cpu().numpy(), subs.cpu().numpy()[:next_plan.total_elems]


def to_dev_bf16(bits: np.ndarray) -> torch.Tensor:
    """uint16 bf16 bit patterns -> device tensor of dtype bfloat16 with the same bits."""
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def from_dev_bf16(t: torch.Tensor) -> np.ndarray:
    """device bfloat16 tensor -> float32 numpy (exact widening)."""
    bits = t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
    return synth.bf16_bits_to_f32(bits)


_workspaces = {}


def workspace(head_dim: int):
    """(tensor, bytes): device scratch for lp_attention, allocated once per head_dim and
    refilled with NaN at every request, so that a read of a slot nobody wrote IN THIS CALL
    shows up in the result (data left by an earlier call would look plausible)."""
    if head_dim not in _workspaces:
        nbytes = lp.lp_attention_workspace_size(head_dim)
        _workspaces[head_dim] = (torch.empty((nbytes // 4,), dtype=torch.float32, device="cuda"), nbytes)
    _workspaces[head_dim][0].fill_(float("nan"))
    return _workspaces[head_dim]


def hip_attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, scale: float = 0.0, balanced: bool = True) -> np.ndarray:
    """q, k, v: uint16 [n, heads, d] token-major.  Returns float32 [n, heads, d].
    balanced=True passes a workspace (the launch configuration the benchmark times);
    False launches one workgroup per query tile and head."""
    n, heads, d = q.shape
    qd, kd, vd = to_dev_bf16(q), to_dev_bf16(k), to_dev_bf16(v)
    od = torch.full((n, heads, d), float("nan"), dtype=torch.bfloat16, device="cuda")
    ws, ws_bytes = workspace(d) if balanced else (None, 0)
    lp.lp_attention(qd, kd, vd, od, n, heads, d, heads * d, d, scale, ws, ws_bytes, stream())
    torch.cuda.synchronize()
    return from_dev_bf16(od)


def hip_attention_batch(items, scale: float = 0.0, balanced: bool = True, layout: str = "outer"):
    """items: list of (q, k, v) uint16 [n, heads, d].  One lp_attention_batch call over all of
    them; returns the list of float32 outputs.  layout "outer": [batch, n, heads, d];
    "inner": [n, batch, heads, d] (the items of a token side by side)."""
    b = len(items)
    n, heads, d = items[0][0].shape
    stack = lambda j: np.stack([it[j] for it in items], axis=0 if layout == "outer" else 1)
    qd, kd, vd = to_dev_bf16(stack(0)), to_dev_bf16(stack(1)), to_dev_bf16(stack(2))
    od = torch.full(tuple(qd.shape), float("nan"), dtype=torch.bfloat16, device="cuda")
    ws, ws_bytes = workspace(d) if balanced else (None, 0)
    if layout == "outer":
        strides = (n * heads * d, heads * d, d)
    else:
        strides = (heads * d, b * heads * d, d)
    lp.lp_attention_batch(qd, kd, vd, od, b, n, heads, d, strides[0], strides[1], strides[2], scale, ws, ws_bytes, stream())
    torch.cuda.synchronize()
    out = from_dev_bf16(od)
    return [out[i] if layout == "outer" else out[:, i] for i in range(b)]


# tolerance of the attention path against the fp32/fp64 oracle on N(0,1) inputs at the default
# scale 1/sqrt(head_dim)
ATT_MAX_ABS = 2e-2
ATT_MEAN_ABS = 2e-3


def assert_attention_close(got: np.ndarray, want: np.ndarray, what="", sharpness: float = 1.0):
    """sharpness = scale * sqrt(head_dim) when a test passes an explicit scale above the default:
    the stated tolerance is for logits of unit variance; with logits `sharpness` times wider the
    softmax concentrates on few keys (outputs no longer average down from |v| ~ 1 to ~ 1/sqrt(n))
    and the rounding of the pre-scaled q to bf16 perturbs every logit `sharpness` times more, so
    both bounds are widened by that factor (never narrowed)."""
    f = max(1.0, float(sharpness))
    assert got.shape == want.shape
    assert np.all(np.isfinite(got)), what
    err = np.abs(got.astype(np.float64) - want.astype(np.float64))
    assert err.max() <= ATT_MAX_ABS * f, (what, float(err.max()))
    assert err.mean() <= ATT_MEAN_ABS * f, (what, float(err.mean()))
