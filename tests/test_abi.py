"""C-ABI surface and host logic of the library -- no GPU needed.

The library's own plan integers (written independently of the oracle) are
compared with the oracle's over random shapes; no device function is called.
"""
import ctypes as C
import os
import re

import pytest
from hypothesis import given, settings, strategies as st

from oracle import lp_oracle as orc
from paper_2512_07350_amd import binding as lp

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "lp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lp_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared_functions()
    assert len(names) >= 14
    assert sorted(lp.EXPORTS) == names
    lib = C.CDLL(lp.LIB_PATH)
    for n in names:
        assert getattr(lib, n) is not None


def test_version_and_strerror():
    assert "gfx950" in lp.lp_version()
    assert lp.lp_strerror(0) == "ok"
    for code in (-1, -2, -3, -4, -5, -6, -99):
        assert lp.lp_strerror(code)


def test_rotation_dim_matches_oracle():
    for i in range(1, 50):
        assert lp.lp_rotation_dim(i) == orc.rotation_dim(i)
    with pytest.raises(lp.LPError):
        lp.lp_rotation_dim(0)


def _same_plan(latent, patch, K, dim, **kw):
    ref = orc.plan(latent, patch, K, dim, overlap_patches=kw.get("overlap_patches", -1), r=kw.get("overlap_ratio", 0.0))
    got = lp.lp_plan_create(latent, patch, K, dim, **kw)
    assert got.K == K and got.dim == dim
    assert got.total_elems == ref.total_elems
    assert got.latent_elems == latent[0] * latent[1] * latent[2] * latent[3]
    for k, (a, b) in enumerate(zip(got.parts(), ref.parts)):
        assert (a.alpha, a.beta, a.alpha_ext, a.beta_ext) == (b.alpha, b.beta, b.alpha_ext, b.beta_ext), k
        assert (a.s, a.e, a.len) == (b.s, b.e, b.len), k
        if b.len:
            assert (a.delta_start, a.delta_end) == (b.delta_start, b.delta_end), k
        assert tuple(a.shape) == b.shape and a.elem_offset == b.elem_offset
        assert a.n_elems == b.n_elems and a.n_tokens == b.n_tokens


@pytest.mark.parametrize("latent,K,O,dims", [
    ((16, 5, 16, 16), 2, 1, (2,)),
    ((16, 9, 60, 104), 4, 1, (0, 1, 2)),
    ((16, 21, 60, 104), 4, 2, (0, 1, 2)),
    ((16, 21, 90, 160), 8, 2, (2,)),
])
def test_plan_matches_oracle_on_benchmark_shapes(latent, K, O, dims):
    for d in dims:
        _same_plan(latent, (1, 2, 2), K, d, overlap_patches=O)


@pytest.mark.parametrize("frames", [49, 81])
@pytest.mark.parametrize("r", [0.5, 1.0])
def test_plan_matches_oracle_with_ratio(frames, r):
    for d in range(3):
        _same_plan((16, 1 + (frames - 1) // 4, 60, 104), (1, 2, 2), 4, d, overlap_ratio=r)


@settings(max_examples=300, deadline=None)
@given(st.tuples(st.integers(1, 4), st.integers(1, 14), st.integers(1, 14), st.integers(1, 14)),
       st.tuples(st.integers(1, 2), st.integers(1, 3), st.integers(1, 3)),
       st.integers(1, 10), st.integers(0, 2), st.integers(0, 8))
def test_plan_matches_oracle_random(npatch, patch, K, dim, O):
    latent = (npatch[0], npatch[1] * patch[0], npatch[2] * patch[1], npatch[3] * patch[2])
    try:
        orc.plan(latent, patch, K, dim, overlap_patches=O)
    except ValueError:
        with pytest.raises(lp.LPError):
            lp.lp_plan_create(latent, patch, K, dim, overlap_patches=O)
        return
    _same_plan(latent, patch, K, dim, overlap_patches=O)


def test_plan_error_codes():
    def status(*a, **kw):
        with pytest.raises(lp.LPError) as e:
            lp.lp_plan_create(*a, **kw)
        return e.value.status
    assert status((16, 5, 15, 16), (1, 2, 2), 2, 1, overlap_patches=1) == lp.LP_ERR_SHAPE
    assert status((16, 5, 16, 16), (1, 0, 2), 2, 1, overlap_patches=1) == lp.LP_ERR_SHAPE
    assert status((16, 5, 16, 16), (1, 2, 2), 0, 1, overlap_patches=1) == lp.LP_ERR_SHAPE          # K < 1
    assert status((16, 5, 16, 16), (1, 2, 2), 2, 3, overlap_patches=1) == lp.LP_ERR_INVALID_ARG    # dim
    assert status((16, 5, 16, 16), (1, 2, 2), 2, 1, overlap_ratio=1.5) == lp.LP_ERR_SHAPE          # r > K - 1
    assert status((16, 5, 16, 16), (1, 2, 2), 2, 1, overlap_patches=5) == lp.LP_ERR_SHAPE          # O > L (K - 1)
    assert status((16, 5, 16, 16), (1, 2, 2), 65, 1, overlap_patches=0) == lp.LP_ERR_SHAPE         # K > LP_MAX_PARTS
    plan = lp.lp_plan_create((16, 5, 16, 16), (1, 2, 2), 2, 1, overlap_patches=1)
    with pytest.raises(lp.LPError):
        lp.lp_plan_query(plan, 2)


def test_device_calls_reject_bad_arguments_without_a_gpu():
    # argument validation happens before any HIP call
    lib = lp._lib()
    plan = lp.lp_plan_create((16, 5, 16, 16), (1, 2, 2), 2, 2, overlap_patches=1)
    assert lib.lp_partition(plan.handle, None, None, None) == lp.LP_ERR_INVALID_ARG
    assert lib.lp_reconstruct(None, 16, 16, None) == lp.LP_ERR_INVALID_ARG
    assert lib.lp_reconstruct_guided_step(plan.handle, 16, None, 1.0, 48, 1.0, 1.0, 64, None) == lp.LP_ERR_INVALID_ARG
    assert lib.lp_reconstruct_guided_step(plan.handle, 16, 32, 1.0, 50, 1.0, 1.0, 64, None) == lp.LP_ERR_INVALID_ARG   # z not float aligned
    other = lp.lp_plan_create((16, 5, 16, 32), (1, 2, 2), 2, 1, overlap_patches=1)                                  # another latent
    assert lib.lp_reconstruct_guided_step_partition(plan.handle, 16, 32, 1.0, 48, 1.0, 1.0, 64, other.handle, 80, None) == lp.LP_ERR_INVALID_ARG
    assert lib.lp_reconstruct_guided_step_partition(plan.handle, 16, 32, 1.0, 48, 1.0, 1.0, 64, None, 80, None) == lp.LP_ERR_INVALID_ARG
    assert lib.lp_attention(16, 32, 48, 64, 10, 4, 96, 384, 96, 0.0, None, 0, None) == lp.LP_ERR_UNSUPPORTED
    assert lib.lp_attention(16, 32, 48, 64, 10, 4, 64, 256, 60, 0.0, None, 0, None) == lp.LP_ERR_INVALID_ARG
    assert lib.lp_attention(16, 32, 48, 8, 10, 4, 64, 256, 64, 0.0, None, 0, None) == lp.LP_ERR_INVALID_ARG
    assert lib.lp_attention(None, None, None, None, 0, 4, 64, 256, 64, 0.0, None, 0, None) == lp.LP_OK
    assert lib.lp_attention(None, None, None, None, -1, 4, 64, 256, 64, 0.0, None, 0, None) == lp.LP_ERR_INVALID_ARG
    assert lib.lp_attention(16, 32, 48, 64, 10, 4, 64, 256, 64, 0.0, 8, 1 << 20, None) == lp.LP_ERR_INVALID_ARG   # workspace alignment
    assert lib.lp_attention(16, 32, 48, 64, 1 << 22, 4, 64, 256, 64, 0.0, None, 0, None) == lp.LP_ERR_UNSUPPORTED  # offsets past 2^31
    # a buffer passed as both input and output is refused (the same address; partial overlaps are the caller's business)
    assert lib.lp_attention(16, 32, 48, 16, 10, 4, 64, 256, 64, 0.0, None, 0, None) == lp.LP_ERR_INVALID_ARG   # o is q
    assert lib.lp_partition(plan.handle, 16, 16, None) == lp.LP_ERR_INVALID_ARG
    assert lib.lp_reconstruct(plan.handle, 16, 16, None) == lp.LP_ERR_INVALID_ARG
    assert lib.lp_reconstruct_guided_step(plan.handle, 16, 32, 1.0, 48, 1.0, 1.0, 32, None) == lp.LP_ERR_INVALID_ARG
    assert lib.lp_attention_workspace_size(96) == lp.LP_ERR_UNSUPPORTED
    # the non-allocating variant checks its arguments the same way, before anything touches a device
    assert lib.lp_attention_static(16, 32, 48, 64, 10, 4, 96, 384, 96, 0.0, None) == lp.LP_ERR_UNSUPPORTED
    assert lib.lp_attention_static(16, 32, 48, 16, 10, 4, 64, 256, 64, 0.0, None) == lp.LP_ERR_INVALID_ARG
    assert lib.lp_attention_static(None, None, None, None, 0, 4, 64, 256, 64, 0.0, None) == lp.LP_OK
    assert lib.lp_attention_static_scratch_bytes() == 2 * 256 * 256 * (128 // 2 + 2) * 4
    # batch: items must not overlap (outer: stride_batch >= one item; inner: fits between token and head strides)
    assert lib.lp_attention_batch(16, 32, 48, 64, 0, 10, 4, 64, 0, 256, 64, 0.0, None, 0, None) == lp.LP_ERR_INVALID_ARG
    assert lib.lp_attention_batch(16, 32, 48, 64, 2, 10, 4, 64, 1280, 256, 64, 0.0, None, 0, None) == lp.LP_ERR_INVALID_ARG
    assert lib.lp_attention_batch(16, 32, 48, 64, 2, 10, 4, 64, 2564, 256, 64, 0.0, None, 0, None) == lp.LP_ERR_INVALID_ARG
    assert lib.lp_attention_batch(None, None, None, None, 2, 0, 4, 64, 2560, 256, 64, 0.0, None, 0, None) == lp.LP_OK


def test_block_calls_reject_bad_arguments_without_a_gpu():
    lib = lp._lib()
    rope = lp.make_rope((1, 1, 4), head_dim=128)
    assert lib.lp_linear(16, 32, None, 48, 4, 100, 128, None) == lp.LP_ERR_UNSUPPORTED        # d_in not a multiple of 64
    assert lib.lp_linear(16, 32, None, 48, 4, 128, 100, None) == lp.LP_ERR_UNSUPPORTED        # d_out not a multiple of 128
    assert lib.lp_linear(16, 32, None, 16, 4, 128, 128, None) == lp.LP_ERR_INVALID_ARG        # y is x
    assert lib.lp_linear(None, None, None, None, 0, 128, 128, None) == lp.LP_OK
    assert lib.lp_qkv_projection(16, 32, None, 48, 64, 1e-6, C.byref(rope), 80, 96, 112, 4, 1, 96, None) == lp.LP_ERR_UNSUPPORTED
    assert lib.lp_qkv_projection(16, 32, None, 48, 64, 1e-6, C.byref(rope), 80, 96, 112, 5, 1, 128, None) == lp.LP_ERR_INVALID_ARG  # grid holds 4 tokens
    bad = lp.make_rope((1, 1, 4), split=(43, 43, 42), head_dim=128)
    assert lib.lp_qkv_projection(16, 32, None, 48, 64, 1e-6, C.byref(bad), 80, 96, 112, 4, 1, 128, None) == lp.LP_ERR_INVALID_ARG   # odd parts
    assert lib.lp_qk_norm_rope(16, 32, 1e-6, C.byref(rope), 4, 1, 128, 128, 100, None) == lp.LP_ERR_INVALID_ARG                     # stride_head < head_dim
