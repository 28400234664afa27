"""Pins for the oracle's attention -- CPU only.

The oracle's loops are compared with things that are not those loops: a
library softmax + matmul on tiny inputs, closed-form special cases, and
symmetries of the definition.
"""
import numpy as np
import pytest
from scipy.special import softmax

from oracle import lp_oracle as orc
from paper_2512_07350_amd import synth


def _lib_attention(q, k, v, scale):
    """softmax(scale q k^T) v per head with numpy/scipy routines in fp64."""
    qf, kf, vf = (synth.bf16_bits_to_f32(a).astype(np.float64) for a in (q, k, v))
    s = np.einsum("ihd,jhd->hij", qf, kf) * scale
    p = softmax(s, axis=-1)
    return np.einsum("hij,jhd->ihd", p, vf)


@pytest.mark.parametrize("n", [1, 2, 63, 64, 65, 200])
@pytest.mark.parametrize("hd", [64, 128])
def test_against_library_softmax_matmul(n, hd):
    q, k, v = synth.qkv_bf16(1000 + n + hd, n, 3, hd)
    got = orc.attention(q, k, v)
    want = _lib_attention(q, k, v, 1.0 / np.sqrt(hd))
    assert got.shape == (n, 3, hd)
    assert np.max(np.abs(got - want)) < 2e-6


def test_explicit_scale_and_rows_subset():
    q, k, v = synth.qkv_bf16(5, 150, 2, 64)
    full = orc.attention(q, k, v, scale=0.3)
    assert np.max(np.abs(full - _lib_attention(q, k, v, 0.3))) < 2e-6
    rows = [149, 0, 77, 77, 3]
    sub = orc.attention(q, k, v, scale=0.3, rows=rows)
    assert np.array_equal(sub, full[rows])
    with pytest.raises(IndexError):
        orc.attention(q, k, v, rows=[150])


def test_zero_queries_give_column_mean_of_v():
    q, k, v = synth.qkv_bf16(6, 97, 2, 64)
    q[:] = 0
    got = orc.attention(q, k, v)
    mean = synth.bf16_bits_to_f32(v).astype(np.float64).mean(axis=0)
    assert np.max(np.abs(got - mean[None])) < 1e-6


def test_identical_keys_give_column_mean_of_v():
    q, k, v = synth.qkv_bf16(7, 50, 2, 64)
    k[:] = k[0:1]
    got = orc.attention(q, k, v)
    mean = synth.bf16_bits_to_f32(v).astype(np.float64).mean(axis=0)
    assert np.max(np.abs(got - mean[None])) < 1e-6


def test_identical_values_and_single_token():
    q, k, v = synth.qkv_bf16(8, 40, 2, 128)
    v[:] = v[3:4]
    got = orc.attention(q, k, v)
    assert np.array_equal(got, np.broadcast_to(synth.bf16_bits_to_f32(v[3]), got.shape))
    q1, k1, v1 = synth.qkv_bf16(9, 1, 4, 64)
    assert np.array_equal(orc.attention(q1, k1, v1), synth.bf16_bits_to_f32(v1))


def test_dominant_key_selects_its_value_row():
    n, hd = 33, 64
    q, k, v = synth.qkv_bf16(10, n, 1, hd)
    big = synth.f32_to_bf16_bits(np.full((hd,), 8.0, dtype=np.float32))
    q[:] = big                       # q . k_5 = 64 * 64 = 4096 >> any other score
    k[5, 0] = big
    got = orc.attention(q, k, v)
    assert np.max(np.abs(got - synth.bf16_bits_to_f32(v[5])[None])) < 1e-6


def test_key_permutation_invariance_and_head_independence():
    q, k, v = synth.qkv_bf16(12, 120, 3, 64)
    base = orc.attention(q, k, v)
    perm = np.random.Generator(np.random.Philox(3)).permutation(120)
    got = orc.attention(q, np.ascontiguousarray(k[perm]), np.ascontiguousarray(v[perm]))
    assert np.max(np.abs(got - base)) < 1e-6
    # head h of the result depends on head h of the inputs only
    k2, v2 = k.copy(), v.copy()
    k2[:, 1] = k[::-1, 1]
    v2[:, 1] = 0
    got2 = orc.attention(q, k2, v2)
    assert np.array_equal(got2[:, 0], base[:, 0]) and np.array_equal(got2[:, 2], base[:, 2])
    assert np.array_equal(got2[:, 1], np.zeros_like(got2[:, 1]))


def test_output_rows_are_convex_combinations():
    q, k, v = synth.qkv_bf16(13, 80, 2, 64)
    got = orc.attention(q, k, v)
    vf = synth.bf16_bits_to_f32(v)
    assert np.all(got <= vf.max(axis=0)[None] + 1e-6) and np.all(got >= vf.min(axis=0)[None] - 1e-6)
    # values all equal to one => row sums of the softmax are 1
    v[:] = synth.f32_to_bf16_bits(np.ones(1, dtype=np.float32))[0]
    assert np.max(np.abs(orc.attention(q, k, v) - 1.0)) < 1e-6


def test_bf16_helpers_round_to_nearest_even():
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 3.1415927, 0.0], dtype=np.float32)
    # 1 + 2^-8 is a tie between 1.0 and 1 + 2^-7 -> even mantissa (1.0); 1 + 3*2^-8 ties up to 1 + 2^-6
    b = synth.f32_to_bf16_bits(x)
    back = synth.bf16_bits_to_f32(b)
    assert back[0] == 1.0 and back[1] == 1.0 and back[2] == 1.015625 and back[3] == -2.5
    assert abs(back[4] - 3.1415927) < 2 ** -7 and back[5] == 0.0
