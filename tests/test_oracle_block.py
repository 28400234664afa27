"""Pins for the oracle's DiT-block operations next to attention -- CPU only.

The paper fixes none of the block's internals (Sec. 5.1 says only "30 DiT blocks"); the reading
taken is the common one: y = x W^T + b, per-head RMS normalisation of q and k, 3-D rotary
encoding over the (t, h, w) patch grid.  The oracle's loops are checked here against things
that are not those loops: hand-worked cases, a library matmul, and the identities a
normalisation and a rotation have to satisfy.
"""
import math

import numpy as np
import pytest

from oracle import lp_oracle as orc
from paper_2512_07350_amd import synth


def _bf16(a):
    return synth.f32_to_bf16_bits(np.asarray(a, dtype=np.float32))


# ---- linear

def test_linear_by_hand():
    # x = [[1, 2, 3], [0, -1, 0.5]],  w rows = [1, 0, -1], [2, 2, 2]  (exact in bf16), bias = [0.5, -1]
    x = _bf16([[1, 2, 3], [0, -1, 0.5]])
    w = _bf16([[1, 0, -1], [2, 2, 2]])
    y = orc.linear(x, w, np.array([0.5, -1.0], dtype=np.float32))
    assert y.tolist() == [[1 - 3 + 0.5, 12 - 1], [-0.5 + 0.5, -2 + 1 - 1]]
    # no bias; the weight is [d_out, d_in]: one row per output feature, not the transpose
    assert orc.linear(x, w).tolist() == [[-2.0, 12.0], [-0.5, -1.0]]


@pytest.mark.parametrize("n,d_in,d_out", [(1, 1, 1), (7, 33, 5), (64, 256, 96)])
def test_linear_against_library_matmul(n, d_in, d_out):
    x = synth.f32_to_bf16_bits(synth.normal_f32(11 + n, (n, d_in)))
    w = synth.f32_to_bf16_bits(synth.normal_f32(12 + n, (d_out, d_in)))
    b = synth.normal_f32(13 + n, (d_out,))
    want = synth.bf16_bits_to_f32(x).astype(np.float64) @ synth.bf16_bits_to_f32(w).astype(np.float64).T + b
    got = orc.linear(x, w, b)
    assert np.max(np.abs(got - want)) <= 1e-5 * max(1.0, np.max(np.abs(want)))


# ---- RMS normalisation

def test_rms_norm_by_hand():
    # (3, 4, 0, 0): mean square 25/4, root 5/2 -> (1.2, 1.6, 0, 0); gains (1, 2, 3, 4) -> (1.2, 3.2, 0, 0)
    x = np.array([[[3, 4, 0, 0], [1, 1, 1, 1]]], dtype=np.float32)            # one token, two heads
    g = np.array([[1, 2, 3, 4], [0.5, 0.5, 2, -1]], dtype=np.float32)
    y = orc.rms_norm_heads(x, g, 0.0)
    assert np.allclose(y[0, 0], [1.2, 3.2, 0, 0], rtol=0, atol=1e-7)
    assert np.allclose(y[0, 1], [0.5, 0.5, 2, -1], rtol=0, atol=1e-7)       # a unit-RMS row is only multiplied by the gain
    # eps enters under the root: all-zero row stays zero, (2, 2, 2, 2) with eps = 5 -> 2 / 3
    z = orc.rms_norm_heads(np.array([[[0, 0, 0, 0], [2, 2, 2, 2]]], dtype=np.float32), np.ones((2, 4), np.float32), 5.0)
    assert np.all(z[0, 0] == 0) and np.allclose(z[0, 1], 2.0 / 3.0, atol=1e-7)


def test_rms_norm_invariants():
    n, heads, hd = 9, 3, 64
    x = synth.normal_f32(21, (n, heads, hd))
    g = 1.0 + 0.1 * synth.normal_f32(22, (heads, hd))
    y = orc.rms_norm_heads(x, g, 0.0)
    # dividing the gain back out leaves rows of mean square exactly 1
    assert np.allclose(np.mean((y / g[None]).astype(np.float64) ** 2, axis=-1), 1.0, atol=1e-5)
    # a positive rescaling of the input changes nothing (eps = 0); heads do not mix
    assert np.allclose(orc.rms_norm_heads(7.5 * x, g, 0.0), y, atol=2e-6)
    x2 = x.copy()
    x2[:, 1] *= -3.0
    y2 = orc.rms_norm_heads(x2, g, 0.0)
    assert np.array_equal(y2[:, 0], y[:, 0]) and np.array_equal(y2[:, 2], y[:, 2]) and np.allclose(y2[:, 1], -y[:, 1], atol=2e-6)


# ---- rotary encoding

def test_rope_by_hand_one_pair_per_axis():
    # head_dim 6 split (2, 2, 2): one pair per axis, frequency base^0 = 1, so the angles are the
    # coordinates themselves.  Grid 2 x 3 x 4; token 23 is the last one: (t, h, w) = (1, 2, 3).
    n = 24
    x = np.zeros((n, 1, 6), dtype=np.float32)
    x[23, 0] = [1, 0, 0, 1, 1, 1]
    y = orc.rope3d(x, (2, 3, 4), split=(2, 2, 2))
    want = [math.cos(1), math.sin(1), -math.sin(2), math.cos(2), math.cos(3) - math.sin(3), math.sin(3) + math.cos(3)]
    assert np.allclose(y[23, 0], want, atol=1e-7)
    assert np.all(y[:23] == 0)
    # token 5 = (0, 1, 1): only the h and w pairs turn
    x[:] = 0
    x[5, 0] = [2, 3, 1, 0, 0, 1]
    y = orc.rope3d(x, (2, 3, 4), split=(2, 2, 2))
    assert np.allclose(y[5, 0], [2, 3, math.cos(1), math.sin(1), -math.sin(1), math.cos(1)], atol=1e-7)


def test_rope_by_hand_frequencies_and_offsets():
    # one axis of size 4 (two pairs): frequencies base^0 and base^(-2/4) = 1/100 for base 10000
    x = np.zeros((3, 1, 4), dtype=np.float32)
    x[2, 0] = [1, 0, 1, 0]
    y = orc.rope3d(x, (1, 1, 3), split=(0, 0, 4))                   # token 2 at w = 2
    assert np.allclose(y[2, 0], [math.cos(2), math.sin(2), math.cos(0.02), math.sin(0.02)], atol=1e-7)
    y = orc.rope3d(x, (1, 1, 3), offset=(5, 7, 10), split=(0, 0, 4))  # the same token at w = 12
    assert np.allclose(y[2, 0], [math.cos(12), math.sin(12), math.cos(0.12), math.sin(0.12)], atol=1e-7)
    y = orc.rope3d(x, (1, 1, 3), split=(0, 0, 4), base=16.0)          # base 16: second frequency 1/4
    assert np.allclose(y[2, 0], [math.cos(2), math.sin(2), math.cos(0.5), math.sin(0.5)], atol=1e-7)
    with pytest.raises(ValueError):
        orc.rope3d(x, (1, 1, 3), split=(1, 1, 2))                    # odd parts
    with pytest.raises(ValueError):
        orc.rope3d(x, (1, 1, 4), split=(0, 0, 4))                    # grid does not hold 3 tokens


def test_rope_identities():
    grid, heads, hd = (3, 4, 5), 2, 128
    n = grid[0] * grid[1] * grid[2]
    q = synth.normal_f32(31, (n, heads, hd))
    k = synth.normal_f32(32, (n, heads, hd))
    rq, rk = orc.rope3d(q, grid), orc.rope3d(k, grid)
    # a rotation: every pair keeps its length, the token at the origin is untouched
    pairs = lambda a: a.reshape(n, heads, hd // 2, 2).astype(np.float64)
    assert np.allclose(np.sum(pairs(rq) ** 2, -1), np.sum(pairs(q) ** 2, -1), rtol=1e-6)
    assert np.array_equal(rq[0], q[0])
    # scores depend on the coordinate difference only: shifting both by the same offset changes nothing
    s0 = np.einsum("ihd,jhd->hij", rq.astype(np.float64), rk.astype(np.float64))
    sq, sk = orc.rope3d(q, grid, offset=(4, 9, 2)), orc.rope3d(k, grid, offset=(4, 9, 2))
    s1 = np.einsum("ihd,jhd->hij", sq.astype(np.float64), sk.astype(np.float64))
    assert np.max(np.abs(s0 - s1)) <= 2e-4
    # rotations compose additively: offset a then offset b on a single-token grid = offset a + b
    one = synth.normal_f32(33, (1, heads, hd))
    ab = orc.rope3d(orc.rope3d(one, (1, 1, 1), offset=(1, 2, 3)), (1, 1, 1), offset=(4, 5, 6))
    assert np.allclose(ab, orc.rope3d(one, (1, 1, 1), offset=(5, 7, 9)), atol=2e-6)
    # the default split: height and width 2 floor(d / 6) each, the rest temporal
    assert orc.rope_split(128) == (44, 42, 42) and orc.rope_split(64) == (24, 20, 20)
    # only the temporal part [0, 44) turns when only t differs from the origin
    t_only = orc.rope3d(q, grid)[grid[1] * grid[2]]                   # token (1, 0, 0)
    assert np.array_equal(t_only[:, 44:], q[grid[1] * grid[2], :, 44:]) and not np.array_equal(t_only[:, :44], q[grid[1] * grid[2], :, :44])


# ---- the chain

def test_qkv_block_sections_and_order():
    # weights that make y = (x, 2x, 3x): the first section is q, the second k, the third v; v is neither
    # normalised nor rotated, q and k are normalised (gain differs) and then rotated
    heads, hd = 2, 6
    dm = heads * hd
    grid = (1, 2, 3)
    n = 6
    xf = synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(synth.normal_f32(41, (n, dm))))
    w = np.concatenate([np.eye(dm), 2 * np.eye(dm), 3 * np.eye(dm)]).astype(np.float32)
    gq = np.full((heads, hd), 1.0, np.float32)
    gk = np.full((heads, hd), 0.5, np.float32)
    q, k, v = orc.qkv_block(_bf16(xf), _bf16(w), None, gq, gk, 0.0, heads, hd, grid, split=(2, 2, 2))
    assert np.array_equal(v, (3 * xf).reshape(n, heads, hd))
    want_q = orc.rope3d(orc.rms_norm_heads(xf.reshape(n, heads, hd), gq, 0.0), grid, split=(2, 2, 2))
    assert np.allclose(q, want_q, atol=1e-6)
    assert np.allclose(k, 0.5 * want_q, atol=1e-6)       # normalisation removes the factor 2, the gain halves
    # a bias on the v section only moves v
    b = np.zeros(3 * dm, np.float32)
    b[2 * dm:] = 1.0
    q2, k2, v2 = orc.qkv_block(_bf16(xf), _bf16(w), b, gq, gk, 0.0, heads, hd, grid, split=(2, 2, 2))
    assert np.array_equal(q2, q) and np.array_equal(k2, k) and np.array_equal(v2, v + 1.0)
