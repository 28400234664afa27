"""The DiT-block operations next to attention on the GPU against the CPU oracle.

Tolerance.  The HIP path accumulates bf16 products in binary32 and rounds its result to bf16
once, on store; the oracle evaluates the same definition in binary64.  With at most 5120 terms of
magnitude <= 1 the binary32 accumulation error stays below 1e-4 absolute, the hardware sine /
cosine of the fractional turn count below 1e-5, and the final rounding is half a bf16 unit in the
last place, 2^-9 relative.  Bound used: |got - want| <= 2^-8 |want| + 3e-4 (inputs scaled so that
results are O(1)).
"""
import numpy as np
import pytest

from oracle import lp_oracle as orc
from paper_2512_07350_amd import synth

pytestmark = pytest.mark.gpu

REL, ABS = 2.0 ** -8, 3e-4


def _close(got, want, what=""):
    got, want = np.asarray(got, np.float64), np.asarray(want, np.float64)
    assert got.shape == want.shape, what
    assert np.all(np.isfinite(got)), what
    excess = np.abs(got - want) - (REL * np.abs(want) + ABS)
    assert excess.max() <= 0, (what, float(excess.max()), float(np.abs(got - want).max()))


def _bits(seed, shape, scale=1.0):
    return synth.f32_to_bf16_bits(np.float32(scale) * synth.normal_f32(seed, shape))


def _dev(a):
    import torch
    a = np.ascontiguousarray(a)
    return torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a).cuda()


def _bf16_out(shape):
    import torch
    return torch.full(shape, float("nan"), dtype=torch.bfloat16, device="cuda")


def _linear(x, w, bias):
    import torch
    from tests import gpu_util as g
    from paper_2512_07350_amd import binding as lp
    n, d_in = x.shape
    d_out = w.shape[0]
    y = _bf16_out((n, d_out))
    lp.lp_linear(_dev(x), _dev(w), None if bias is None else _dev(bias), y, n, d_in, d_out, g.stream())
    torch.cuda.synchronize()
    return g.from_dev_bf16(y)


@pytest.mark.parametrize("n,d_in,d_out,with_bias", [
    (1, 64, 128, True), (33, 128, 128, False), (257, 192, 384, True), (300, 1536, 1536, True), (520, 5120, 640, True),
])
def test_linear_matches_oracle(n, d_in, d_out, with_bias):
    x = _bits(100 + n, (n, d_in))
    w = _bits(200 + n, (d_out, d_in), scale=d_in ** -0.5)
    b = synth.normal_f32(300 + n, (d_out,)) if with_bias else None
    _close(_linear(x, w, b), orc.linear(x, w, b), "linear %dx%d->%d" % (n, d_in, d_out))


def _qkv(x, w, bias, gq, gk, eps, heads, hd, grid, offset, split, base):
    import torch
    from tests import gpu_util as g
    from paper_2512_07350_amd import binding as lp
    n = x.shape[0]
    q, k, v = (_bf16_out((n, heads, hd)) for _ in range(3))
    rope = lp.make_rope(grid, offset, split, base, head_dim=hd)
    lp.lp_qkv_projection(_dev(x), _dev(w), None if bias is None else _dev(bias), _dev(gq), _dev(gk), eps, rope, q, k, v,
                         n, heads, hd, g.stream())
    torch.cuda.synchronize()
    return tuple(g.from_dev_bf16(t) for t in (q, k, v))


@pytest.mark.parametrize("heads,hd,grid,offset,split,base,with_bias", [
    (2, 64, (2, 5, 7), (0, 0, 0), None, 10000.0, True),          # two heads of 64 in one wave tile
    (4, 64, (1, 1, 1), (3, 4, 5), (24, 20, 20), 10000.0, False),  # a single token placed by its offset
    (1, 128, (3, 4, 30), (0, 7, 2), None, 10000.0, True),        # 360 tokens: a ragged second token tile
    (12, 128, (3, 10, 13), (5, 0, 11), None, 10000.0, True),     # the 1.3B-shaped block: d_model 1536
    (3, 128, (2, 3, 50), (0, 0, 0), (128, 0, 0), 100.0, True),   # all of head_dim on one axis, another base
])
def test_qkv_projection_matches_oracle(heads, hd, grid, offset, split, base, with_bias):
    dm = heads * hd
    n = grid[0] * grid[1] * grid[2]
    x = _bits(400 + n, (n, dm))
    w = _bits(500 + n, (3 * dm, dm), scale=dm ** -0.5)
    b = 0.5 * synth.normal_f32(600 + n, (3 * dm,)) if with_bias else None
    gq = 1.0 + 0.2 * synth.normal_f32(700 + n, (heads, hd))
    gk = 1.0 + 0.2 * synth.normal_f32(800 + n, (heads, hd))
    eps = 1e-6
    want = orc.qkv_block(x, w, b, gq, gk, eps, heads, hd, grid, offset, split, base)
    got = _qkv(x, w, b, gq, gk, eps, heads, hd, grid, offset, split, base)
    for name, a, e in zip("qkv", got, want):
        _close(a, e, "%s heads=%d hd=%d grid=%s" % (name, heads, hd, grid))


def test_qkv_projection_at_benchmark_size_sampled_tokens():
    """The 1.3B-shaped block over one 720p-wide sub-latent's token count (13230 = 21 x 45 x 14): the
    oracle evaluates 256 sampled tokens, each placed by its own coordinates."""
    heads, hd, grid = 12, 128, (21, 45, 14)
    dm, n = heads * hd, 21 * 45 * 14
    x = _bits(901, (n, dm))
    w = _bits(902, (3 * dm, dm), scale=dm ** -0.5)
    b = 0.5 * synth.normal_f32(903, (3 * dm,))
    gq = 1.0 + 0.2 * synth.normal_f32(904, (heads, hd))
    gk = 1.0 + 0.2 * synth.normal_f32(905, (heads, hd))
    got = _qkv(x, w, b, gq, gk, 1e-6, heads, hd, grid, (0, 0, 8), None, 10000.0)
    assert all(np.all(np.isfinite(a)) for a in got)
    rows = synth.sample_rows(n, 256, seed=9, tile=256)
    for r in rows:
        t, h, wv = r // (45 * 14), (r // 14) % 45, r % 14
        want = orc.qkv_block(x[r:r + 1], w, b, gq, gk, 1e-6, heads, hd, (1, 1, 1), (t, h, wv + 8), None, 10000.0)
        for name, a, e in zip("qkv", got, want):
            _close(a[r:r + 1], e, "%s token %d" % (name, r))


def test_block_at_headline_size_sampled_tokens():
    """The 40-head block (d_model 5120) over the headline workload's largest sub-latent (13230 tokens):
    QKV projection with normalisation and rotation, then the output projection of a seeded o, each on
    96 sampled tokens (every 256-token tile edge among the first and last tiles, plus random ones)."""
    heads, hd, grid = 40, 128, (21, 45, 14)
    dm, n = heads * hd, 21 * 45 * 14
    x = _bits(911, (n, dm))
    w = _bits(912, (3 * dm, dm), scale=dm ** -0.5)
    b = 0.5 * synth.normal_f32(913, (3 * dm,))
    gq = 1.0 + 0.2 * synth.normal_f32(914, (heads, hd))
    gk = 1.0 + 0.2 * synth.normal_f32(915, (heads, hd))
    got = _qkv(x, w, b, gq, gk, 1e-6, heads, hd, grid, (0, 0, 8), None, 10000.0)
    assert all(np.all(np.isfinite(a)) for a in got)
    rows = synth.sample_rows(n, 96, seed=19, tile=256)
    for r in rows:
        t, h, wv = r // (45 * 14), (r // 14) % 45, r % 14
        want = orc.qkv_block(x[r:r + 1], w, b, gq, gk, 1e-6, heads, hd, (1, 1, 1), (t, h, wv + 8), None, 10000.0)
        for name, a, e in zip("qkv", got, want):
            _close(a[r:r + 1], e, "%s token %d" % (name, r))
    w_o = w[:dm]
    y = _linear(x, w_o, b[:dm])
    assert np.all(np.isfinite(y))
    _close(y[rows], orc.linear(x[rows], w_o, b[:dm]), "output projection, sampled tokens")


@pytest.mark.parametrize("hd", [64, 128])
def test_qk_norm_rope_in_place_with_padded_strides(hd):
    import torch
    from tests import gpu_util as g
    from paper_2512_07350_amd import binding as lp
    heads, grid, offset = 3, (2, 3, 11), (1, 0, 4)
    n = grid[0] * grid[1] * grid[2]
    xb = _bits(1000 + hd, (n, heads, hd), scale=3.0)
    gain = 1.0 + 0.3 * synth.normal_f32(1001 + hd, (heads, hd))
    stride_head, stride_tok = hd + 8, heads * (hd + 8) + 16
    buf = np.zeros(n * stride_tok + 8, dtype=np.uint16)
    idx = (np.arange(n)[:, None, None] * stride_tok + np.arange(heads)[None, :, None] * stride_head + np.arange(hd)[None, None, :])
    buf[idx] = xb
    marker = synth.f32_to_bf16_bits(np.float32([123.0]))[0]
    pad = np.ones(buf.shape, dtype=bool)
    pad[idx] = False
    buf[pad] = marker
    d = g.to_dev_bf16(buf)
    rope = lp.make_rope(grid, offset, None, 10000.0, head_dim=hd)
    lp.lp_qk_norm_rope(d, _dev(gain), 1e-5, rope, n, heads, hd, stride_tok, stride_head, g.stream())
    torch.cuda.synchronize()
    out = g.from_dev_bf16(d)
    want = orc.rope3d(orc.rms_norm_heads(synth.bf16_bits_to_f32(xb), gain, 1e-5), grid, offset)
    _close(out[idx], want, "norm+rope hd=%d" % hd)
    assert np.all(out[pad] == 123.0)          # nothing outside the rows was touched


def test_block_chain_projection_attention_projection():
    """x -> q, k, v (projection, normalisation, rotation) -> attention -> output projection, every
    stage on the GPU, against the same chain on the oracle (which hands bf16-rounded q, k, v and o
    from stage to stage, as the HIP path stores them)."""
    import torch
    from tests import gpu_util as g
    from paper_2512_07350_amd import binding as lp
    heads, hd, grid = 4, 128, (2, 6, 25)
    dm, n = heads * hd, 2 * 6 * 25
    x = _bits(1101, (n, dm))
    w_qkv = _bits(1102, (3 * dm, dm), scale=dm ** -0.5)
    w_o = _bits(1103, (dm, dm), scale=dm ** -0.5)
    b_o = synth.normal_f32(1104, (dm,))
    gq = 1.0 + 0.2 * synth.normal_f32(1105, (heads, hd))
    gk = 1.0 + 0.2 * synth.normal_f32(1106, (heads, hd))
    # oracle chain
    q, k, v = (synth.f32_to_bf16_bits(a) for a in orc.qkv_block(x, w_qkv, None, gq, gk, 1e-6, heads, hd, grid))
    o = synth.f32_to_bf16_bits(orc.attention(q, k, v))
    want = orc.linear(o.reshape(n, dm), w_o, b_o)
    # HIP chain, device resident
    qd, kd, vd = (_bf16_out((n, heads, hd)) for _ in range(3))
    od, yd = _bf16_out((n, heads, hd)), _bf16_out((n, dm))
    rope = lp.make_rope(grid, head_dim=hd)
    ws, ws_bytes = g.workspace(hd)
    st = g.stream()
    lp.lp_qkv_projection(_dev(x), _dev(w_qkv), None, _dev(gq), _dev(gk), 1e-6, rope, qd, kd, vd, n, heads, hd, st)
    lp.lp_attention(qd, kd, vd, od, n, heads, hd, heads * hd, hd, 0.0, ws, ws_bytes, st)
    lp.lp_linear(od, _dev(w_o), _dev(b_o), yd, n, dm, dm, st)
    torch.cuda.synchronize()
    got = g.from_dev_bf16(yd)
    assert np.all(np.isfinite(got))
    # the attention stage carries the attention tolerance (2e-2 / 2e-3 on O(1/sqrt(n)) outputs); the output
    # projection of rows of that size keeps the error at the same absolute level
    err = np.abs(got - want)
    assert err.max() <= 2e-2 and err.mean() <= 2e-3, (float(err.max()), float(err.mean()))
