"""lp_attention on the GPU against the CPU oracle.

Tolerance (stated by the task for N(0,1) inputs, bf16 products, fp32 softmax):
max-abs <= 2e-2 and mean-abs <= 2e-3 against the oracle's fp32 output.
"""
import numpy as np
import pytest

from oracle import lp_oracle as orc
from paper_2512_07350_amd import synth

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("balanced", [True, False], ids=["balanced", "tile-per-workgroup"])
@pytest.mark.parametrize("hd", [64, 128])
@pytest.mark.parametrize("n", [1, 2, 31, 32, 33, 63, 64, 65, 95, 96, 97, 127, 128, 129, 200, 255, 256, 257, 320, 513, 1000])
def test_small_full_oracle(n, hd, balanced):
    from tests import gpu_util as g
    heads = 3
    q, k, v = synth.qkv_bf16(4000 + 2 * n + hd, n, heads, hd)
    got = g.hip_attention(q, k, v, balanced=balanced)
    want = orc.attention(q, k, v)
    g.assert_attention_close(got, want, "n=%d hd=%d" % (n, hd))


@pytest.mark.parametrize("n,heads,hd", [(3000, 1, 128), (2048, 2, 128), (700, 5, 64), (5000, 7, 64), (64, 40, 128)])
def test_work_split_across_workgroups(n, heads, hd):
    """Few (query tile, head) units: with a workspace every unit is shared by several
    workgroups and the merge kernel produces the output; must agree with the oracle and
    with the unsplit launch."""
    from tests import gpu_util as g
    q, k, v = synth.qkv_bf16(9000 + n + heads, n, heads, hd)
    rows = synth.sample_rows(n, 160, seed=n, tile=256)
    want = orc.attention(q, k, v, rows=rows)
    split = g.hip_attention(q, k, v, balanced=True)
    plain = g.hip_attention(q, k, v, balanced=False)
    g.assert_attention_close(split[rows], want, "split n=%d" % n)
    g.assert_attention_close(plain[rows], want, "plain n=%d" % n)
    assert np.all(np.isfinite(split)) and np.all(np.isfinite(plain))
    assert np.max(np.abs(split - plain)) <= 2e-2


@pytest.mark.parametrize("layout", ["outer", "inner"])
@pytest.mark.parametrize("balanced", [True, False], ids=["balanced", "tile-per-workgroup"])
@pytest.mark.parametrize("n,heads,hd,batch", [(1000, 3, 128, 2), (333, 2, 64, 3), (64, 1, 128, 2), (1, 2, 64, 2)])
def test_batch_items_are_independent_calls(n, heads, hd, batch, balanced, layout):
    """lp_attention_batch (the conditional / unconditional pair of Eq. 4 is batch = 2): every item
    against the oracle on that item alone."""
    from tests import gpu_util as g
    items = [synth.qkv_bf16(7000 + 10 * n + b, n, heads, hd) for b in range(batch)]
    got = g.hip_attention_batch(items, balanced=balanced, layout=layout)
    for b, (q, k, v) in enumerate(items):
        g.assert_attention_close(got[b], orc.attention(q, k, v), "n=%d item %d %s" % (n, b, layout))


def test_batch_pair_at_benchmark_size_sampled_rows():
    # the 33-frame H partition of 4212 tokens, 12 x 128, as a conditional / unconditional pair
    from tests import gpu_util as g
    n, heads, hd = 4212, 12, 128
    items = [synth.qkv_bf16(synth.seed_for(1, 1, 0, tensor=20 + b), n, heads, hd) for b in range(2)]
    got = g.hip_attention_batch(items)
    rows = synth.sample_rows(n, 256, seed=5, tile=256)
    for b, (q, k, v) in enumerate(items):
        g.assert_attention_close(got[b][rows], orc.attention(q, k, v, rows=rows), "pair item %d" % b)
        assert np.all(np.isfinite(got[b]))
    # and an item of the pair agrees with the same item computed alone
    alone = g.hip_attention(*items[1])
    assert np.max(np.abs(alone - got[1])) <= 2e-2


def test_tiny_config_partitions_full_oracle():
    # tiny config: 2 partitions of 200 tokens, 4 heads x 64
    from tests import gpu_util as g
    for k_part in range(2):
        q, k, v = synth.qkv_bf16(synth.seed_for(0, 2, k_part), 200, 4, 64)
        g.assert_attention_close(g.hip_attention(q, k, v), orc.attention(q, k, v), "tiny k=%d" % k_part)


@pytest.mark.parametrize("balanced", [True, False], ids=["balanced", "tile-per-workgroup"])
def test_medium_full_oracle_spans_many_tiles(balanced):
    # 3276 tokens (the smallest 33-frame partition along H), all rows, 2 heads
    from tests import gpu_util as g
    q, k, v = synth.qkv_bf16(77, 3276, 2, 128)
    g.assert_attention_close(g.hip_attention(q, k, v, balanced=balanced), orc.attention(q, k, v), "n=3276")


def test_explicit_scale_and_default_scale():
    from tests import gpu_util as g
    q, k, v = synth.qkv_bf16(78, 300, 2, 128)
    g.assert_attention_close(g.hip_attention(q, k, v, scale=0.05), orc.attention(q, k, v, scale=0.05), "scale=.05")
    a = g.hip_attention(q, k, v, scale=0.0)
    b = g.hip_attention(q, k, v, scale=float(1.0 / np.sqrt(128.0)))
    assert np.array_equal(a, b)


def test_special_cases():
    from tests import gpu_util as g
    n, hd = 300, 64
    q, k, v = synth.qkv_bf16(79, n, 2, hd)
    vf = synth.bf16_bits_to_f32(v)
    # zero queries -> uniform softmax -> column mean of V
    q0 = np.zeros_like(q)
    got = g.hip_attention(q0, k, v)
    assert np.max(np.abs(got - vf.mean(axis=0)[None])) < 1e-2
    # identical value rows -> that row exactly (softmax weights sum to one; bf16 of a bf16 value)
    v1 = np.broadcast_to(v[7:8], v.shape).copy()
    got = g.hip_attention(q, k, v1)
    assert np.max(np.abs(got - synth.bf16_bits_to_f32(v1))) <= 2 ** -7 * np.max(np.abs(vf))
    # one dominant key -> its value row
    big = synth.f32_to_bf16_bits(np.full((hd,), 8.0, dtype=np.float32))
    q2, k2 = q.copy(), k.copy()
    q2[:] = big
    k2[5, :] = big
    got = g.hip_attention(q2, k2, v)
    assert np.max(np.abs(got - vf[5][None])) < 1e-6
    # large logits must not overflow: scores of magnitude ~ 4096
    k3 = np.broadcast_to(big, k.shape).copy()
    got = g.hip_attention(q2, k3, v)
    assert np.all(np.isfinite(got))
    assert np.max(np.abs(got - vf.mean(axis=0)[None])) < 1e-2


def test_head_major_strides_and_in_place_views():
    # same data laid out [heads, n, d]: stride_tok = d, stride_head = n*d
    from tests import gpu_util as g
    import torch
    from paper_2512_07350_amd import binding as lp
    n, heads, hd = 333, 3, 128
    q, k, v = synth.qkv_bf16(80, n, heads, hd)
    want = g.hip_attention(q, k, v)
    qd, kd, vd = (g.to_dev_bf16(np.ascontiguousarray(a.transpose(1, 0, 2))) for a in (q, k, v))
    od = torch.zeros((heads, n, hd), dtype=torch.bfloat16, device="cuda")
    lp.lp_attention(qd, kd, vd, od, n, heads, hd, hd, n * hd, 0.0, None, 0, g.stream())
    torch.cuda.synchronize()
    got = g.from_dev_bf16(od).transpose(1, 0, 2)
    assert np.array_equal(got, g.hip_attention(q, k, v, balanced=False))
    ws, ws_bytes = g.workspace(hd)
    lp.lp_attention(qd, kd, vd, od, n, heads, hd, hd, n * hd, 0.0, ws, ws_bytes, g.stream())
    torch.cuda.synchronize()
    assert np.array_equal(g.from_dev_bf16(od).transpose(1, 0, 2), want)


def test_zero_tokens_is_a_noop():
    from paper_2512_07350_amd import binding as lp
    lp.lp_attention(0, 0, 0, 0, 0, 4, 64, 256, 64)


# rows the oracle evaluates per partition (each over all keys and all heads) at the full sizes
FULL_SIZE_ROWS = 256

# (workload index, partition dim): every partition of these is checked on sampled rows --
# the rotating 33-frame workload, the 81-frame H step, and the T and W steps of the 81-frame loop
FULL_SIZE = [(1, 0), (1, 1), (1, 2), (2, 1), (4, 0), (4, 2)]


def _check_partition_sampled(cfg, dim, kp, n, w, seed):
    from tests import gpu_util as g
    q, k, v = synth.qkv_bf16(synth.seed_for(cfg, dim, kp), n, w.heads, w.head_dim)
    got = g.hip_attention(q, k, v)
    rows = synth.sample_rows(n, FULL_SIZE_ROWS, seed=seed, tile=256)
    assert len(rows) >= min(FULL_SIZE_ROWS, n)
    want = orc.attention(q, k, v, rows=rows)
    g.assert_attention_close(got[rows], want, "cfg%d %s k=%d n=%d" % (cfg, synth.DIM_NAMES[dim], kp, n))
    assert np.all(np.isfinite(got))


@pytest.mark.parametrize("cfg,dim", FULL_SIZE)
def test_full_size_partitions_sampled_rows(cfg, dim):
    """Benchmark shapes, in the launch configuration the benchmark times; the oracle
    evaluates sampled query rows (each over all keys)."""
    w = synth.WORKLOADS[cfg]
    pl = orc.plan(w.latent, w.patch, w.K, dim, **w.overlap_args())
    for kp, part in enumerate(pl.parts):
        if part.n_tokens:
            _check_partition_sampled(cfg, dim, kp, part.n_tokens, w, seed=kp + 10 * dim)


@pytest.mark.parametrize("cfg", [7, 8, 9, 10])
def test_device_count_sweep_temporal_only_and_long_clip_shapes_sampled_rows(cfg):
    """81 frames with K = 2, K = 8 and the temporal-only variant, and the 10-second clip (161
    frames, r = 0.5, sub-latents of up to 34112 tokens): along every dimension the workload
    visits, its largest sub-latent and its last non-empty one (the odd-sized one)."""
    w = synth.WORKLOADS[cfg]
    for dim in sorted(set(w.dims)):
        pl = orc.plan(w.latent, w.patch, w.K, dim, **w.overlap_args())
        sizes = [p.n_tokens for p in pl.parts]
        picks = {int(np.argmax(sizes)), max(i for i, n in enumerate(sizes) if n)}
        for kp in sorted(picks):
            _check_partition_sampled(cfg, dim, kp, sizes[kp], w, seed=cfg + kp)


def test_full_sequence_K1_sampled_rows():
    # the non-LP comparison of the 81-frame config: all 32760 tokens in one sequence
    w = synth.WORKLOADS[2]
    n = orc.plan(w.latent, w.patch, 1, 1, overlap_patches=0).parts[0].n_tokens
    assert n == 32760
    _check_partition_sampled(2, 1, 15, n, w, seed=5)


def test_14b_shape_sampled_rows():
    # 720p, 40 heads (the benchmark's default workload): the first partition (11340 tokens),
    # an interior one (13230) and the last
    w = synth.WORKLOADS[3]
    pl = orc.plan(w.latent, w.patch, w.K, 2, **w.overlap_args())
    for kp in (0, 3, w.K - 1):
        _check_partition_sampled(3, 2, kp, pl.parts[kp].n_tokens, w, seed=kp)


def test_random_shapes_and_layouts():
    """Seeded random token counts, head counts, head dims, batch sizes and padded strides, in both
    launch modes; every item against the oracle on all rows."""
    from tests import gpu_util as g
    import torch
    from paper_2512_07350_amd import binding as lp
    rng = np.random.default_rng(7350)
    for case in range(24):
        n = int(rng.choice([rng.integers(1, 70), rng.integers(70, 700), rng.integers(700, 2600)]))
        heads = int(rng.integers(1, 6))
        hd = int(rng.choice([64, 128]))
        batch = int(rng.integers(1, 4))
        balanced = bool(rng.integers(0, 2))
        scale = float(rng.choice([0.0, 0.03, 0.25]))   # 0 selects 1/sqrt(head_dim)
        pad_h = 8 * int(rng.integers(0, 3))            # gap between heads of a token
        pad_t = 8 * int(rng.integers(0, 3))            # gap between tokens
        stride_head = hd + pad_h
        stride_tok = heads * stride_head + pad_t
        stride_batch = n * stride_tok + 8 * int(rng.integers(0, 5))
        items = [synth.qkv_bf16(60000 + 10 * case + b, n, heads, hd) for b in range(batch)]
        total = batch * stride_batch + 64

        def pack(j):
            buf = np.zeros(total, dtype=np.uint16)
            for b, it in enumerate(items):
                for h in range(heads):
                    idx = (b * stride_batch + np.arange(n)[:, None] * stride_tok + h * stride_head + np.arange(hd)[None, :])
                    buf[idx] = it[j][:, h, :]
            return g.to_dev_bf16(buf)

        qd, kd, vd = pack(0), pack(1), pack(2)
        od = torch.full((total,), float("nan"), dtype=torch.bfloat16, device="cuda")
        ws, ws_bytes = g.workspace(hd) if balanced else (None, 0)
        lp.lp_attention_batch(qd, kd, vd, od, batch, n, heads, hd, stride_batch, stride_tok, stride_head, scale,
                              ws, ws_bytes, g.stream())
        torch.cuda.synchronize()
        out = g.from_dev_bf16(od)
        written = np.zeros(total, dtype=bool)
        for b, (q, k, v) in enumerate(items):
            want = orc.attention(q, k, v, scale=scale if scale > 0 else None)
            for h in range(heads):
                idx = (b * stride_batch + np.arange(n)[:, None] * stride_tok + h * stride_head + np.arange(hd)[None, :])
                written[idx] = True
                g.assert_attention_close(out[idx], want[:, h, :], "case %d item %d head %d n=%d hd=%d" % (case, b, h, n, hd),
                                         sharpness=scale * np.sqrt(hd))
        # nothing outside the rows of O was touched
        assert np.all(np.isnan(out[~written])), "case %d wrote outside its rows" % case


@pytest.mark.parametrize("balanced", [True, False], ids=["balanced", "tile-per-workgroup"])
def test_scores_that_keep_rising_along_the_keys(balanced):
    """Keys ordered so that the scores grow by about two octaves from one 32-key round to the
    next: the running maximum has to be raised (and the accumulated output rescaled) over and
    over, across tiles and across the parts of a query tile that different workgroups compute."""
    from tests import gpu_util as g
    n, heads, hd = 1500, 2, 128
    rng = np.random.default_rng(99)
    base = rng.standard_normal((heads, hd)).astype(np.float32)
    base /= np.linalg.norm(base, axis=1, keepdims=True)
    qf = np.broadcast_to(base[None] * np.float32(np.sqrt(hd)) * 4.0, (n, heads, hd)) + 0.05 * rng.standard_normal((n, heads, hd)).astype(np.float32)
    ramp = (np.arange(n, dtype=np.float32) / 32.0 * 0.35)[:, None, None]       # log-score slope per round, before scale
    kf = base[None] * ramp + 0.05 * rng.standard_normal((n, heads, hd)).astype(np.float32)
    vf = rng.standard_normal((n, heads, hd)).astype(np.float32)
    q, k, v = (synth.f32_to_bf16_bits(a) for a in (qf, kf, vf))
    got = g.hip_attention(q, k, v, balanced=balanced)
    want = orc.attention(q, k, v)
    g.assert_attention_close(got, want, "rising scores")
    # and the same keys in reverse order (the first round already holds the maximum)
    got_r = g.hip_attention(q, k[::-1].copy(), v[::-1].copy(), balanced=balanced)
    g.assert_attention_close(got_r, want, "falling scores")


@pytest.mark.parametrize("balanced", [True, False], ids=["balanced", "tile-per-workgroup"])
@pytest.mark.parametrize("hd", [64, 128])
@pytest.mark.parametrize("profile", ["ramp", "cliff"])
def test_scores_far_above_the_first_round(balanced, hd, profile):
    """Scores that climb 8 log2 units per 32-key round up to 2^256 times the first round's level
    and stay there ("ramp"), or get there in one step ("cliff"): exp2 of a score relative to the first round's maximum overflows
    binary32, which the kernel has to notice and recover from (it repeats the segment with the
    running-maximum check).  Every operand is exactly representable, the scale is chosen so that
    the pre-scaled queries are too, so the stated tolerance applies unchanged."""
    from tests import gpu_util as g
    n, heads = 1500, 2
    rng = np.random.default_rng(1234)
    base = np.where(rng.random((heads, hd)) < 0.5, -1.0, 1.0).astype(np.float32)       # q . k = hd * (q level) * (k level)
    if profile == "ramp":
        level = np.minimum(np.floor(np.arange(n) / 32.0), 32.0).astype(np.float32)      # 0, 1, ..., 32, 32, ...
    else:                                            # one step of 2^256 inside the second round: also met by a
        level = np.where(np.arange(n) < 40, 0.0, 32.0).astype(np.float32)   # workgroup that holds only the first tiles
    qf = np.broadcast_to(base[None] * np.float32(64.0 / hd), (n, heads, hd)).copy()
    kf = base[None] * level[:, None, None]
    vf = rng.standard_normal((n, heads, hd)).astype(np.float32)
    q, k, v = (synth.f32_to_bf16_bits(a) for a in (qf, kf, vf))
    scale = 0.125 / np.log2(np.e)                    # scores in log2 units: 64 * level * 0.125 = 8 * level
    got = g.hip_attention(q, k, v, scale=scale, balanced=balanced)
    want = orc.attention(q, k, v, scale=scale)
    g.assert_attention_close(got, want, "scores far above the first round")
    plateau = synth.bf16_bits_to_f32(v)[level == 32.0].mean(axis=0)
    assert np.max(np.abs(want[700] - plateau)) < 1e-2          # the oracle itself: the plateau's keys carry the weight

