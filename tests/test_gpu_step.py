"""One whole LP step on the GPU (partition -> attention per sub-latent -> reconstruct)
against the same chain on the oracle."""
import numpy as np
import pytest

from oracle import lp_oracle as orc
from paper_2512_07350_amd import synth

pytestmark = pytest.mark.gpu


def test_tiny_step_end_to_end():
    from tests import gpu_util as g
    w = synth.WORKLOADS[0]
    dim = w.dims[0]
    z = synth.latent(synth.seed_for(0, dim, 0, tensor=9), w.latent)
    ref_plan = orc.plan(w.latent, w.patch, w.K, dim, **w.overlap_args())
    plan = g.make_plan(w.latent, w.patch, w.K, dim, **w.overlap_args())
    subs = g.hip_partition(plan, z)
    assert subs.tobytes() == orc.partition(ref_plan, z).tobytes()
    for kp, (a, b) in enumerate(zip(plan.parts(), ref_plan.parts)):
        assert a.n_tokens == b.n_tokens == 200
        q, k, v = synth.qkv_bf16(synth.seed_for(0, dim, kp), a.n_tokens, w.heads, w.head_dim)
        g.assert_attention_close(g.hip_attention(q, k, v), orc.attention(q, k, v), "k=%d" % kp)
    # predictions = sub-latent + seeded perturbation, so overlaps really blend
    preds = subs + np.float32(0.1) * synth.normal_f32(synth.seed_for(0, dim, 0, tensor=10), subs.shape)
    got = g.hip_reconstruct(plan, preds, w.latent)
    assert got.tobytes() == orc.reconstruct(ref_plan, preds).tobytes()


@pytest.mark.parametrize("cfg", [5, 6])
def test_ratio_overlap_workloads_step(cfg):
    """49 frames at 480p, K = 4, overlap given as the ratio r (0.5: pairwise overlaps; 1.0: three
    partitions meet): latent ops bit-exact on all three dims, the guided step too, and attention
    on the largest sub-latent of the H step on sampled rows."""
    from tests import gpu_util as g
    w = synth.WORKLOADS[cfg]
    z = synth.latent(synth.seed_for(cfg, 0, 0, tensor=9), w.latent)
    for dim in w.dims:
        ref_plan = orc.plan(w.latent, w.patch, w.K, dim, **w.overlap_args())
        plan = g.make_plan(w.latent, w.patch, w.K, dim, **w.overlap_args())
        assert [p.n_tokens for p in plan.parts()] == [p.n_tokens for p in ref_plan.parts]
        subs = g.hip_partition(plan, z)
        assert subs.tobytes() == orc.partition(ref_plan, z).tobytes()
        preds = synth.normal_f32(synth.seed_for(cfg, dim, 0, tensor=10), (ref_plan.total_elems,))
        uncond = synth.normal_f32(synth.seed_for(cfg, dim, 0, tensor=11), (ref_plan.total_elems,))
        assert g.hip_reconstruct(plan, preds, w.latent).tobytes() == orc.reconstruct(ref_plan, preds).tobytes()
        want = orc.guided_step(ref_plan, preds, uncond, 5.0, z, 1.0, -0.04)
        assert g.hip_guided_step(plan, preds, uncond, 5.0, z, 1.0, -0.04).tobytes() == want.tobytes()
    dim = 1
    ref_plan = orc.plan(w.latent, w.patch, w.K, dim, **w.overlap_args())
    kp = int(np.argmax([p.n_tokens for p in ref_plan.parts]))
    n = ref_plan.parts[kp].n_tokens
    q, k, v = synth.qkv_bf16(synth.seed_for(cfg, dim, kp), n, w.heads, w.head_dim)
    rows = synth.sample_rows(n, 64, seed=cfg, tile=256)
    got = g.hip_attention(q, k, v)
    g.assert_attention_close(got[rows], orc.attention(q, k, v, rows=rows), "cfg %d n=%d" % (cfg, n))
    assert np.all(np.isfinite(got))
