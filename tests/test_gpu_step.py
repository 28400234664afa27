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
    ref_plan = orc.plan(w.latent, w.patch, w.K, dim, overlap_patches=w.overlap_patches)
    plan = g.make_plan(w.latent, w.patch, w.K, dim, overlap_patches=w.overlap_patches)
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
