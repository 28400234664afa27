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


@pytest.mark.parametrize("cfg", [5, 6, 10])
def test_ratio_overlap_workloads_step(cfg):
    """49 frames at 480p, K = 4, overlap given as the ratio r (0.5: pairwise overlaps; 1.0: three
    partitions meet), and the 161-frame clip at r = 0.5: latent ops bit-exact on all three dims, the guided step too, and attention
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
    rows = synth.sample_rows(n, 256, seed=cfg, tile=256)
    got = g.hip_attention(q, k, v)
    g.assert_attention_close(got[rows], orc.attention(q, k, v, rows=rows), "cfg %d n=%d" % (cfg, n))
    assert np.all(np.isfinite(got))


def test_step_replays_from_a_captured_graph():
    """The calls enqueue work only (no allocation, no synchronisation, no memset nodes), so a
    whole step can be captured in a HIP graph after one eager warm-up.  Three replays with
    the program's own eager work and synchronisations in between, each checked against the
    eager result of the same inputs."""
    import torch
    from tests import gpu_util as g
    from paper_2512_07350_amd import binding as lp
    w = synth.WORKLOADS[0]
    dim = w.dims[0]
    plan = g.make_plan(w.latent, w.patch, w.K, dim, **w.overlap_args())
    parts = plan.parts()
    n, heads, hd = parts[0].n_tokens, w.heads, w.head_dim
    zd = torch.from_numpy(synth.latent(1, w.latent)).cuda()
    subs = torch.empty(plan.total_elems, dtype=torch.float32, device="cuda")
    uncond = torch.from_numpy(synth.normal_f32(2, (plan.total_elems,))).cuda()
    out = torch.empty_like(zd)
    q, k, v = (g.to_dev_bf16(a) for a in synth.qkv_bf16(3, n, heads, hd))
    o = torch.empty_like(q)
    ws, ws_bytes = g.workspace(hd)
    # a second, larger call whose query tiles are shared between workgroups (workspace + merge kernel)
    n2, heads2, hd2 = 1000, 3, 128
    q2, k2, v2 = (g.to_dev_bf16(a) for a in synth.qkv_bf16(4, n2, heads2, hd2))
    o2 = torch.empty_like(q2)
    ws2, ws2_bytes = g.workspace(hd2)

    def step(stream):
        lp.lp_partition(plan, zd, subs, stream)
        lp.lp_attention(q, k, v, o, n, heads, hd, heads * hd, hd, 0.0, ws, ws_bytes, stream)
        lp.lp_attention(q2, k2, v2, o2, n2, heads2, hd2, heads2 * hd2, hd2, 0.0, ws2, ws2_bytes, stream)
        lp.lp_reconstruct_guided_step(plan, subs, uncond, 2.0, zd, 1.0, -0.25, out, stream)

    step(g.stream())                      # eager warm-up: one-time function attributes are set here
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step(torch.cuda.current_stream().cuda_stream)
    for rep in range(3):
        zd.copy_(torch.from_numpy(synth.latent(10 + rep, w.latent)))
        q.copy_(g.to_dev_bf16(synth.qkv_bf16(20 + rep, n, heads, hd)[0]))
        k2.copy_(g.to_dev_bf16(synth.qkv_bf16(30 + rep, n2, heads2, hd2)[1]))
        for t in (out, o, o2, subs):
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got_out, got_o, got_o2, got_subs = out.clone(), o.clone(), o2.clone(), subs.clone()
        for t in (out, o, o2, subs):
            t.fill_(float("nan"))
        step(g.stream())
        torch.cuda.synchronize()
        assert torch.equal(got_subs, subs), rep
        assert torch.equal(got_out, out), rep
        assert torch.equal(got_o.view(torch.int16), o.view(torch.int16)), rep
        assert torch.equal(got_o2.view(torch.int16), o2.view(torch.int16)), rep
        assert not torch.isnan(o2.float()).any()
    # and the last eager result is the oracle's
    ref_plan = orc.plan(w.latent, w.patch, w.K, dim, **w.overlap_args())
    z_h = zd.cpu().numpy()
    want = orc.guided_step(ref_plan, orc.partition(ref_plan, z_h), uncond.cpu().numpy(), 2.0, z_h, 1.0, -0.25)
    assert out.cpu().numpy().tobytes() == want.tobytes()


def test_chained_guided_steps_carry_the_latent():
    """Seven denoising steps in a row, rotating T -> H -> W (Eq. 3), the way a sampling loop runs
    them: step i's fused call updates the latent in place (Eq. 4-6) and writes the sub-latents
    step i + 1 starts from (Eq. 10 along the next dimension); the latent and the packed
    sub-latents never leave the device between steps.  Every intermediate latent and packed
    buffer is compared bit for bit with the oracle's guided step -> partition chain."""
    import torch
    from tests import gpu_util as g
    from paper_2512_07350_amd import binding as lp
    latent, patch, K, O = (4, 6, 8, 12), (1, 2, 2), 3, 1
    plans = [g.make_plan(latent, patch, K, d, overlap_patches=O) for d in range(3)]
    refs = [orc.plan(latent, patch, K, d, overlap_patches=O) for d in range(3)]
    z_ref = synth.latent(4242, latent)
    zd = torch.from_numpy(z_ref.copy()).cuda()
    dim = lp.lp_rotation_dim(1)
    subs_d = torch.full((plans[dim].total_elems,), float("nan"), dtype=torch.float32, device="cuda")
    lp.lp_partition(plans[dim], zd, subs_d, g.stream())
    subs_ref = orc.partition(refs[dim], z_ref)
    for i in range(1, 8):
        dim, nxt = lp.lp_rotation_dim(i), lp.lp_rotation_dim(i + 1)
        assert dim == orc.rotation_dim(i) and nxt == (dim + 1) % 3
        torch.cuda.synchronize()
        assert subs_d.cpu().numpy().tobytes() == subs_ref.tobytes(), "sub-latents entering step %d" % i
        # stand-in predictions: the step's sub-latents plus seeded noise (both sides get the same arrays)
        cond = subs_ref + np.float32(0.1) * synth.normal_f32(5000 + i, subs_ref.shape)
        uncond = subs_ref + np.float32(0.1) * synth.normal_f32(6000 + i, subs_ref.shape)
        w, a, b = 3.5, 1.0, np.float32(-0.05 - 0.01 * i).item()
        next_d = torch.full((plans[nxt].total_elems,), float("nan"), dtype=torch.float32, device="cuda")
        lp.lp_reconstruct_guided_step_partition(plans[dim], torch.from_numpy(cond).cuda(), torch.from_numpy(uncond).cuda(),
                                                w, zd, a, b, zd, plans[nxt], next_d, g.stream())
        z_ref = orc.guided_step(refs[dim], cond, uncond, w, z_ref, a, b)
        subs_ref = orc.partition(refs[nxt], z_ref)
        subs_d = next_d
        torch.cuda.synchronize()
        assert zd.cpu().numpy().tobytes() == z_ref.tobytes(), "latent after step %d" % i
    assert subs_d.cpu().numpy().tobytes() == subs_ref.tobytes()
