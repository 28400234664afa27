"""lp_partition / lp_reconstruct on the GPU against the CPU oracle: bit-exact."""
import numpy as np
import pytest

from oracle import lp_oracle as orc
from paper_2512_07350_amd import synth

pytestmark = pytest.mark.gpu

P122 = (1, 2, 2)

# (latent, patch, K, overlap patches, dims)
CASES = [
    ((16, 5, 16, 16), P122, 2, 1, (0, 1, 2)),            # tiny config (+ the two other dims)
    ((16, 9, 60, 104), P122, 4, 1, (0, 1, 2)),           # 33-frame 480p, rotating
    ((16, 21, 60, 104), P122, 4, 2, (0, 1, 2)),          # 81-frame 480p
    ((16, 21, 90, 160), P122, 8, 2, (2,)),               # 81-frame 720p, K = 8
    ((3, 4, 6, 10), (1, 1, 1), 3, 1, (0, 1, 2)),         # patch 1: slices only 4-byte aligned along W
    ((2, 6, 9, 15), (2, 3, 5), 2, 1, (0, 1, 2)),         # odd extents, scalar path
    ((5, 8, 12, 36), P122, 5, 3, (0, 1, 2)),             # overlap wider than the core: 3 partitions meet
    ((1, 2, 2, 2), P122, 1, 0, (0, 1, 2)),               # smallest latent, K = 1
    ((2, 3, 4, 6), P122, 7, 0, (0, 1, 2)),               # K > N: empty partitions
    ((16, 21, 60, 104), P122, 2, 2, (0, 1, 2)),          # 81-frame 480p on 2 devices
    ((16, 21, 60, 104), P122, 8, 2, (0, 1, 2)),          # ... on 8 (along T: last core past the end)
    ((2, 3, 4, 40), P122, 8, 2, (2,)),                   # a core wholly past the end: front ramp longer than the partition
    ((3, 5, 7, 40), (1, 1, 4), 4, 1, (2,)),              # split along W by rows through LDS: 105 rows, the last workgroup takes 9
    ((2, 2, 3, 8208), (1, 1, 4), 3, 2, (2,)),            # a row of 32832 bytes: too long for the row kernel's LDS share
    ((1, 1, 70, 24), (1, 1, 4), 2, 1, (2,)),             # rows of 24 floats, sub-latent rows of 16
]


def _flat(cases):
    out = []
    for latent, patch, K, O, dims in cases:
        for d in dims:
            out.append(pytest.param(latent, patch, K, O, d, id="%s-K%d-O%d-%s" % ("x".join(map(str, latent)), K, O, synth.DIM_NAMES[d])))
    return out


@pytest.mark.parametrize("latent,patch,K,O,dim", _flat(CASES))
def test_partition_bit_exact(latent, patch, K, O, dim):
    from tests import gpu_util as g
    z = synth.latent(synth.seed_for(9, dim, K), latent)
    ref_plan = orc.plan(latent, patch, K, dim, overlap_patches=O)
    want = orc.partition(ref_plan, z)
    plan = g.make_plan(latent, patch, K, dim, overlap_patches=O)
    got = g.hip_partition(plan, z)
    assert got.shape == want.shape
    assert got.tobytes() == want.tobytes()
    # and on an index-coded latent, where any wrong source index shows up as a wrong value
    zi = synth.index_coded(latent)
    assert g.hip_partition(plan, zi).tobytes() == orc.partition(ref_plan, zi).tobytes()


@pytest.mark.parametrize("latent,patch,K,O,dim", _flat(CASES))
def test_reconstruct_bit_exact(latent, patch, K, O, dim):
    from tests import gpu_util as g
    ref_plan = orc.plan(latent, patch, K, dim, overlap_patches=O)
    preds = synth.normal_f32(synth.seed_for(9, dim, K, tensor=5), (ref_plan.total_elems,))
    want = orc.reconstruct(ref_plan, preds)
    plan = g.make_plan(latent, patch, K, dim, overlap_patches=O)
    got = g.hip_reconstruct(plan, preds, latent)
    assert got.tobytes() == want.tobytes()


@pytest.mark.parametrize("latent,patch,K,O,dim", _flat(CASES))
def test_guided_step_bit_exact(latent, patch, K, O, dim):
    # Eq. 4-6 in one pass against the oracle's three stages; also updating z in place
    from tests import gpu_util as g
    ref_plan = orc.plan(latent, patch, K, dim, overlap_patches=O)
    cond = synth.normal_f32(synth.seed_for(9, dim, K, tensor=6), (ref_plan.total_elems,))
    uncond = synth.normal_f32(synth.seed_for(9, dim, K, tensor=7), (ref_plan.total_elems,))
    z = synth.latent(synth.seed_for(9, dim, K, tensor=8), latent)
    w, a, b = 5.0, 0.9921875, -0.03125 * 1.37
    want = orc.guided_step(ref_plan, cond, uncond, w, z, a, b)
    plan = g.make_plan(latent, patch, K, dim, overlap_patches=O)
    got = g.hip_guided_step(plan, cond, uncond, w, z, a, b)
    assert got.tobytes() == want.tobytes()
    assert g.hip_guided_step(plan, cond, uncond, w, z, a, b, in_place=True).tobytes() == want.tobytes()


@pytest.mark.parametrize("latent,patch,K,O,dim", _flat(CASES))
def test_guided_step_with_next_partition_bit_exact(latent, patch, K, O, dim):
    # the fused call = the guided step, then Eq. 10 of its result along every possible next dim
    from tests import gpu_util as g
    ref_plan = orc.plan(latent, patch, K, dim, overlap_patches=O)
    cond = synth.normal_f32(synth.seed_for(9, dim, K, tensor=6), (ref_plan.total_elems,))
    uncond = synth.normal_f32(synth.seed_for(9, dim, K, tensor=7), (ref_plan.total_elems,))
    z = synth.latent(synth.seed_for(9, dim, K, tensor=8), latent)
    w, a, b = 5.0, 0.9921875, -0.03125 * 1.37
    want_z = orc.guided_step(ref_plan, cond, uncond, w, z, a, b)
    plan = g.make_plan(latent, patch, K, dim, overlap_patches=O)
    for nxt in range(3):
        next_ref = orc.plan(latent, patch, K, nxt, overlap_patches=O)
        next_plan = g.make_plan(latent, patch, K, nxt, overlap_patches=O)
        got_z, got_subs = g.hip_guided_step_partition(plan, cond, uncond, w, z, a, b, next_plan, in_place=(nxt == 1))
        assert got_z.tobytes() == want_z.tobytes(), nxt
        assert got_subs.tobytes() == orc.partition(next_ref, want_z).tobytes(), nxt


def test_guided_step_special_values_and_ratio_overlap():
    from tests import gpu_util as g
    latent = (16, 13, 60, 104)
    for dim in range(3):
        ref_plan = orc.plan(latent, P122, 4, dim, r=1.5)
        cond = synth.normal_f32(2234 + dim, (ref_plan.total_elems,))
        uncond = synth.normal_f32(3234 + dim, (ref_plan.total_elems,))
        z = synth.latent(4234 + dim, latent)
        plan = g.make_plan(latent, P122, 4, dim, overlap_ratio=1.5)
        for w, a, b in ((0.0, 0.0, 1.0), (1.0, 1.0, 1.0), (7.5, 1.0, -1.0 / 3.0)):
            want = orc.guided_step(ref_plan, cond, uncond, w, z, a, b)
            assert g.hip_guided_step(plan, cond, uncond, w, z, a, b).tobytes() == want.tobytes()
        # w = 0, a = 0, b = 1 is plain reconstruction of the unconditional set
        assert g.hip_guided_step(plan, cond, uncond, 0.0, z, 0.0, 1.0).tobytes() == g.hip_reconstruct(plan, uncond, latent).tobytes()


def test_guided_step_misaligned_buffers():
    # base pointers offset by one float: the kernels must fall back to narrower vectors
    from tests import gpu_util as g
    import torch
    from paper_2512_07350_amd import binding as lp
    latent = (16, 9, 60, 104)
    ref_plan = orc.plan(latent, P122, 4, 1, overlap_patches=1)
    n, nz = ref_plan.total_elems, int(np.prod(latent))
    cond = synth.normal_f32(91, (n,)); uncond = synth.normal_f32(92, (n,)); z = synth.latent(93, latent)
    want = orc.guided_step(ref_plan, cond, uncond, 4.0, z, 1.0, -0.125)
    plan = g.make_plan(latent, P122, 4, 1, overlap_patches=1)
    for offs in ((1, 0, 0, 0), (0, 1, 0, 0), (0, 0, 1, 0), (0, 0, 0, 1), (2, 2, 2, 2)):
        bufs = []
        for host, off in zip((cond, uncond, z.reshape(-1), np.full(nz, np.nan, np.float32)), offs):
            t = torch.empty(host.size + 4, dtype=torch.float32, device="cuda")
            t[off:off + host.size].copy_(torch.from_numpy(host))
            bufs.append(t[off:off + host.size])
        lp.lp_reconstruct_guided_step(plan, bufs[0], bufs[1], 4.0, bufs[2], 1.0, -0.125, bufs[3], g.stream())
        torch.cuda.synchronize()
        assert bufs[3].cpu().numpy().tobytes() == want.tobytes(), offs


@pytest.mark.parametrize("r", [0.5, 1.0, 1.5])
def test_reconstruct_bit_exact_with_ratio_overlap(r):
    # r = 1.0 and 1.5 give non-dyadic ramps (Delta = 16, 26 ...) and three-way overlaps
    from tests import gpu_util as g
    latent = (16, 13, 60, 104)
    for dim in range(3):
        ref_plan = orc.plan(latent, P122, 4, dim, r=r)
        preds = synth.normal_f32(1234 + dim, (ref_plan.total_elems,))
        plan = g.make_plan(latent, P122, 4, dim, overlap_ratio=r)
        assert g.hip_reconstruct(plan, preds, latent).tobytes() == orc.reconstruct(ref_plan, preds).tobytes()


def test_roundtrip_on_device():
    # partition then reconstruct of the same field returns it (index-coded: exactly)
    from tests import gpu_util as g
    import torch
    from paper_2512_07350_amd import binding as lp
    latent = (16, 21, 60, 104)
    z = synth.index_coded(latent)
    for dim in range(3):
        plan = g.make_plan(latent, P122, 4, dim, overlap_patches=2)
        zd = torch.from_numpy(z).cuda()
        subs = torch.empty(plan.total_elems, dtype=torch.float32, device="cuda")
        out = torch.empty_like(zd)
        lp.lp_partition(plan, zd, subs, g.stream())
        lp.lp_reconstruct(plan, subs, out, g.stream())
        torch.cuda.synchronize()
        assert torch.equal(out, zd)


def test_misaligned_buffers_fall_back_to_narrower_vectors():
    from tests import gpu_util as g
    import torch
    from paper_2512_07350_amd import binding as lp
    latent = (4, 6, 12, 16)
    z = synth.latent(77, latent)
    for dim in range(3):
        ref_plan = orc.plan(latent, P122, 3, dim, overlap_patches=1)
        plan = g.make_plan(latent, P122, 3, dim, overlap_patches=1)
        n_lat = z.size
        for shift in (1, 2):       # buffers only 4- or 8-byte aligned
            zbuf = torch.zeros(n_lat + 4, dtype=torch.float32, device="cuda")
            sbuf = torch.zeros(plan.total_elems + 4, dtype=torch.float32, device="cuda")
            obuf = torch.zeros(n_lat + 4, dtype=torch.float32, device="cuda")
            zbuf[shift:shift + n_lat] = torch.from_numpy(z.ravel()).cuda()
            lp.lp_partition(plan, zbuf.data_ptr() + 4 * shift, sbuf.data_ptr() + 4 * shift, g.stream())
            lp.lp_reconstruct(plan, sbuf.data_ptr() + 4 * shift, obuf.data_ptr() + 4 * shift, g.stream())
            torch.cuda.synchronize()
            subs = sbuf[shift:shift + plan.total_elems].cpu().numpy()
            assert subs.tobytes() == orc.partition(ref_plan, z).tobytes()
            out = obuf[shift:shift + n_lat].cpu().numpy().reshape(latent)
            assert out.tobytes() == orc.reconstruct(ref_plan, subs).tobytes()
            assert float(sbuf[:shift].abs().sum()) == 0.0 and float(obuf[shift + n_lat:].abs().sum()) == 0.0


def test_random_shapes_bit_exact():
    """Seeded random latents, patches, K, overlaps (count or ratio) and dims: partition,
    reconstruction and the guided step against the oracle, bit for bit."""
    from tests import gpu_util as g
    rng = np.random.default_rng(20251207)
    done = 0
    while done < 40:
        patch = tuple(int(rng.integers(1, 4)) for _ in range(3))
        latent = (int(rng.integers(1, 6)),) + tuple(int(p * rng.integers(1, 13)) for p in patch)
        dim = int(rng.integers(0, 3))
        K = int(rng.integers(1, 9))
        N = latent[1 + dim] // patch[dim]
        L = -(-N // K)
        if rng.random() < 0.5:
            kw = {"overlap_patches": int(rng.integers(0, L * (K - 1) + 1))}
        else:
            kw = {"overlap_patches": -1, "overlap_ratio": float(rng.uniform(0.0, K - 1))}
        ref_plan = orc.plan(latent, patch, K, dim, **kw)
        plan = g.make_plan(latent, patch, K, dim, **kw)
        assert plan.total_elems == ref_plan.total_elems, (latent, patch, K, dim, kw)
        z = synth.latent(1000 + done, latent)
        assert g.hip_partition(plan, z).tobytes() == orc.partition(ref_plan, z).tobytes(), (latent, patch, K, dim, kw)
        cond = synth.normal_f32(2000 + done, (ref_plan.total_elems,))
        uncond = synth.normal_f32(3000 + done, (ref_plan.total_elems,))
        assert g.hip_reconstruct(plan, cond, latent).tobytes() == orc.reconstruct(ref_plan, cond).tobytes(), (latent, patch, K, dim, kw)
        want = orc.guided_step(ref_plan, cond, uncond, 3.5, z, 0.875, 0.3)
        assert g.hip_guided_step(plan, cond, uncond, 3.5, z, 0.875, 0.3).tobytes() == want.tobytes(), (latent, patch, K, dim, kw)
        # ... and fused with the partition of the result along another dim, with another K
        nxt, K2 = int(rng.integers(0, 3)), int(rng.integers(1, 9))
        next_ref = orc.plan(latent, patch, K2, nxt, overlap_patches=0)
        next_plan = g.make_plan(latent, patch, K2, nxt, overlap_patches=0)
        got_z, got_subs = g.hip_guided_step_partition(plan, cond, uncond, 3.5, z, 0.875, 0.3, next_plan)
        assert got_z.tobytes() == want.tobytes(), (latent, patch, K, dim, kw, nxt, K2)
        assert got_subs.tobytes() == orc.partition(next_ref, want).tobytes(), (latent, patch, K, dim, kw, nxt, K2)
        done += 1
