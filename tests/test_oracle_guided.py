"""Pins for the oracle's guided denoising step (Eq. 4-6: per-partition classifier-free guidance,
reconstruction, sampler update) -- CPU only."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import lp_oracle as orc
from paper_2512_07350_amd import synth

P122 = (1, 2, 2)


def test_by_hand_on_the_tiny_config():
    # latent W = 16, p = 2, K = 2, O = 1: partitions [0,10) and [6,16) with weights
    # W1 = 1 x9, 1/2 and W2 = 0, 1/2, 1 x8 (Eq. 12), so on columns 6..9 the pairs are
    # (1,0) (1,1/2) (1,1) (1/2,1).
    # Eq. 4 with w = 2: g1 = 1 + 2 (3 - 1) = 5,  g2 = 2 + 2 (5 - 2) = 8.
    # Eq. 5: 5, (5 + 4)/1.5 = 6, 13/2 = 6.5, (2.5 + 8)/1.5 = 7, then 8.
    # Eq. 6 with z = 10, a = 1, b = -1/4: 10 - pred/4.
    latent = (16, 5, 16, 16)
    pl = orc.plan(latent, P122, 2, 2, overlap_patches=1)
    cond = np.empty(pl.total_elems, dtype=np.float32)
    uncond = np.empty_like(cond)
    n0 = pl.parts[0].n_elems
    cond[:n0], uncond[:n0] = 3.0, 1.0
    cond[n0:], uncond[n0:] = 5.0, 2.0
    z = np.full(latent, 10.0, dtype=np.float32)
    out = orc.guided_step(pl, cond, uncond, 2.0, z, 1.0, -0.25)
    want = [8.75] * 6 + [8.75, 8.5, 8.375, 8.25] + [8.0] * 6
    assert np.array_equal(out, np.broadcast_to(np.array(want, dtype=np.float32), latent))
    # the two prediction sets are not interchangeable
    swapped = orc.guided_step(pl, uncond, cond, 2.0, z, 1.0, -0.25)
    assert not np.array_equal(out, swapped)


@pytest.mark.parametrize("dim", [0, 1, 2])
def test_zero_guidance_zero_carry_is_plain_reconstruction(dim):
    # w = 0: g = u + 0 (c - u) = u;  a = 0, b = 1: z' = 0 z + pred = pred.  Bitwise.
    latent = (4, 6, 12, 20)
    pl = orc.plan(latent, P122, 3, dim, overlap_patches=1)
    cond = synth.normal_f32(11 + dim, (pl.total_elems,))
    uncond = synth.normal_f32(21 + dim, (pl.total_elems,))
    z = synth.normal_f32(31 + dim, latent)
    out = orc.guided_step(pl, cond, uncond, 0.0, z, 0.0, 1.0)
    assert np.array_equal(out, orc.reconstruct(pl, uncond))


@pytest.mark.parametrize("dim", [0, 1, 2])
def test_against_exact_rational_arithmetic(dim):
    # r = 1.5 gives positions covered by three partitions
    latent = (2, 6, 12, 12)
    pl = orc.plan(latent, P122, 4, dim, r=1.5)
    cond = synth.normal_f32(41 + dim, (pl.total_elems,))
    uncond = synth.normal_f32(51 + dim, (pl.total_elems,))
    z = synth.normal_f32(61 + dim, latent)
    w, a, b = np.float32(5.0), np.float32(0.98), np.float32(-0.0625)
    out = orc.guided_step(pl, cond, uncond, w, z, a, b)
    for idx in np.ndindex(*latent):
        x = idx[1 + dim]
        A = Fraction(0)
        Z = Fraction(0)
        for q in pl.parts:
            if not (q.s <= x < q.e):
                continue
            j = x - q.s
            if j < q.delta_start:
                wt = Fraction(j, q.delta_start)
            elif j < q.len - q.delta_end:
                wt = Fraction(1)
            else:
                wt = Fraction(q.len - j, q.delta_end)
            loc = list(idx)
            loc[1 + dim] = j
            li = q.elem_offset + np.ravel_multi_index(tuple(loc), q.shape)
            c, u = Fraction(float(cond[li])), Fraction(float(uncond[li]))
            A += wt * (u + Fraction(float(w)) * (c - u))
            Z += wt
        exact = float(Fraction(float(a)) * Fraction(float(z[idx])) + Fraction(float(b)) * A / Z)
        # |g| reaches ~ 5 * 6 sigma; a handful of binary32 roundings of values of that size, times |b|
        assert abs(float(out[idx]) - exact) <= 2e-6 * max(1.0, abs(exact)) + 1e-6, (idx, float(out[idx]), exact)


def test_guidance_commutes_with_reconstruction_up_to_rounding():
    # F is linear in the predictions: F(u + w (c - u)) = F(u) + w (F(c) - F(u))
    latent = (3, 5, 16, 24)
    pl = orc.plan(latent, P122, 4, 1, overlap_patches=2)
    cond = synth.normal_f32(71, (pl.total_elems,))
    uncond = synth.normal_f32(72, (pl.total_elems,))
    z = synth.normal_f32(73, latent)
    w, a, b = 7.5, 1.0, -0.02
    out = orc.guided_step(pl, cond, uncond, w, z, a, b).astype(np.float64)
    fc = orc.reconstruct(pl, cond).astype(np.float64)
    fu = orc.reconstruct(pl, uncond).astype(np.float64)
    want = a * z.astype(np.float64) + b * (fu + w * (fc - fu))
    assert np.max(np.abs(out - want)) < 5e-6


def test_unit_guidance_with_exact_data_keeps_the_conditional_prediction():
    # small integers: every step is exact, and w = 1 gives g = c
    latent = (2, 4, 8, 16)
    pl = orc.plan(latent, P122, 2, 2, overlap_patches=1)
    rng = np.random.default_rng(5)
    cond = rng.integers(-8, 9, pl.total_elems).astype(np.float32)
    uncond = rng.integers(-8, 9, pl.total_elems).astype(np.float32)
    z = rng.integers(-8, 9, latent).astype(np.float32)
    out = orc.guided_step(pl, cond, uncond, 1.0, z, 1.0, 1.0)
    assert np.array_equal(out, z + orc.reconstruct(pl, cond))
