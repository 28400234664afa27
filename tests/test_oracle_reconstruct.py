"""Pins for the oracle's weights, partition and reconstruction (Eq. 10-17) -- CPU only."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import lp_oracle as orc
from paper_2512_07350_amd import synth

P122 = (1, 2, 2)


def _weights(part):
    return [float(orc.weight(j, part.len, part.delta_start, part.delta_end)) for j in range(part.len)]


def _Z(pl, extent):
    z = [0.0] * extent
    for q in pl.parts:
        for j, w in enumerate(_weights(q)):
            z[q.s + j] += w
    return z


def test_weights_tiny_config_by_hand():
    # latent W = 16, p = 2, K = 2, O = 1: N = 8, L = 4; partitions [0,10) and [6,16).
    # Eq. 11: Delta_end(1) = (5-4)*2 = 2, Delta_start(2) = (4-3)*2 = 2.
    # Eq. 12: rear ramp (l-j)/Delta = 1, 1/2 ; front ramp j/Delta = 0, 1/2.
    pl = orc.plan((16, 5, 16, 16), P122, 2, 2, overlap_patches=1)
    assert _weights(pl.parts[0]) == [1.0] * 9 + [0.5]
    assert _weights(pl.parts[1]) == [0.0, 0.5] + [1.0] * 8
    assert _Z(pl, 16)[6:10] == [1.0, 1.5, 2.0, 1.5]


def test_weights_delta4_by_hand():
    # 81-frame 480p along H, K = 4, O = 2: Delta = 4 on interior edges.
    pl = orc.plan((16, 21, 60, 104), P122, 4, 1, overlap_patches=2)
    w1 = _weights(pl.parts[1])            # latent rows [12, 36): front ramp, 16 core rows, rear ramp
    assert w1[:4] == [0.0, 0.25, 0.5, 0.75]
    assert w1[4:20] == [1.0] * 16
    assert w1[20:] == [1.0, 0.75, 0.5, 0.25]
    # overlap of partitions 1 and 2 spans rows 12..19: rear ramp of 1 + front ramp of 2
    assert _Z(pl, 60)[12:20] == [1.0, 1.25, 1.5, 1.75, 2.0, 1.75, 1.5, 1.25]


def test_weights_last_core_past_the_end():
    # 33-frame along T: N = 9, K = 4, L = 3, O = 1: the 4th core starts at 9 = N, so the
    # 4th partition is [8, 9): pure front overlap with weight 0/1 = 0 (Eq. 12, first case).
    pl = orc.plan((16, 9, 60, 104), P122, 4, 0, overlap_patches=1)
    assert [(q.s, q.e) for q in pl.parts] == [(0, 4), (2, 7), (5, 9), (8, 9)]
    assert _weights(pl.parts[3]) == [0.0]
    # third partition [5,9): core [6,9) reaches N, so Delta_end = 0 and there is no rear ramp
    assert _weights(pl.parts[2]) == [0.0, 1.0, 1.0, 1.0]
    assert _Z(pl, 9) == [1.0, 1.0, 1.0, 2.0, 1.0, 1.0, 2.0, 1.0, 1.0]


def test_weights_and_blend_where_a_core_lies_wholly_past_the_end_by_hand():
    # W = 40, p = 2, K = 8, O = 2: N = 20, L = ceil(20/8) = 3; cores [0,3) ... [18,21), [21,24).
    # 8th partition (the paper's k = 8): alpha = 21 > N, alpha' = 19, beta' = min(20, 26) = 20, so it is
    # the latent range [38, 40) with l = 2, and Eq. 11 as written gives
    #   Delta_start = (21 - 19) * 2 = 4  (> l),   Delta_end = (20 - 24) * 2 = -8.
    # Eq. 12, first case (j < Delta_start) holds for both positions: weights 0/4 and 1/4.
    # (A Delta_start cut off at the end of the latent, (20 - 19) * 2 = 2, would give 0 and 1/2:
    # this is where evaluating Eq. 11-12 as written and a clamped ramp length part ways.)
    pl = orc.plan((1, 1, 2, 40), P122, 8, 2, overlap_patches=2)
    p6, p7, p8 = pl.parts[5], pl.parts[6], pl.parts[7]
    assert (p8.s, p8.e, p8.len, p8.delta_start, p8.delta_end) == (38, 40, 2, 4, -8)
    assert _weights(p8) == [0.0, 0.25]
    # 7th: core [18,21) runs past N: alpha' = 16, beta' = 20 -> [32, 40), Delta_start = 4, Delta_end = -2:
    # front ramp 0, 1/4, 1/2, 3/4, then the second case up to j < 8 + 2, i.e. to the end
    assert (p7.s, p7.e, p7.delta_start, p7.delta_end) == (32, 40, 4, -2)
    assert _weights(p7) == [0.0, 0.25, 0.5, 0.75, 1.0, 1.0, 1.0, 1.0]
    # 6th: core [15,18): alpha' = 13, beta' = 20 -> [26, 40), Delta = 4 on both sides
    assert (p6.s, p6.e, p6.delta_start, p6.delta_end) == (26, 40, 4, 4)
    assert _weights(p6) == [0.0, 0.25, 0.5, 0.75] + [1.0] * 6 + [1.0, 0.75, 0.5, 0.25]
    # columns 36..39 are covered by partitions 6, 7 (and 8 from column 38): Z = W6 + W7 + W8
    assert _Z(pl, 40)[36:40] == [2.0, 1.75, 1.5, 1.5]
    # blend of three constants (1, 2, 4 for partitions 6, 7, 8; 0 elsewhere), columns 36..39:
    #   (1*1 + 1*2)/2, (.75*1 + 1*2)/1.75, (.5*1 + 1*2 + 0*4)/1.5, (.25*1 + 1*2 + .25*4)/1.5
    preds = np.zeros(pl.total_elems, dtype=np.float32)
    for q, c in ((p6, 1.0), (p7, 2.0), (p8, 4.0)):
        preds[q.elem_offset:q.elem_offset + q.n_elems] = c
    out = orc.reconstruct(pl, preds)
    f = np.float32
    want = [f(3.0) / f(2.0), f(2.75) / f(1.75), f(2.5) / f(1.5), f(3.25) / f(1.5)]
    assert out[0, 0, 0, 36:40].tolist() == want and out[0, 0, 1, 36:40].tolist() == want


@pytest.mark.parametrize("K,O,dim", [(2, 1, 2), (4, 2, 1), (4, 1, 0), (3, 5, 1), (8, 2, 2), (5, 0, 1)])
def test_weight_closed_form_and_normalisation(K, O, dim):
    latent = (2, 12, 36, 40)
    pl = orc.plan(latent, P122, K, dim, overlap_patches=O)
    extent = latent[1 + dim]
    Z = [Fraction(0)] * extent
    for q in pl.parts:
        for j in range(q.len):
            # Eq. 12 in exact rational arithmetic, from the plan's integers
            if j < q.delta_start:
                w = Fraction(j, q.delta_start)
            elif j < q.len - q.delta_end:
                w = Fraction(1)
            else:
                w = Fraction(q.len - j, q.delta_end)
            assert Fraction(float(orc.weight(j, q.len, q.delta_start, q.delta_end))).limit_denominator(1 << 12) == w
            assert 0 <= w <= 1
            Z[q.s + j] += w
    # every position lies in exactly one core, so Z >= 1; normalised weights then sum to 1 (Eq. 17)
    assert all(z >= 1 for z in Z)


def test_partition_is_a_slice():
    latent = (3, 6, 8, 10)
    z = synth.index_coded(latent)
    for dim in range(3):
        pl = orc.plan(latent, P122, 3, dim, overlap_patches=1)
        subs = orc.partition(pl, z)
        for q in pl.parts:
            sl = [slice(None)] * 4
            sl[1 + dim] = slice(q.s, q.e)
            want = z[tuple(sl)]
            got = subs[q.elem_offset:q.elem_offset + q.n_elems].reshape(q.shape)
            assert np.array_equal(got, want)


@pytest.mark.parametrize("dim", [0, 1, 2])
def test_roundtrip_identity_K1_and_zero_overlap(dim):
    latent = (4, 6, 12, 20)
    z = synth.latent(11 + dim, latent)
    for K, O in ((1, 0), (3, 0), (4, 0)):
        pl = orc.plan(latent, P122, K, dim, overlap_patches=O)
        out = orc.reconstruct(pl, orc.partition(pl, z))
        assert out.tobytes() == z.tobytes()          # bitwise: weights are all 1, Z = 1


@pytest.mark.parametrize("latent,K,O,dim", [
    ((16, 5, 16, 16), 2, 1, 2),      # Delta = 2
    ((4, 9, 12, 16), 4, 1, 0),       # Delta = 1, last core past the end
    ((4, 6, 60, 8), 4, 2, 1),        # Delta = 4
    ((2, 4, 8, 160), 8, 2, 2),       # Delta = 4, K = 8
])
def test_slices_of_one_field_reconstruct_to_it_bitwise(latent, K, O, dim):
    # If every prediction is the matching slice of one field G, A/Z = G.  With G holding
    # integers < 2^20 and Delta in {1,2,4} every product, sum and the divide are exact.
    G = synth.index_coded(latent)
    pl = orc.plan(latent, P122, K, dim, overlap_patches=O)
    out = orc.reconstruct(pl, orc.partition(pl, G))
    assert out.tobytes() == G.tobytes()


def test_two_constant_predictions_blend_by_hand():
    # tiny config along W; prediction 1 is constant 1, prediction 2 constant 3.
    # Columns 6..9 (weights worked above): (1*1+0*3)/1, (1+1.5)/1.5, (1+3)/2, (0.5+3)/1.5
    latent = (16, 5, 16, 16)
    pl = orc.plan(latent, P122, 2, 2, overlap_patches=1)
    preds = np.empty(pl.total_elems, dtype=np.float32)
    preds[:pl.parts[0].n_elems] = 1.0
    preds[pl.parts[1].elem_offset:] = 3.0
    out = orc.reconstruct(pl, preds)
    want_row = [1.0] * 6 + [1.0, np.float32(2.5) / np.float32(1.5), 2.0, np.float32(3.5) / np.float32(1.5)] + [3.0] * 6
    assert np.array_equal(out, np.broadcast_to(np.array(want_row, dtype=np.float32), latent))


@pytest.mark.parametrize("dim", [0, 1, 2])
def test_reconstruct_against_exact_rational_brute_force(dim):
    # r = 1.5: three partitions overlap at some positions (sum over all k, Eq. 15-16)
    latent = (2, 6, 12, 12)
    K = 4
    pl = orc.plan(latent, P122, K, dim, r=1.5)
    preds = synth.normal_f32(77 + dim, (pl.total_elems,))
    out = orc.reconstruct(pl, preds)
    multi = 0
    for idx in np.ndindex(*latent):
        x = idx[1 + dim]
        A = Fraction(0)
        Z = Fraction(0)
        n_in = 0
        for q in pl.parts:
            if not (q.s <= x < q.e):
                continue
            n_in += 1
            j = x - q.s
            if j < q.delta_start:
                w = Fraction(j, q.delta_start)
            elif j < q.len - q.delta_end:
                w = Fraction(1)
            else:
                w = Fraction(q.len - j, q.delta_end)
            loc = list(idx)
            loc[1 + dim] = j
            li = np.ravel_multi_index(tuple(loc), q.shape)
            A += w * Fraction(float(preds[q.elem_offset + li]))
            Z += w
        multi += n_in >= 3
        exact = float(A / Z)
        assert abs(float(out[idx]) - exact) <= 4e-7 * max(1.0, abs(exact)), (idx, float(out[idx]), exact)
    assert multi > 0


def test_reconstruct_is_a_convex_combination():
    latent = (3, 6, 16, 20)
    pl = orc.plan(latent, P122, 4, 2, overlap_patches=2)
    preds = np.empty(pl.total_elems, dtype=np.float32)
    for k, q in enumerate(pl.parts):
        preds[q.elem_offset:q.elem_offset + q.n_elems] = float(k)
    out = orc.reconstruct(pl, preds)
    # constant along every non-partition coordinate, monotone non-decreasing along W
    prof = out[0, 0, 0, :]
    assert np.array_equal(out, np.broadcast_to(prof, latent))
    assert np.all(np.diff(prof) >= 0) and prof[0] == 0.0
    assert np.all((prof >= 0.0) & (prof <= 3.0))
    # last column: rear ramp of partition 3 still gives 1/2 there (Eq. 12 ends at 1/Delta, not 0)
    assert prof[-1] == np.float32(0.5 * 2 + 3) / np.float32(1.5)
    const = np.full(pl.total_elems, 0.7, dtype=np.float32)
    assert np.allclose(orc.reconstruct(pl, const), np.float32(0.7), rtol=0, atol=1e-7)
