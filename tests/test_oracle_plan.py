"""Pins for the oracle's integer plan (Eq. 3, 7-9, 11) -- CPU only.

The strongest pin is the paper's own Table 1: the LP rows are communication
volumes, which are pure functions of the sub-latent sizes the plan produces.
"""
import math
import os

import pytest
from hypothesis import given, settings, strategies as st

from oracle import lp_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "table1_lp_rows.txt")


def _table1_rows():
    rows = []
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            t = line.split()
            rows.append((int(t[0]), float(t[1]), [float(x) for x in t[2:6]], float(t[6])))
    return rows


@pytest.mark.parametrize("frames,r,per_gpu,total", _table1_rows())
def test_table1_lp_rows(frames, r, per_gpu, total):
    """Table 1, LP rows.  Accounting (Sec. 5.1 + supplement 'Communication Overhead of LP'):
    fp32 latent [16, 1+(F-1)/4, 60, 104], patch (1,2,2), K = 4, 60 steps = 20 per
    dimension (Eq. 3); each worker moves its sub-latent once out and once back per
    step; the master additionally touches the whole latent once per step; MB = 2^20 B."""
    latent = (16, 1 + (frames - 1) // 4, 60, 104)
    s_z = 4 * math.prod(latent)
    got = [0.0] * 4
    steps_per_dim = [sum(1 for i in range(1, 61) if orc.rotation_dim(i) == d) for d in range(3)]
    assert steps_per_dim == [20, 20, 20]
    for d in range(3):
        pl = orc.plan(latent, (1, 2, 2), 4, d, r=r)
        for k, p in enumerate(pl.parts):
            got[k] += 2 * steps_per_dim[d] * 4 * p.n_elems
    got[0] += 60 * s_z
    for k in range(4):
        assert round(got[k] / 2**20, 2) == pytest.approx(per_gpu[k], abs=0.0051), (k, got[k] / 2**20)
    assert round(sum(got) / 2**20, 2) == pytest.approx(total, abs=0.0051)


def test_rotation_schedule():
    # Eq. 3: indices 1,2,3 -> temporal, height, width, then repeating.
    assert [orc.rotation_dim(i) for i in range(1, 8)] == [0, 1, 2, 0, 1, 2, 0]
    # consecutive steps never share a dimension (used by the 2-completeness theorem)
    for i in range(1, 100):
        assert orc.rotation_dim(i) != orc.rotation_dim(i + 1)
    with pytest.raises(ValueError):
        orc.rotation_dim(0)


# Patch ranges [alpha', beta') and token counts worked by hand from Eq. 7-8 for the
# benchmark shapes (N, L, O in the comment).
HAND = [
    # latent, K, O, dim, ranges, tokens
    ((16, 5, 16, 16), 2, 1, 2, [(0, 5), (3, 8)], [200, 200]),                         # N=8 L=4
    ((16, 9, 60, 104), 4, 1, 0, [(0, 4), (2, 7), (5, 9), (8, 9)], [6240, 7800, 6240, 1560]),   # N=9 L=3
    ((16, 9, 60, 104), 4, 1, 1, [(0, 9), (7, 17), (15, 25), (23, 30)], [4212, 4680, 4680, 3276]),  # N=30 L=8
    ((16, 9, 60, 104), 4, 1, 2, [(0, 14), (12, 27), (25, 40), (38, 52)], [3780, 4050, 4050, 3780]),  # N=52 L=13
    ((16, 21, 60, 104), 4, 2, 1, [(0, 10), (6, 18), (14, 26), (22, 30)], [10920, 13104, 13104, 8736]),
    ((16, 21, 90, 160), 8, 2, 2,
     [(0, 12), (8, 22), (18, 32), (28, 42), (38, 52), (48, 62), (58, 72), (68, 80)],
     [11340] + [13230] * 6 + [11340]),
    ((16, 21, 60, 104), 4, 2, 0, [(0, 8), (4, 14), (10, 20), (16, 21)], [12480, 15600, 15600, 7800]),
]


@pytest.mark.parametrize("latent,K,O,dim,ranges,tokens", HAND)
def test_hand_worked_ranges(latent, K, O, dim, ranges, tokens):
    pl = orc.plan(latent, (1, 2, 2), K, dim, overlap_patches=O)
    assert [(p.alpha_ext, p.beta_ext) for p in pl.parts] == ranges
    assert [p.n_tokens for p in pl.parts] == tokens
    p_d = (1, 2, 2)[dim]
    assert [(p.s, p.e) for p in pl.parts] == [(a * p_d, b * p_d) for a, b in ranges]   # Eq. 9


def test_overlap_from_ratio_is_floor():
    # O = floor(L * r): L = 13, r = 0.5 -> 6 (the 480p width case of Table 1)
    pl = orc.plan((16, 13, 60, 104), (1, 2, 2), 4, 2, r=0.5)
    assert pl.parts[1].alpha - pl.parts[1].alpha_ext == 6
    pl = orc.plan((16, 13, 60, 104), (1, 2, 2), 4, 2, r=1.0)
    assert pl.parts[1].alpha - pl.parts[1].alpha_ext == 13


def test_rejects_undefined_arguments():
    with pytest.raises(ValueError):
        orc.plan((16, 5, 15, 16), (1, 2, 2), 2, 1, overlap_patches=1)   # H not a multiple of p_H
    with pytest.raises(ValueError):
        orc.plan((16, 5, 16, 16), (1, 2, 2), 2, 1, r=1.5)               # r > K - 1
    with pytest.raises(ValueError):
        orc.plan((16, 5, 16, 16), (1, 2, 2), 2, 1, r=-0.1)
    with pytest.raises(ValueError):
        orc.plan((16, 5, 16, 16), (1, 2, 2), 0, 1)


shape_st = st.tuples(st.integers(1, 3), st.integers(1, 12), st.integers(1, 12), st.integers(1, 12))
patch_st = st.tuples(st.integers(1, 2), st.integers(1, 3), st.integers(1, 3))


@settings(max_examples=300, deadline=None)
@given(shape_st, patch_st, st.integers(1, 9), st.integers(0, 2), st.integers(0, 6))
def test_plan_invariants(npatches, patch, K, dim, O):
    latent = (npatches[0] + 1, npatches[1] * patch[0], npatches[2] * patch[1], npatches[3] * patch[2])
    N = npatches[1 + dim]
    L = -(-N // K)
    if O > L * (K - 1):
        with pytest.raises(ValueError):
            orc.plan(latent, patch, K, dim, overlap_patches=O)
        return
    pl = orc.plan(latent, patch, K, dim, overlap_patches=O)
    p = patch[dim]
    covered = [0] * (N * p)
    cores = [0] * N
    for k, q in enumerate(pl.parts):
        assert q.alpha == k * L and q.beta == q.alpha + L                      # Eq. 7
        assert q.s % p == 0 and q.e % p == 0                                   # patch aligned, Eq. 9
        assert 0 <= q.s <= q.e <= N * p
        assert q.len == q.e - q.s
        if q.len:
            assert q.alpha_ext == max(0, q.alpha - O) and q.beta_ext == min(N, q.beta + O)   # Eq. 8
            assert q.delta_start == (q.alpha - q.alpha_ext) * p                # Eq. 11
            assert q.delta_end == (q.beta_ext - q.beta) * p
        for x in range(q.s, q.e):
            covered[x] += 1
        for a in range(min(q.alpha, N), min(q.beta, N)):
            cores[a] += 1
    assert all(c >= 1 for c in covered)          # the partitions cover the latent
    assert all(c == 1 for c in cores)            # clamped cores tile [0, N)
    # packed layout: back to back in k order
    off = 0
    for q in pl.parts:
        assert q.elem_offset == off
        assert q.n_elems == math.prod(q.shape)
        off += q.n_elems
    assert pl.total_elems == off
    gamma = pl.total_elems / math.prod(latent)
    assert 1.0 <= gamma <= K                     # supplement: gamma >= 1 and gamma / K <= 1


def test_gamma_monotone_in_r_and_K():
    latent = (16, 21, 60, 104)
    for dim in range(3):
        prev = 0.0
        for r in (0.0, 0.1, 0.25, 0.5, 0.75, 1.0, 1.5, 2.0, 3.0):
            g = orc.plan(latent, (1, 2, 2), 4, dim, r=r).total_elems
            assert g >= prev
            prev = g
    # in K at fixed overlap ratio, on an extent every K divides (no ceil effects)
    prev = orc.plan((4, 4, 120, 8), (1, 2, 2), 1, 1, r=0.0).total_elems   # K = 1 admits r = 0 only
    for K in (2, 3, 4, 5, 6):
        g = orc.plan((4, 4, 120, 8), (1, 2, 2), K, 1, r=0.5).total_elems
        assert g >= prev
        prev = g


def _reach(latent, patch, K, O, dims):
    """Receptive field of one position after partitioning along dims[0] then dims[1]
    (attention mixes everything inside a sub-latent).  Returns the set of positions."""
    T, H, W = latent[1:]
    start = {(0, 0, 0)}
    cur = start
    for d in dims:
        pl = orc.plan(latent, patch, K, d, overlap_patches=O)
        nxt = set()
        for q in pl.parts:
            inside = [pos for pos in cur if q.s <= pos[d] < q.e]
            if not inside:
                continue
            rng = [range(T), range(H), range(W)]
            rng[d] = range(q.s, q.e)
            nxt.update((t, h, w) for t in rng[0] for h in rng[1] for w in rng[2])
        cur = nxt
    return cur


@pytest.mark.parametrize("dims", [(0, 1), (1, 2), (2, 0)])
def test_two_completeness(dims):
    # Theorem 1 (supplement): after two consecutive steps (different dims) the
    # receptive field of any position is the whole latent -- even with no overlap.
    latent = (2, 6, 8, 8)
    got = _reach(latent, (1, 2, 2), 3, 0, dims)
    assert len(got) == 6 * 8 * 8
    # one step alone is not complete
    assert len(_reach(latent, (1, 2, 2), 3, 0, dims[:1])) < 6 * 8 * 8
