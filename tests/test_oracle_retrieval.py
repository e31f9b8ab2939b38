"""Pins for the oracle's World Retrieval (Sec. 4.2 Eq. 4, Sec. 5.1 distance) -- CPU only."""
import math
import os

import numpy as np
import pytest
from scipy.spatial.transform import Rotation

import oracle
import wk_synth as ws

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _wrap(a):
    return (a + math.pi) % (2 * math.pi) - math.pi


def test_geodesic_special_cases():
    assert oracle.geodesic(0.3, -0.2, 0.3, -0.2) < 2e-8   # arccos near 1 limits this to ~1.5e-8
    for d in [0.1, 1.0, 3.0, -2.5, 4.0, 6.0]:
        assert abs(oracle.geodesic(0.7, 0.0, 0.7 + d, 0.0) - abs(_wrap(d))) < 1e-9
    for d in [0.1, 1.0, -0.9]:   # same yaw, pitch differing by d
        assert abs(oracle.geodesic(1.1, 0.2, 1.1, 0.2 + d) - abs(d)) < 1e-9
    assert abs(oracle.geodesic(0, 0, math.pi, 0) - math.pi) < 1e-7


def test_geodesic_matches_quaternion_library_and_closed_form():
    rng = np.random.default_rng(0)
    for _ in range(200):
        ya, pa, yb, pb = rng.uniform(-math.pi, math.pi, 4)
        got = oracle.geodesic(ya, pa, yb, pb)
        Ra = Rotation.from_euler("YX", [ya, pa])   # intrinsic: R_y(yaw) R_x(pitch)
        Rb = Rotation.from_euler("YX", [yb, pb])
        lib = (Ra.inv() * Rb).magnitude()
        assert abs(got - lib) < 1e-7, (got, lib)
        # rotation angle depends only on the yaw and pitch differences
        cD, cd = math.cos(yb - ya), math.cos(pb - pa)
        closed = math.acos(max(-1.0, min(1.0, (cD + cd + cD * cd - 1.0) / 2.0)))
        assert abs(got - closed) < 1e-7
        assert abs(got - oracle.geodesic(yb, pb, ya, pa)) < 1e-7   # symmetric
        assert 0.0 <= got <= math.pi


def test_retrieval_hand_values():
    rows = []
    for line in open(os.path.join(GOLD, "retrieval_hand.txt")):
        line = line.strip()
        if line and not line.startswith("#"):
            rows.append([float(x) for x in line.split()])
    poses = np.array([[r[0], r[1], r[2], r[3] * math.pi, r[4] * math.pi] for r in rows], np.float32)
    ids, d_sel, d_all = oracle.score_chunks(poses, np.zeros(5, np.float32), 4)
    np.testing.assert_allclose(d_all, [r[5] for r in rows], atol=1e-6)  # float32 pi in the inputs
    # chunks 1 and 3 tie at 0.5 up to the float32 rounding of the angles; both follow chunk 0
    assert ids[0] == 0 and set(ids[1:3]) == {1, 3} and ids[3] == 2


def test_topk_brute_force_and_ties():
    rng = np.random.default_rng(1)
    for M in [1, 2, 5, 16]:
        for _ in range(20):
            poses = rng.integers(-2, 3, (M, 5)).astype(np.float32)   # coarse grid: many exact ties
            poses[:, 3:] *= 0.5
            cur = rng.integers(-1, 2, 5).astype(np.float32)
            for R in [0, 1, 2, M, M + 3]:
                ids, d_sel, d_all = oracle.score_chunks(poses, cur, R)
                order = np.lexsort((np.arange(M), d_all))[: min(R, M)]
                np.testing.assert_array_equal(ids, order)
                np.testing.assert_array_equal(d_sel, d_all[order])
    ids, _, _ = oracle.score_chunks(np.zeros((0, 5), np.float32), np.zeros(5, np.float32), 3)
    assert ids.size == 0
    # exact ties go to the lower (older) chunk id
    poses = np.array([[1, 0, 0, 0, 0], [-1, 0, 0, 0, 0], [0, 0, 1, 0, 0], [5, 0, 0, 1, 0]], np.float32)
    ids, _, _ = oracle.score_chunks(poses, np.zeros(5, np.float32), 2)
    np.testing.assert_array_equal(ids, [0, 1])


def test_max_normalisation_invariants():
    poses, cur = ws.make_poses(40, 123)
    ids, d_sel, d_all = oracle.score_chunks(poses, cur, 6)
    # both terms lie in [0, 1]
    assert d_all.min() >= 0 and d_all.max() <= 2.0 + 1e-12
    # scaling all translations (stored and current) by c > 0 leaves D unchanged
    p2, c2 = poses.copy(), cur.copy()
    p2[:, :3] *= 4.0
    c2[:3] *= 4.0
    ids2, _, d_all2 = oracle.score_chunks(p2, c2, 6)
    np.testing.assert_allclose(d_all2, d_all, atol=1e-12)
    np.testing.assert_array_equal(ids2, ids)
    # a stored pose equal to the current one has D = 0 and ranks first
    p3 = poses.copy()
    p3[17] = cur
    ids3, d3, _ = oracle.score_chunks(p3, cur, 3)
    assert ids3[0] == 17 and d3[0] < 1e-7
    # all candidates at the same place: the translation term is 0, not NaN
    p4 = poses.copy()
    p4[:, :3] = cur[:3]
    _, _, d4 = oracle.score_chunks(p4, cur, 3)
    assert np.isfinite(d4).all() and d4.max() <= 1.0 + 1e-12


@pytest.mark.parametrize("M", [16, 60, 120, 1000])
def test_planted_loop_closure_is_retrieved(M):
    poses, cur = ws.make_poses(M, ws.get_config(1).seed)
    ids, _, _ = oracle.score_chunks(poses, cur, 2)
    assert set(ids) == {0, M - 1}


def test_normalisation_variants_are_defined():
    poses, cur = ws.make_poses(30, 9)
    dt = ((poses[:, :3].astype(np.float64) - cur[:3].astype(np.float64)) ** 2).sum(1)
    dr = np.array([oracle.geodesic(float(cur[3]), float(cur[4]), float(p[3]), float(p[4])) for p in poses])
    _, _, d_max = oracle.score_chunks(poses, cur, 1, oracle.NORM_MAX)
    _, _, d_mm = oracle.score_chunks(poses, cur, 1, oracle.NORM_MINMAX)
    _, _, d_mean = oracle.score_chunks(poses, cur, 1, oracle.NORM_MEAN)
    np.testing.assert_allclose(d_max, dt / dt.max() + dr / dr.max(), atol=1e-12)
    np.testing.assert_allclose(d_mm, (dt - dt.min()) / (dt.max() - dt.min()) + (dr - dr.min()) / (dr.max() - dr.min()),
                               atol=1e-12)
    np.testing.assert_allclose(d_mean, dt / dt.mean() + dr / dr.mean(), atol=1e-12)


def test_accumulate_actions_closed_cases():
    W, A, S, D, YM, YP, PM, PP = range(8)
    deg15 = math.radians(15)
    p = oracle.accumulate_actions([YP] * 4 + [W])
    np.testing.assert_allclose(p[-1], [math.sin(4 * deg15), 0, math.cos(4 * deg15), 4 * deg15, 0], atol=1e-6)
    p = oracle.accumulate_actions([YM] * 2 + [W])   # yaw- turns the heading towards -x
    np.testing.assert_allclose(p[-1], [-math.sin(2 * deg15), 0, math.cos(2 * deg15), -2 * deg15, 0], atol=1e-6)
    p = oracle.accumulate_actions([YM, YP, PM, PP])
    np.testing.assert_allclose(p[-1], 0, atol=1e-7)
    p = oracle.accumulate_actions([W, W, S, S])
    np.testing.assert_allclose(p[-1], 0, atol=1e-7)
    np.testing.assert_allclose(p[1], [0, 0, 2, 0, 0], atol=1e-7)
    p = oracle.accumulate_actions([A])           # left of heading +z is -x
    np.testing.assert_allclose(p[0], [-1, 0, 0, 0, 0], atol=1e-7)
    p = oracle.accumulate_actions([D, A])
    np.testing.assert_allclose(p[-1], 0, atol=1e-7)
    p = oracle.accumulate_actions([PP] * 6)      # clamped at 60 degrees
    assert abs(p[-1, 4] - math.radians(60)) < 1e-6 and abs(p[3, 4] - math.radians(60)) < 1e-6
    p = oracle.accumulate_actions([PM] * 9)
    assert abs(p[-1, 4] + math.radians(60)) < 1e-6
    # a square: (forward, turn 90 degrees) four times returns to the start
    p = oracle.accumulate_actions(([W] + [YP] * 6) * 4)
    np.testing.assert_allclose(p[-1, :3], 0, atol=1e-6)
    assert abs(p[-1, 3] - 2 * math.pi) < 1e-5
    with pytest.raises(ValueError):
        oracle.accumulate_actions([8])
    # integrated labels give a valid pose table for retrieval
    labels = ws.make_action_labels(1000, 5)
    poses = oracle.accumulate_actions(labels)
    assert poses.shape == (1000, 5) and np.isfinite(poses).all()
    ids, _, _ = oracle.score_chunks(poses, poses[500], 4)
    assert ids[0] == 500 or np.allclose(poses[ids[0]], poses[500])


# ---- query-based retrieval (Sec. 4.2, App. C) ---------------------------------------------------

def _query_setup(seed=0, H=2, Nq=9, d=8, lens=(5, 7, 3, 6)):
    import torch
    g = torch.Generator().manual_seed(seed)
    Q = torch.randn(H, Nq, d, generator=g)
    Ks = [torch.randn(H, n, d, generator=g) for n in lens]
    return Q, Ks


def test_query_retrieval_mass_against_library_softmax():
    import torch
    Q, Ks = _query_setup(1)
    ids, m_sel, m_all = oracle.score_chunks_query(Q, Ks, 2)
    K_all = torch.cat(Ks, 1).double()
    P = torch.softmax(torch.einsum("hqd,hkd->hqk", Q.double(), K_all) / math.sqrt(Q.shape[-1]), -1)
    bounds = np.cumsum([0] + [k.shape[1] for k in Ks])
    expect = np.array([P[:, :, bounds[c]:bounds[c + 1]].sum(-1).mean().item() for c in range(len(Ks))])
    np.testing.assert_allclose(m_all, expect, atol=1e-14)
    assert abs(m_all.sum() - 1.0) < 1e-13                    # masses of all candidates sum to one
    order = np.lexsort((np.arange(len(Ks)), -m_all))[:2]
    np.testing.assert_array_equal(ids, order)
    np.testing.assert_allclose(m_sel, m_all[order], atol=0)
    # the mass of a chunk is what attention returns for V = indicator of that chunk (window = all candidates)
    ind = torch.zeros(K_all.shape[0], K_all.shape[1], Q.shape[-1])
    ind[:, bounds[2]:bounds[3]] = 1.0
    mass2 = oracle.attention(Q, torch.cat(Ks, 1).contiguous(), ind.contiguous())[..., 0].mean()
    assert abs(mass2 - m_all[2]) < 1e-14


def test_query_retrieval_invariants():
    import torch
    Q, Ks = _query_setup(2)
    _, _, base = oracle.score_chunks_query(Q, Ks, 4)
    # a chunk holding copies of the queries (scaled up) draws almost all the mass
    Ks2 = list(Ks)
    Ks2[1] = (Q[:, :7] * 4.0).contiguous()
    ids, m_sel, m_all = oracle.score_chunks_query(Q, Ks2, 1)
    assert ids[0] == 1 and m_all[1] > 0.5
    # duplicating a chunk under a new id: both copies get the same mass, the lower id ranks first
    Ks3 = Ks + [Ks[2].clone()]
    ids, _, m3 = oracle.score_chunks_query(Q, Ks3, 5)
    assert abs(m3[2] - m3[4]) < 1e-15 and list(ids).index(2) < list(ids).index(4)
    # one candidate: mass 1; R > M; empty store
    ids, m_sel, m_all = oracle.score_chunks_query(Q, Ks[:1], 3)
    assert list(ids) == [0] and abs(m_all[0] - 1.0) < 1e-14
    ids, _, _ = oracle.score_chunks_query(Q, [], 3)
    assert ids.size == 0
    # adding a constant vector to every key of every chunk changes nothing
    c = torch.tensor([0.5, -1.0] * 4)
    Ks4 = [((k * 64).round() / 64) for k in Ks]
    _, _, a = oracle.score_chunks_query(Q, Ks4, 4)
    _, _, b = oracle.score_chunks_query(Q, [(k + c).contiguous() for k in Ks4], 4)
    np.testing.assert_allclose(a, b, atol=1e-13)
