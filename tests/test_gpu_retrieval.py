"""GPU parity of wk_score_chunks against the oracle (Sec. 4.2 Eq. 4, Sec. 5.1 distance)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2605_22718_amd as wk
import wk_synth as ws
from wkt import TIE_BAND, dev

pytestmark = pytest.mark.gpu


def _gpu_score(poses, cur, R, norm_mode=wk.WK_NORM_MAX):
    d = dev()
    M = poses.shape[0]
    p = torch.from_numpy(np.ascontiguousarray(poses, np.float32)).to(d) if M else torch.zeros((1, 5), device=d)
    ids = torch.full((max(R, 1),), -7, dtype=torch.int32, device=d)
    dist = torch.full((max(R, 1),), -7.0, dtype=torch.float64, device=d)
    nf = torch.full((1,), -7, dtype=torch.int32, device=d)
    wk.wk_score_chunks(p, M, cur, norm_mode, R, ids, dist, nf)
    torch.cuda.synchronize()
    return ids.cpu().numpy()[:R], dist.cpu().numpy()[:R], int(nf.item())


def _compare(poses, cur, R, norm_mode=wk.WK_NORM_MAX):
    ids, dist, nf = _gpu_score(poses, cur, R, norm_mode)
    o_ids, o_d, o_all = oracle.score_chunks(poses, cur, R, norm_mode)
    assert nf == o_ids.size == min(R, poses.shape[0])
    assert np.all(ids[nf:] == -1) and np.all(np.isinf(dist[nf:]))
    g = ids[:nf]
    assert len(set(g.tolist())) == nf
    np.testing.assert_allclose(dist[:nf], o_all[g], rtol=0, atol=1e-7)
    assert np.all(np.diff(dist[:nf]) >= 0)
    if not np.array_equal(g, o_ids):
        # positions may differ only between candidates whose fp64 distances are within the tie band
        assert np.abs(o_all[g] - o_d).max() < TIE_BAND
    return g


@pytest.mark.parametrize("M", [1, 2, 16, 60, 120, 1000, 1025, 4096])
@pytest.mark.parametrize("norm_mode", [wk.WK_NORM_MAX, wk.WK_NORM_MINMAX, wk.WK_NORM_MEAN])
def test_looping_trajectories(M, norm_mode):
    poses, cur = ws.make_poses(M, 1000 + M)
    for R in sorted({0, 1, 2, min(M, 16), M, M + 5} if M <= 120 else {2, 16}):
        g = _compare(poses, cur, R, norm_mode)
        if norm_mode == wk.WK_NORM_MAX and R == 2 and M >= 16:
            assert set(g.tolist()) == {0, M - 1}        # the planted loop closure


def test_empty_store_and_exact_ties():
    ids, dist, nf = _gpu_score(np.zeros((0, 5), np.float32), np.zeros(5, np.float32), 3)
    assert nf == 0 and np.all(ids == -1)
    rng = np.random.default_rng(5)
    for _ in range(10):
        poses = rng.integers(-2, 3, (40, 5)).astype(np.float32)    # coarse grid: many exact ties
        poses[:, 3:] *= 0.5
        cur = rng.integers(-1, 2, 5).astype(np.float32)
        g = _compare(poses, cur, 12)
    # all candidates in one place and one orientation: every distance is 0, ids come out 0,1,2,...
    poses = np.tile(np.array([[1, 2, 3, 0.5, 0.1]], np.float32), (9, 1))
    g = _compare(poses, poses[0], 4)
    np.testing.assert_array_equal(g, [0, 1, 2, 3])


def test_action_integrated_poses():
    labels = ws.make_action_labels(1000, 77)
    poses = wk.wk_accumulate_actions(labels).numpy()
    _compare(poses, poses[400], 16)
