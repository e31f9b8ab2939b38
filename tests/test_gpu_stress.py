"""Config 4 (compression / retrieval stress at the LingBot shape) at full size on the GPU:
a batch of 64 chunks compressed at P in {0.25, 0.5, 0.75}, top-16 retrieval over a 1,000-chunk store
indexed by walked poses and by integrated action labels, and the window gathered from pinned host
memory.  One chunk of the batch is compressed by the whole oracle at each ratio (all scores, kept-index set,
compacted rows); for the other 63 the oracle checks sampled scores and the rest is checked by properties
that hold at any size (exact selection of the GPU's own scores, byte-exact copies)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2605_22718_amd as wk
import wk_synth as ws
from wkt import assert_selection_matches, bits, dev

pytestmark = pytest.mark.gpu
BATCH, POOL = 64, 64


@pytest.fixture(scope="module")
def batch64():
    cfg = ws.get_config(4)
    d = dev()
    K = torch.empty((BATCH, cfg.H, cfg.chunk_tokens, cfg.d), dtype=torch.bfloat16, device=d)
    V = torch.empty_like(K)
    for c in range(BATCH):
        k, v, _ = ws.make_chunk(cfg, c, d)
        K[c], V[c] = k, v
    return cfg, K, V


_ORACLE_CHUNK = 5      # the chunk of the batch that the whole oracle compresses, once per ratio
_ORACLE_CACHE = {}


def _oracle_chunk(cfg, K, V, P):
    if P not in _ORACLE_CACHE:
        _ORACLE_CACHE[P] = oracle.compress(K[_ORACLE_CHUNK].cpu(), V[_ORACLE_CHUNK].cpu(), None, cfg.T, cfg.F, P,
                                           wk.WK_RATIO_NONANCHOR)
    return _ORACLE_CACHE[P]


@pytest.mark.timeout(600)
@pytest.mark.parametrize("algo", [wk.WK_SCORE_FACTORED, wk.WK_SCORE_GEMM])
@pytest.mark.parametrize("P,n_out", [(0.25, 2340), (0.5, 3120), (0.75, 3900)])
def test_batch_compress_at_three_ratios(batch64, P, n_out, algo):
    cfg, K, V = batch64
    d = dev()
    desc = wk.make_compress_desc(cfg.H, cfg.T, cfg.F, cfg.dtype, P, batch=BATCH, ratio_kind=wk.WK_RATIO_NONANCHOR,
                                 score_algo=algo)
    wsb = torch.empty(wk.wk_compress_workspace_bytes(desc), dtype=torch.uint8, device=d)
    idx = torch.empty((BATCH, 1, n_out), dtype=torch.int32, device=d)
    Ko = torch.empty((BATCH, cfg.H, n_out, cfg.d), dtype=torch.bfloat16, device=d)
    Vo = torch.empty_like(Ko)
    assert wk.wk_compress_chunk(desc, K, V, None, idx, Ko, Vo, wsb) == n_out
    torch.cuda.synchronize()
    n_cand, n_keep = 2 * cfg.T, n_out - cfg.T
    scores = wsb[: BATCH * n_cand * 8].view(torch.float64).view(BATCH, n_cand)
    # the kept set is exactly the n_keep lowest of the scores, ties to the lower index (checked on the GPU
    # with a stable sort of the same fp64 scores), anchors kept in full, indices ascending
    order = torch.sort(scores, dim=1, stable=True).indices[:, :n_keep]
    expect = torch.sort(order, dim=1).values.to(torch.int32) + cfg.T
    assert torch.equal(idx[:, 0, cfg.T:], expect)
    assert torch.equal(idx[:, 0, :cfg.T], torch.arange(cfg.T, dtype=torch.int32, device=d).expand(BATCH, -1))
    # compaction is a verbatim row copy, for K and V, every chunk and head
    gi = idx[:, 0].long()
    for b in (0, 31, 63):
        sel = gi[b]
        assert torch.equal(bits(Ko[b]), bits(K[b][:, sel])) and torch.equal(bits(Vo[b]), bits(V[b][:, sel]))
    # one chunk of the batch against the whole oracle: all 3,120 scores, the kept-index set, the compacted rows
    o_idx, o_K, o_V, o_scores = _oracle_chunk(cfg, K, V, P)
    b = _ORACLE_CHUNK
    assert np.abs(scores[b].cpu().numpy() - o_scores[0]).max() <= 1e-7
    g_idx = idx[b, 0].cpu().numpy()
    np.testing.assert_array_equal(g_idx[:cfg.T], o_idx[0, :cfg.T])
    assert_selection_matches(g_idx[cfg.T:] - cfg.T, o_idx[0, cfg.T:] - cfg.T, o_scores[0], f"chunk {b} at P={P}")
    if np.array_equal(g_idx, o_idx[0]):
        assert torch.equal(bits(Ko[b].cpu()), bits(o_K)) and torch.equal(bits(Vo[b].cpu()), bits(o_V))
    # oracle scores on sampled candidates of two more chunks
    rng = np.random.default_rng(int(P * 100))
    sel = np.unique(np.concatenate([[0, n_cand - 1], rng.integers(0, n_cand, 24)])).astype(np.int32)
    for b in (17, 40):
        o = oracle.compress_scores(K[b].cpu(), None, cfg.T, cfg.F, cand_sel=sel)
        assert np.abs(scores[b].cpu().numpy()[sel] - o[0, sel]).max() <= 1e-7


def test_retrieval_over_1000_chunks_and_gather_from_pinned_host(batch64):
    cfg, K, V = batch64
    d = dev()
    n_out = 2340
    # store payloads: POOL compressed chunks in pinned host memory back 1,000 logical chunk ids (id mod POOL)
    desc = wk.make_compress_desc(cfg.H, cfg.T, cfg.F, cfg.dtype, 0.25, batch=POOL, ratio_kind=wk.WK_RATIO_NONANCHOR)
    wsb = torch.empty(wk.wk_compress_workspace_bytes(desc), dtype=torch.uint8, device=d)
    pool_k = torch.empty((POOL, cfg.H, n_out, cfg.d), dtype=torch.bfloat16, pin_memory=True)
    pool_v = torch.empty_like(pool_k).pin_memory()
    wk.wk_compress_chunk(desc, K[:POOL], V[:POOL], None, None, pool_k, pool_v, wsb)   # K_out/V_out in mapped host memory
    torch.cuda.synchronize()
    store = wk.Store([pool_k[c % POOL] for c in range(cfg.M)], [pool_v[c % POOL] for c in range(cfg.M)])
    tables = []
    poses, cur = ws.make_poses(cfg.M, cfg.seed)
    tables.append((poses, cur))
    acts = wk.wk_accumulate_actions(ws.make_action_labels(cfg.M, cfg.seed)).numpy()
    tables.append((acts, acts[123]))
    for table, cur_pose in tables:
        ids = torch.empty(cfg.R, dtype=torch.int32, device=d)
        nf = torch.empty(1, dtype=torch.int32, device=d)
        wk.wk_score_chunks(torch.from_numpy(table).to(d), cfg.M, cur_pose, wk.WK_NORM_MAX, cfg.R, ids, None, nf)
        cap = cfg.R * n_out
        Kw = torch.zeros((cfg.H, cap, cfg.d), dtype=torch.bfloat16, device=d)
        Vw = torch.zeros_like(Kw)
        n_win = torch.empty(1, dtype=torch.int32, device=d)
        wk.wk_gather_window(store.desc, ids, nf, cfg.R, None, None, 0, Kw, Vw, cap, n_win)
        torch.cuda.synchronize()
        o_ids, o_d, o_all = oracle.score_chunks(table, cur_pose, cfg.R)
        g = ids.cpu().numpy()
        if not np.array_equal(g, o_ids):     # interchangeable only within the tie band
            assert np.abs(o_all[g] - o_d).max() < 1e-6
        assert int(n_win.item()) == cap
        for r in (0, 7, 15):
            c = int(g[r]) % POOL
            assert torch.equal(bits(Kw[:, r * n_out:(r + 1) * n_out].cpu()), bits(pool_k[c]))
            assert torch.equal(bits(Vw[:, r * n_out:(r + 1) * n_out].cpu()), bits(pool_v[c]))
    # the pinned payloads are the compressed chunks: compare one with a device-side compression
    d1 = wk.make_compress_desc(cfg.H, cfg.T, cfg.F, cfg.dtype, 0.25, ratio_kind=wk.WK_RATIO_NONANCHOR)
    w1 = torch.empty(wk.wk_compress_workspace_bytes(d1), dtype=torch.uint8, device=d)
    k1 = torch.empty((cfg.H, n_out, cfg.d), dtype=torch.bfloat16, device=d)
    v1 = torch.empty_like(k1)
    wk.wk_compress_chunk(d1, K[9], V[9], None, None, k1, v1, w1)
    torch.cuda.synchronize()
    assert torch.equal(bits(k1.cpu()), bits(pool_k[9])) and torch.equal(bits(v1.cpu()), bits(pool_v[9]))
