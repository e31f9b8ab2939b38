"""Run-twice determinism: every entry point, called twice on the same inputs, must return the same bits
(no atomics on results, fixed reduction orders, fixed merge order of key-range splits)."""
import numpy as np
import pytest
import torch

import paper_2605_22718_amd as wk
import wk_synth as ws
from wkt import dev

pytestmark = pytest.mark.gpu


def _same(a, b):
    return all(torch.equal(x.view(torch.uint8), y.view(torch.uint8)) for x, y in zip(a, b))


def _twice(fn):
    a = fn()
    torch.cuda.synchronize()
    b = fn()
    torch.cuda.synchronize()
    assert _same(a, b)


@pytest.mark.parametrize("algo", [wk.WK_SCORE_FACTORED, wk.WK_SCORE_GEMM])
@pytest.mark.parametrize("head_mode", [wk.WK_HEADS_SHARED, wk.WK_HEADS_INDEPENDENT])
def test_compress(head_mode, algo):
    d = dev()
    cfg = ws.get_config(1).with_(H=6, T=333)
    K, V, _ = ws.make_chunk(cfg, 2, d)
    desc = wk.make_compress_desc(cfg.H, cfg.T, cfg.F, cfg.dtype, 0.5, head_mode=head_mode, score_algo=algo)
    n_out, _ = wk.wk_keep_count(0.5, wk.WK_RATIO_CHUNK, cfg.anchor_mode, cfg.F, cfg.T)
    G = cfg.H if head_mode == wk.WK_HEADS_INDEPENDENT else 1

    def run():
        wsb = torch.zeros(wk.wk_compress_workspace_bytes(desc), dtype=torch.uint8, device=d)
        idx = torch.zeros((G, n_out), dtype=torch.int32, device=d)
        Ko = torch.zeros((cfg.H, n_out, cfg.d), dtype=K.dtype, device=d)
        Vo = torch.zeros_like(Ko)
        wk.wk_compress_chunk(desc, K, V, None, idx, Ko, Vo, wsb)
        n_cand = (cfg.F - 1) * cfg.T
        return idx, Ko, Vo, wsb[: G * n_cand * 8].clone()     # the Eq. 5 scores, bit for bit
    _twice(run)


def test_retrieval_gather_and_attention_variants():
    d = dev()
    cfg = ws.get_config(1).with_(H=5, T=200, M=40, R=4)
    poses, cur = ws.make_poses(cfg.M, cfg.seed)
    poses_d = torch.from_numpy(poses).to(d)
    n_tok = 300
    ks = [ws.make_native(cfg.with_(index=80 + c), d, n_rows=n_tok)[0] for c in range(cfg.M)]
    vs = [ws.make_native(cfg.with_(index=80 + c), d, n_rows=n_tok)[1] for c in range(cfg.M)]
    store = wk.Store(ks, vs)
    Q = ws.make_queries(cfg, d)
    Kn, Vn = ws.make_native(cfg, d)
    cap = cfg.n_native + cfg.R * n_tok

    def path():
        ids = torch.zeros(cfg.R, dtype=torch.int32, device=d)
        dist = torch.zeros(cfg.R, dtype=torch.float64, device=d)
        nf = torch.zeros(1, dtype=torch.int32, device=d)
        wk.wk_score_chunks(poses_d, cfg.M, cur, wk.WK_NORM_MAX, cfg.R, ids, dist, nf)
        Kw = torch.zeros((cfg.H, cap, cfg.d), dtype=torch.bfloat16, device=d)
        Vw = torch.zeros_like(Kw)
        n_win = torch.zeros(1, dtype=torch.int32, device=d)
        wk.wk_gather_window(store.desc, ids, nf, cfg.R, Kn, Vn, cfg.n_native, Kw, Vw, cap, n_win)
        O = torch.zeros_like(Q)
        lse = torch.zeros(Q.shape[:2], dtype=torch.float32, device=d)
        wk.wk_attention(Q, Kw, Vw, O, lse, N_kv=cap, n_kv_dev=n_win)
        O2 = torch.zeros_like(Q)
        lse2 = torch.zeros_like(lse)
        wk.wk_attention_in_place(Q, Kn, Vn, cfg.n_native, store.desc, ids, nf, cfg.R, O2, lse2)
        O3 = torch.zeros_like(Q)
        wsb = torch.zeros(wk.wk_attention_block_causal_workspace_bytes(cfg.H, cfg.N_q), dtype=torch.uint8, device=d)
        wk.wk_attention_block_causal(Q, Kw, Vw, O3, cfg.n_native - cfg.N_q, cfg.T, wsb, N_kv=cap)
        return ids, dist, nf, Kw, Vw, n_win, O, lse, O2, lse2, O3
    _twice(path)


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_attention_with_key_range_splits(dtype):
    """Few (head, query tile) items over a long window: partial results of the splits are merged in a fixed order."""
    d = dev()
    g = torch.Generator().manual_seed(3)
    H, N_q, N_kv = 2, 300, 6000
    Q = torch.randn(H, N_q, 128, generator=g).to(dtype).to(d)
    K = torch.randn(H, N_kv, 128, generator=g).to(dtype).to(d)
    V = torch.randn(H, N_kv, 128, generator=g).to(dtype).to(d)
    need = wk.wk_attention_workspace_bytes(H, N_q, N_kv, wk.WK_BF16 if dtype == torch.bfloat16 else wk.WK_F32)
    assert need > 0

    def run():
        wsb = torch.zeros(need, dtype=torch.uint8, device=d)
        O = torch.zeros_like(Q)
        lse = torch.zeros((H, N_q), dtype=torch.float32, device=d)
        wk.wk_attention(Q, K, V, O, lse, workspace=wsb)
        return O, lse
    _twice(run)


def test_query_based_retrieval_and_window_update():
    d = dev()
    cfg = ws.get_config(1).with_(H=4, T=100)
    Q = ws.make_queries(cfg, d)
    lens = [150] * 10
    ks, _ = ws.make_revisit_keys(cfg, Q, lens, d)
    vs = [k.clone() for k in ks]
    store = wk.Store(ks, vs)
    M, R = len(lens), 3
    n_rows = cfg.H * cfg.N_q

    def query():
        lse = torch.zeros((M, cfg.H, cfg.N_q), dtype=torch.float32, device=d)
        wk.wk_chunk_lse(store.desc, Q, lse)
        wsb = torch.zeros(wk.wk_score_chunks_query_workspace_bytes(M, n_rows), dtype=torch.uint8, device=d)
        ids = torch.zeros(R, dtype=torch.int32, device=d)
        mass = torch.zeros(R, dtype=torch.float64, device=d)
        nf = torch.zeros(1, dtype=torch.int32, device=d)
        wk.wk_score_chunks_query(lse.view(M, n_rows), M, n_rows, R, ids, mass, nf, wsb)
        return lse, ids, mass, nf, wsb[: M * 8].clone()
    _twice(query)

    def update():
        slot_ids = torch.tensor([7, -1, 2], dtype=torch.int32, device=d)
        ids = torch.tensor([2, 5, 9], dtype=torch.int32, device=d)
        cap = 64 + R * 150
        Kw = torch.zeros((cfg.H, cap, cfg.d), dtype=torch.bfloat16, device=d)
        Vw = torch.zeros_like(Kw)
        n_win = torch.zeros(1, dtype=torch.int32, device=d)
        n_f = torch.zeros(1, dtype=torch.int32, device=d)
        wsb = torch.zeros(wk.wk_window_update_workspace_bytes(R), dtype=torch.uint8, device=d)
        wk.wk_window_update(store.desc, ids, None, R, 150, slot_ids, 64, Kw, Vw, cap, n_win, n_f, wsb)
        return slot_ids, Kw, Vw, n_win, n_f
    _twice(update)
