"""Whole hot path on the GPU (compress -> score -> gather -> attention) against the same path
through the oracle, plus the invariants the method fixes (Sec. 4.1, Sec. 5.4)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2605_22718_amd as wk
import wk_synth as ws
from wkt import (ATT_MAX_ABS_BF16, ATT_MAX_ABS_F32, ATT_MEAN_ABS_BF16, assert_attention_close_bf16,
                 assert_selection_matches, attention_errors, bits, dev, sample_rows)

pytestmark = pytest.mark.gpu


def _gpu_path(cfg, chunks, poses, cur, Q, Kn, Vn, rho=None, R=None):
    d = dev()
    dt = ws.torch_dtype(cfg.dtype)
    rho = cfg.rho if rho is None else rho
    R = cfg.R if R is None else R
    n_out, _ = wk.wk_keep_count(rho, cfg.ratio_kind, cfg.anchor_mode, cfg.F, cfg.T)
    desc = wk.make_compress_desc(cfg.H, cfg.T, cfg.F, cfg.dtype, rho, ratio_kind=cfg.ratio_kind,
                                 anchor_mode=cfg.anchor_mode)
    wsb = torch.empty(wk.wk_compress_workspace_bytes(desc), dtype=torch.uint8, device=d)
    sk, sv, idxs = [], [], []
    for K, V, A in chunks:
        Ko = torch.empty((cfg.H, n_out, cfg.d), dtype=dt, device=d)
        Vo = torch.empty_like(Ko)
        idx = torch.empty((1, n_out), dtype=torch.int32, device=d)
        wk.wk_compress_chunk(desc, K.to(d), V.to(d), None if A is None else A.to(d), idx, Ko, Vo, wsb)
        sk.append(Ko), sv.append(Vo), idxs.append(idx)
    store = wk.Store(sk, sv)
    M = len(chunks)
    ids = torch.empty(max(R, 1), dtype=torch.int32, device=d)
    nf = torch.empty(1, dtype=torch.int32, device=d)
    wk.wk_score_chunks(torch.from_numpy(poses).to(d), M, cur, wk.WK_NORM_MAX, R, ids, None, nf)
    cap = Kn.shape[1] + R * n_out
    Kw = torch.zeros((cfg.H, cap, cfg.d), dtype=dt, device=d)
    Vw = torch.zeros_like(Kw)
    n_win = torch.empty(1, dtype=torch.int32, device=d)
    wk.wk_gather_window(store.desc, ids, nf, R, Kn.to(d), Vn.to(d), Kn.shape[1], Kw, Vw, cap, n_win)
    O = torch.empty(Q.shape, dtype=dt, device=d)
    wk.wk_attention(Q.to(d), Kw, Vw, O, None, N_kv=cap, n_kv_dev=n_win)     # no host sync anywhere above
    torch.cuda.synchronize()
    return dict(idx=[i.cpu().numpy() for i in idxs], ids=ids.cpu().numpy()[:R], n_win=int(n_win.item()),
                Kw=Kw.cpu(), Vw=Vw.cpu(), O=O, n_out=n_out, cap=cap)


def _oracle_path(cfg, chunks, poses, cur, Q, Kn, Vn, rows=None, rho=None, R=None):
    rho = cfg.rho if rho is None else rho
    R = cfg.R if R is None else R
    comp = [oracle.compress(K, V, A, cfg.T, cfg.F, rho, cfg.ratio_kind, anchor_mode=cfg.anchor_mode)
            for K, V, A in chunks]
    ids, _, _ = oracle.score_chunks(poses, cur, R)
    n_out = comp[0][1].shape[1]
    cap = Kn.shape[1] + R * n_out
    Kw, Vw, n_win = oracle.gather([c[1] for c in comp], [c[2] for c in comp], ids, Kn, Vn, cap)
    O = oracle.attention(Q, Kw, Vw, N_kv=n_win, rows=rows)
    return dict(idx=[c[0] for c in comp], ids=ids, n_win=n_win, Kw=Kw, Vw=Vw, O=O)


def _assert_same(cfg, g, o, rows=None):
    for gi, oi in zip(g["idx"], o["idx"]):
        np.testing.assert_array_equal(gi, oi)          # kept-token sets, bit-exact on these seeds
    np.testing.assert_array_equal(g["ids"], o["ids"])  # retrieved chunk ids
    assert g["n_win"] == o["n_win"]
    assert torch.equal(bits(g["Kw"]), bits(o["Kw"])) and torch.equal(bits(g["Vw"]), bits(o["Vw"]))
    Og = g["O"] if rows is None else g["O"][:, torch.as_tensor(rows, dtype=torch.long)]
    mx, mean = attention_errors(Og, o["O"])
    if cfg.dtype == ws.configs.DT_F32:
        assert mx <= ATT_MAX_ABS_F32, mx
    else:
        assert mx <= ATT_MAX_ABS_BF16 and mean <= ATT_MEAN_ABS_BF16, (mx, mean)
    return mx, mean


def test_config0_whole_path():
    cfg = ws.get_config(0)
    chunks = [ws.make_chunk(cfg, c) for c in range(cfg.M)]
    poses, cur = ws.make_poses(cfg.M, cfg.seed)
    Q, (Kn, Vn) = ws.make_queries(cfg), ws.make_native(cfg)
    g = _gpu_path(cfg, chunks, poses, cur, Q, Kn, Vn)
    o = _oracle_path(cfg, chunks, poses, cur, Q, Kn, Vn)
    assert g["n_win"] == 2640 and set(g["ids"].tolist()) == {0, cfg.M - 1}
    mx, mean = _assert_same(cfg, g, o)
    print(f"config0 whole path: max-abs {mx:.2e} mean-abs {mean:.2e}")


def _whole_path_full_store(cfg, n_random):
    """The path as the config defines it, store at full size: every chunk of the store is compressed by the
    GPU into the store (HBM, or pinned host memory written by the kernel through its mapped address), pose
    retrieval picks R of them, the window is assembled from the store and attended.  The oracle walks the
    same path; it compresses only the chunks its own retrieval returns, since the others reach no output."""
    d = dev()
    dt = ws.torch_dtype(cfg.dtype)
    pinned = cfg.store == "pinned"
    n_out, _ = wk.wk_keep_count(cfg.rho, cfg.ratio_kind, cfg.anchor_mode, cfg.F, cfg.T)
    # retrieval first (both sides), so that the raw rows of the retrieved chunks can be kept for the oracle
    poses, cur = ws.make_poses(cfg.M, cfg.seed)
    ids = torch.empty(cfg.R, dtype=torch.int32, device=d)
    nf = torch.empty(1, dtype=torch.int32, device=d)
    wk.wk_score_chunks(torch.from_numpy(poses).to(d), cfg.M, cur, wk.WK_NORM_MAX, cfg.R, ids, None, nf)
    o_ids, _, _ = oracle.score_chunks(poses, cur, cfg.R)
    np.testing.assert_array_equal(ids.cpu().numpy(), o_ids)            # retrieved chunk ids, bit-exact
    assert int(nf.item()) == cfg.R and {0, cfg.M - 1} <= set(o_ids.tolist())   # the planted loop closure
    # the store
    shape = (cfg.M, cfg.H, n_out, cfg.d)
    if pinned:
        store_k = torch.empty(shape, dtype=dt, pin_memory=True)
        store_v = torch.empty(shape, dtype=dt, pin_memory=True)
    else:
        store_k = torch.empty(shape, dtype=dt, device=d)
        store_v = torch.empty(shape, dtype=dt, device=d)
    desc = wk.make_compress_desc(cfg.H, cfg.T, cfg.F, cfg.dtype, cfg.rho, ratio_kind=cfg.ratio_kind,
                                 anchor_mode=cfg.anchor_mode)
    wsb = torch.empty(wk.wk_compress_workspace_bytes(desc), dtype=torch.uint8, device=d)
    raw, g_idx = {}, {}
    for c in range(cfg.M):
        K, V, _ = ws.make_chunk(cfg, c, d)
        idx = torch.empty((1, n_out), dtype=torch.int32, device=d)
        wk.wk_compress_chunk(desc, K, V, None, idx, store_k[c], store_v[c], wsb)
        if c in set(o_ids.tolist()):
            raw[c] = (K.cpu(), V.cpu())
            g_idx[c] = idx.cpu().numpy()[0]
    torch.cuda.synchronize()
    # kept-token sets and compacted rows of the retrieved chunks against the oracle
    comp = {}
    for c in o_ids.tolist():
        o_idx, o_K, o_V, o_scores = oracle.compress(raw[c][0], raw[c][1], None, cfg.T, cfg.F, cfg.rho, cfg.ratio_kind)
        np.testing.assert_array_equal(g_idx[c][:cfg.T], o_idx[0, :cfg.T])
        assert_selection_matches(g_idx[c][cfg.T:] - cfg.T, o_idx[0, cfg.T:] - cfg.T, o_scores[0], f"chunk {c}")
        if not np.array_equal(g_idx[c], o_idx[0]):     # differs inside the tie band only: follow the GPU's set
            sel = torch.as_tensor(g_idx[c], dtype=torch.long)
            o_K, o_V = raw[c][0][:, sel].contiguous(), raw[c][1][:, sel].contiguous()
        assert torch.equal(bits(store_k[c].cpu()), bits(o_K)) and torch.equal(bits(store_v[c].cpu()), bits(o_V))
        comp[c] = (o_K, o_V)
    # window assembly from the store, attention over the assembled window (no host sync between the calls)
    store = wk.Store([store_k[c] for c in range(cfg.M)], [store_v[c] for c in range(cfg.M)])
    Q = ws.make_queries(cfg, d)
    Kn, Vn = ws.make_native(cfg, d)
    cap = cfg.n_native + cfg.R * n_out
    Kw = torch.zeros((cfg.H, cap, cfg.d), dtype=dt, device=d)
    Vw = torch.zeros_like(Kw)
    n_win = torch.empty(1, dtype=torch.int32, device=d)
    wk.wk_gather_window(store.desc, ids, nf, cfg.R, Kn, Vn, cfg.n_native, Kw, Vw, cap, n_win)
    O = torch.empty_like(Q)
    lse = torch.empty(Q.shape[:2], dtype=torch.float32, device=d)
    wk.wk_attention(Q, Kw, Vw, O, lse, N_kv=cap, n_kv_dev=n_win)
    torch.cuda.synchronize()
    order = o_ids.tolist()
    oKw, oVw, o_n = oracle.gather([comp[c][0] for c in order], [comp[c][1] for c in order], np.arange(cfg.R),
                                  Kn.cpu(), Vn.cpu(), cap)
    assert int(n_win.item()) == o_n == cap
    assert torch.equal(bits(Kw.cpu()), bits(oKw)) and torch.equal(bits(Vw.cpu()), bits(oVw))   # window, byte for byte
    rows = sample_rows(cfg.N_q, 256, n_random, seed=cfg.index)
    ref, ref_lse = oracle.attention(Q.cpu(), oKw, oVw, N_kv=o_n, rows=rows, want_lse=True)
    sel = torch.as_tensor(rows, dtype=torch.long)
    return assert_attention_close_bf16(O[:, sel], ref, lse[:, sel], ref_lse, full_size=True), len(rows)


@pytest.mark.timeout(600)
def test_config1_whole_path():
    """Matrix-Game shape as defined: 60 chunks in an HBM store, R = 4, window of 10,560 keys."""
    cfg = ws.get_config(1)
    (mx, mean), n = _whole_path_full_store(cfg, n_random=256)
    print(f"config1 whole path: {n} rows/head, max-abs {mx:.2e} mean-abs {mean:.2e}")


@pytest.mark.timeout(900)
def test_config2_whole_path():
    """LingBot shape as defined: 120 chunks in pinned host memory (5.75 GB), R = 8, window of 28,080 keys."""
    cfg = ws.get_config(2)
    assert cfg.store == "pinned" and cfg.M == 120 and cfg.R == 8
    (mx, mean), n = _whole_path_full_store(cfg, n_random=256)
    print(f"config2 whole path: {n} rows/head, max-abs {mx:.2e} mean-abs {mean:.2e}")


def test_retrieving_nothing_is_sliding_window_attention():
    cfg = ws.get_config(1).with_(H=2, T=100, M=4)
    chunks = [ws.make_chunk(cfg, c) for c in range(cfg.M)]
    poses, cur = ws.make_poses(cfg.M, cfg.seed)
    Q, (Kn, Vn) = ws.make_queries(cfg), ws.make_native(cfg)
    g = _gpu_path(cfg, chunks, poses, cur, Q, Kn, Vn, R=0)
    assert g["n_win"] == cfg.n_native
    d = dev()
    O = torch.empty(Q.shape, dtype=Q.dtype, device=d)
    wk.wk_attention(Q.to(d), Kn.to(d), Vn.to(d), O)
    torch.cuda.synchronize()
    assert torch.equal(bits(O), bits(g["O"]))      # identical kernel, identical window: identical bits
    mx, mean = attention_errors(O, oracle.attention(Q, Kn, Vn))
    assert mx <= ATT_MAX_ABS_BF16 and mean <= ATT_MEAN_ABS_BF16


def test_retrieving_everything_uncompressed_is_full_kv_attention():
    cfg = ws.get_config(1).with_(H=2, T=100, M=5)
    chunks = [ws.make_chunk(cfg, c) for c in range(cfg.M)]
    poses, cur = ws.make_poses(cfg.M, cfg.seed)
    Q, (Kn, Vn) = ws.make_queries(cfg), ws.make_native(cfg)
    g = _gpu_path(cfg, chunks, poses, cur, Q, Kn, Vn, rho=1.0, R=cfg.M)
    assert g["n_win"] == cfg.n_native + cfg.M * cfg.chunk_tokens
    K_full = torch.cat([Kn] + [c[0] for c in chunks], 1)
    V_full = torch.cat([Vn] + [c[1] for c in chunks], 1)
    mx, mean = attention_errors(g["O"], oracle.attention(Q, K_full, V_full))
    assert mx <= ATT_MAX_ABS_BF16 and mean <= ATT_MEAN_ABS_BF16
    # the window holds exactly the history's rows (in retrieval order)
    assert sorted(map(tuple, g["Kw"][0].view(torch.int16)[:, :4].tolist())) == \
        sorted(map(tuple, K_full[0].view(torch.int16)[:, :4].tolist()))
