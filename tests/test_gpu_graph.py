"""The hot-path step (compress -> score -> gather -> attention) captured in a HIP graph: every replay,
with eager work and synchronisations in between and with new inputs written into the same buffers, gives
bit for bit what the eager calls give.  The library allocates nothing and clears nothing with memsets, so
its calls are capturable as they are."""
import numpy as np
import pytest
import torch

import paper_2605_22718_amd as wk
import wk_synth as ws
from wkt import bits, dev

pytestmark = pytest.mark.gpu


def test_step_captured_in_a_graph_replays_like_eager():
    d = dev()
    cfg = ws.get_config(1).with_(H=4, T=200, M=10, R=3)
    dt = ws.torch_dtype(cfg.dtype)
    n_out, _ = wk.wk_keep_count(cfg.rho, cfg.ratio_kind, cfg.anchor_mode, cfg.F, cfg.T)
    desc = wk.make_compress_desc(cfg.H, cfg.T, cfg.F, cfg.dtype, cfg.rho)
    wsb = torch.empty(wk.wk_compress_workspace_bytes(desc), dtype=torch.uint8, device=d)
    sk = torch.empty((cfg.M, cfg.H, n_out, cfg.d), dtype=dt, device=d)
    sv = torch.empty_like(sk)
    idx = torch.empty((1, n_out), dtype=torch.int32, device=d)
    for c in range(cfg.M):
        K, V, _ = ws.make_chunk(cfg, c, d)
        wk.wk_compress_chunk(desc, K, V, None, idx, sk[c], sv[c], wsb)
    store = wk.Store([sk[c] for c in range(cfg.M)], [sv[c] for c in range(cfg.M)], d)
    poses_np, cur = ws.make_poses(cfg.M, 3)
    poses = torch.from_numpy(poses_np).to(d)
    N_kv = cfg.n_native + cfg.R * n_out
    # static buffers the graph reads and writes
    evK = torch.empty((cfg.H, cfg.F * cfg.T, cfg.d), dtype=dt, device=d)
    evV = torch.empty_like(evK)
    evKo = torch.empty((cfg.H, n_out, cfg.d), dtype=dt, device=d)
    evVo = torch.empty_like(evKo)
    Q = torch.empty((cfg.H, cfg.N_q, cfg.d), dtype=dt, device=d)
    Kw = torch.zeros((cfg.H, N_kv, cfg.d), dtype=dt, device=d)
    Vw = torch.zeros_like(Kw)
    O = torch.empty_like(Q)
    lse = torch.empty((cfg.H, cfg.N_q), dtype=torch.float32, device=d)
    ids = torch.empty(cfg.R, dtype=torch.int32, device=d)
    nf = torch.empty(1, dtype=torch.int32, device=d)
    n_win = torch.empty(1, dtype=torch.int32, device=d)
    aws_n = wk.wk_attention_workspace_bytes(cfg.H, cfg.N_q, N_kv, cfg.dtype)
    aws = torch.empty(max(aws_n, 256), dtype=torch.uint8, device=d)

    def step():
        wk.wk_compress_chunk(desc, evK, evV, None, idx, evKo, evVo, wsb)
        wk.wk_score_chunks(poses, cfg.M, cur, wk.WK_NORM_MAX, cfg.R, ids, None, nf)
        wk.wk_gather_window(store.desc, ids, nf, cfg.R, None, None, cfg.n_native, Kw, Vw, N_kv, n_win)
        wk.wk_attention(Q, Kw, Vw, O, lse, N_kv=N_kv, n_kv_dev=n_win, workspace=aws if aws_n else None)

    def load_inputs(seed):
        K, V, _ = ws.make_chunk(cfg, 100 + seed, d)
        evK.copy_(K), evV.copy_(V)
        Q.copy_(ws.make_queries(cfg.with_(index=50 + seed), d))
        Kn, Vn = ws.make_native(cfg.with_(index=70 + seed), d)
        Kw[:, :cfg.n_native] = Kn
        Vw[:, :cfg.n_native] = Vn

    load_inputs(0)
    step()                                   # warm-up outside capture
    torch.cuda.synchronize()
    side = torch.cuda.Stream()               # default priority
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    for seed in range(1, 5):
        load_inputs(seed)
        O.fill_(float("nan")), evKo.fill_(float("nan")), lse.fill_(float("nan")), ids.fill_(-9)
        graph.replay()
        torch.cuda.synchronize()
        got = (O.clone(), lse.clone(), evKo.clone(), evVo.clone(), ids.clone(), idx.clone(), int(n_win.item()))
        # eager work between replays: the same step, on the default stream
        O.fill_(float("nan")), evKo.fill_(float("nan")), lse.fill_(float("nan")), ids.fill_(-9)
        step()
        torch.cuda.synchronize()
        assert got[6] == int(n_win.item()) == N_kv
        assert torch.equal(got[4], ids) and torch.equal(got[5], idx)
        assert torch.equal(bits(got[0]), bits(O)) and torch.equal(got[1], lse)
        assert torch.equal(bits(got[2]), bits(evKo)) and torch.equal(bits(got[3]), bits(evVo))
        assert torch.isfinite(O.float()).all()
