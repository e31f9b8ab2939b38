"""Compression-ratio / retrieval-budget sweep of the hot path (the settings of the paper's ablation,
Sec. 5.4, Tab. 2): a 3-frame chunk is stored as r frame-equivalents, r in {1.0, 1.25, 1.5, 2.0, 2.5, 3.0}
(anchor only ... no pruning), and the 9-frame retrieved region then holds floor(9 / r) chunks -- which
contains the three inter-chunk rows (3 -> 3: r = 3.0, 6 -> 3: r = 1.5, 9 -> 3: r = 1.0).

The paper's table reports image quality, which needs the trained world models.  What can be measured
on synthetic K/V of the same shape is the cost side and the chunk-level attention map (Fig. 3): per
setting the time of each call, the window length, the bytes a chunk occupies in the store, and the
share of the queries' attention mass that lands on the native rows and on each retrieved chunk.

    python -m paper_2605_22718_amd.sweep [--config 2] [--store 12]

prints one JSON object per setting.  Runs on the GPU through the C-ABI entry points only.
"""
import argparse
import json

import numpy as np
import torch

import paper_2605_22718_amd as wk
import wk_synth as ws

RETRIEVED_FRAMES = 9
SETTINGS = (1.0, 1.25, 1.5, 2.0, 2.5, 3.0)


def _time(fn, reps=5):
    fn()
    torch.cuda.synchronize()
    s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    s.record()
    for _ in range(reps):
        fn()
    e.record()
    torch.cuda.synchronize()
    return s.elapsed_time(e) / reps


def run_setting(cfg, r, n_store, dev):
    dt = ws.torch_dtype(cfg.dtype)
    P = (r - 1.0) / (cfg.F - 1)                        # kept fraction of the non-anchor tokens
    n_out, n_keep = wk.wk_keep_count(P, wk.WK_RATIO_NONANCHOR, wk.WK_ANCHOR_FIRST_FRAME, cfg.F, cfg.T)
    R = min(int(RETRIEVED_FRAMES / r), n_store)
    desc = wk.make_compress_desc(cfg.H, cfg.T, cfg.F, cfg.dtype, P, ratio_kind=wk.WK_RATIO_NONANCHOR,
                                 anchor_mode=wk.WK_ANCHOR_FIRST_FRAME)
    wsb = torch.empty(wk.wk_compress_workspace_bytes(desc), dtype=torch.uint8, device=dev)
    sk = torch.empty((n_store, cfg.H, n_out, cfg.d), dtype=dt, device=dev)
    sv = torch.empty_like(sk)
    idx = torch.empty((1, n_out), dtype=torch.int32, device=dev)
    t_comp = []
    for c in range(n_store):
        K, V, _ = ws.make_chunk(cfg, c, dev)
        t_comp.append(_time(lambda: wk.wk_compress_chunk(desc, K, V, None, idx, sk[c], sv[c], wsb), 3))
    store = wk.Store([sk[c] for c in range(n_store)], [sv[c] for c in range(n_store)], dev)
    poses, cur = ws.make_poses(n_store, cfg.seed)
    poses = torch.from_numpy(poses).to(dev)
    ids = torch.empty(R, dtype=torch.int32, device=dev)
    nf = torch.empty(1, dtype=torch.int32, device=dev)
    Q = ws.make_queries(cfg, dev)
    Kn, Vn = ws.make_native(cfg, dev)
    N_kv = cfg.n_native + R * n_out
    Kw = torch.zeros((cfg.H, N_kv, cfg.d), dtype=dt, device=dev)
    Vw = torch.zeros_like(Kw)
    Kw[:, :cfg.n_native] = Kn
    Vw[:, :cfg.n_native] = Vn
    n_win = torch.empty(1, dtype=torch.int32, device=dev)
    O = torch.empty_like(Q)
    aws_n = wk.wk_attention_workspace_bytes(cfg.H, cfg.N_q, N_kv, cfg.dtype)
    aws = torch.empty(aws_n, dtype=torch.uint8, device=dev) if aws_n else None
    t_score = _time(lambda: wk.wk_score_chunks(poses, n_store, cur, wk.WK_NORM_MAX, R, ids, None, nf))
    t_gather = _time(lambda: wk.wk_gather_window(store.desc, ids, nf, R, None, None, cfg.n_native, Kw, Vw, N_kv,
                                                 n_win))
    t_att = _time(lambda: wk.wk_attention(Q, Kw, Vw, O, None, N_kv=N_kv, n_kv_dev=n_win, workspace=aws))
    # chunk-level attention map: mass on the native rows and on each retrieved chunk
    got = ids.cpu().tolist()
    parts = wk.Store([Kn] + [sk[c] for c in got], [Kn] + [sk[c] for c in got], dev)
    n_rows = cfg.H * cfg.N_q
    lse = torch.empty((1 + R, n_rows), dtype=torch.float32, device=dev)
    top = torch.empty(1 + R, dtype=torch.int32, device=dev)
    qws = torch.empty(wk.wk_score_chunks_query_workspace_bytes(1 + R, n_rows), dtype=torch.uint8, device=dev)
    wk.wk_chunk_lse(parts.desc, Q, lse)
    wk.wk_score_chunks_query(lse, 1 + R, n_rows, 1 + R, top, None, nf, qws)
    torch.cuda.synchronize()
    mass = qws[: 8 * (1 + R)].view(torch.float64).cpu().numpy()
    flops = 4.0 * cfg.N_q * N_kv * cfg.d * cfg.H
    return {
        "setting": f"3->{r:g}", "retrieved_chunks": R, "kept_fraction_of_non_anchor": P, "stored_tokens": n_out,
        "store_MB_per_chunk_per_layer": 2 * cfg.H * n_out * cfg.d * Q.element_size() / 1e6,
        "N_kv": N_kv, "ms_compress": float(np.median(t_comp)), "ms_score": t_score, "ms_gather": t_gather,
        "ms_attention": t_att, "attention_tflops": flops / (t_att * 1e-3) / 1e12,
        "retrieved_ids": got, "mass_native": float(mass[0]), "mass_per_retrieved_chunk": [float(x) for x in mass[1:]],
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, default=2)
    ap.add_argument("--store", type=int, default=12, help="chunks in the synthetic store (>= 9)")
    a = ap.parse_args()
    assert torch.cuda.is_available(), "the sweep needs a GPU"
    dev = torch.device("cuda:0")
    cfg = ws.get_config(a.config)
    for r in SETTINGS:
        print(json.dumps(run_setting(cfg, r, a.store, dev)), flush=True)


if __name__ == "__main__":
    main()
