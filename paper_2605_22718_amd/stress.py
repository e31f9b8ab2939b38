"""Compression / retrieval stress measurement: the LingBot-shaped stress configuration (index 4 of
wk_synth.configs): a batch of 64 three-frame chunks (3.07 GB of K, as much of V) compressed in one
wk_compress_chunk call at P = 25 %, 50 % and 75 % (the settings 3 -> 1.5 / 2.0 / 2.5 of the paper's
ablation, Sec. 5.4, Tab. 2), with Eq. 5 evaluated in factored form and as the similarity GEMM on the matrix
cores; top-16 retrieval over 1,000 stored poses (Sec. 5.1); window assembly of 16 compressed chunks from a
store in pinned host memory (CPU offloading, Sec. 7; 1,000 logical chunk ids backed by 64 payloads).

    python -m paper_2605_22718_amd.stress [--reps 3]

prints one JSON object per measurement.  Runs on the GPU through the C-ABI entry points only; inputs are the
seeded synthetic chunks of wk_synth.
"""
import argparse
import json

import torch

import paper_2605_22718_amd as wk
import wk_synth as ws

BATCH = 64
PEAK_BF16_TFLOPS = 2500.0
PEAK_HBM_GBPS = 8000.0


def _time(fn, reps):
    fn()
    torch.cuda.synchronize()
    s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    s.record()
    for _ in range(reps):
        fn()
    e.record()
    torch.cuda.synchronize()
    return s.elapsed_time(e) / reps


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--reps", type=int, default=3)
    a = ap.parse_args()
    assert torch.cuda.is_available(), "stress.py needs a GPU"
    dev = torch.device("cuda:0")
    cfg = ws.get_config(4)
    row = cfg.d * 2
    K = torch.empty((BATCH, cfg.H, cfg.chunk_tokens, cfg.d), dtype=torch.bfloat16, device=dev)
    V = torch.empty_like(K)
    for c in range(BATCH):
        k, v, _ = ws.make_chunk(cfg, c, dev)
        K[c], V[c] = k, v
    for P in (0.25, 0.5, 0.75):
        n_out, _ = wk.wk_keep_count(P, wk.WK_RATIO_NONANCHOR, wk.WK_ANCHOR_FIRST_FRAME, cfg.F, cfg.T)
        for algo, name in ((wk.WK_SCORE_FACTORED, "factored"), (wk.WK_SCORE_GEMM, "gemm")):
            desc = wk.make_compress_desc(cfg.H, cfg.T, cfg.F, cfg.dtype, P, batch=BATCH,
                                         ratio_kind=wk.WK_RATIO_NONANCHOR, score_algo=algo)
            wsb = torch.empty(wk.wk_compress_workspace_bytes(desc), dtype=torch.uint8, device=dev)
            idx = torch.empty((BATCH, 1, n_out), dtype=torch.int32, device=dev)
            Ko = torch.empty((BATCH, cfg.H, n_out, cfg.d), dtype=torch.bfloat16, device=dev)
            Vo = torch.empty_like(Ko)
            t = _time(lambda: wk.wk_compress_chunk(desc, K, V, None, idx, Ko, Vo, wsb), a.reps)
            # algorithmic bytes: K read once, the kept rows of K and V read and written
            moved = BATCH * cfg.H * (cfg.chunk_tokens + 4 * n_out) * row
            out = {"call": "wk_compress_chunk", "batch": BATCH, "P": P, "scoring": name, "n_out": n_out, "ms": t,
                   "us_per_chunk": t / BATCH * 1e3, "algorithmic_GBps": moved / t / 1e6,
                   "frac_hbm_peak": moved / t / 1e6 / PEAK_HBM_GBPS}
            if algo == wk.WK_SCORE_GEMM:
                flop = 2.0 * (cfg.F - 1) * cfg.T * cfg.T * cfg.H * cfg.d * BATCH
                out["similarity_gemm_flop"] = flop
                out["similarity_gemm_tflops_over_whole_call"] = flop / t / 1e9
            print(json.dumps(out), flush=True)
            del Ko, Vo, idx, wsb
    poses_np, cur = ws.make_poses(cfg.M, cfg.seed)
    poses = torch.from_numpy(poses_np).to(dev)
    ids = torch.empty(cfg.R, dtype=torch.int32, device=dev)
    n_found = torch.empty(1, dtype=torch.int32, device=dev)
    t = _time(lambda: wk.wk_score_chunks(poses, cfg.M, cur, wk.WK_NORM_MAX, cfg.R, ids, None, n_found), 20)
    print(json.dumps({"call": "wk_score_chunks", "M": cfg.M, "R": cfg.R, "us": t * 1e3}), flush=True)
    n_out, _ = wk.wk_keep_count(0.25, wk.WK_RATIO_NONANCHOR, wk.WK_ANCHOR_FIRST_FRAME, cfg.F, cfg.T)
    pool_k = torch.zeros((BATCH, cfg.H, n_out, cfg.d), dtype=torch.bfloat16, pin_memory=True)
    pool_v = torch.zeros((BATCH, cfg.H, n_out, cfg.d), dtype=torch.bfloat16, pin_memory=True)
    store = wk.Store([pool_k[c % BATCH] for c in range(cfg.M)], [pool_v[c % BATCH] for c in range(cfg.M)])
    cap = cfg.R * n_out
    Kw = torch.zeros((cfg.H, cap, cfg.d), dtype=torch.bfloat16, device=dev)
    Vw = torch.zeros_like(Kw)
    n_win = torch.empty(1, dtype=torch.int32, device=dev)
    t = _time(lambda: wk.wk_gather_window(store.desc, ids, n_found, cfg.R, None, None, 0, Kw, Vw, cap, n_win), a.reps)
    print(json.dumps({"call": "wk_gather_window", "store": "pinned host", "chunks": cfg.R, "bytes": 2 * cfg.H * cap * row,
                      "ms": t, "GBps": 2 * cfg.H * cap * row / t / 1e6}), flush=True)


if __name__ == "__main__":
    main()
