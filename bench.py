#!/usr/bin/env python3
"""Benchmark of the WorldKV hot path on one MI355X.

A step = one pass of the whole path for one transformer layer and one denoising step on the
LingBot-World-Fast-shaped workload (40 heads, d = 128, 1,560 tokens/frame): compress one evicted
3-frame chunk (wk_compress_chunk), score the 120-chunk store and pick R = 8 (wk_score_chunks),
assemble the 28,080-key window (wk_gather_window) and attend 4,680 queries over it (wk_attention).
All inputs are seeded synthetic tensors already resident in HBM when the timed region starts.

Prints one JSON line.  `value` is attention FLOP per step (4*N_q*N_kv*d*H) divided by the time of
the whole step with the chunk store resident in HBM (`value_hbm_store` repeats it); the same step with the
store in pinned host memory, as the workload is defined, is timed too and reported as `value_pinned_store`
(host-link inclusive, therefore never `value`).  The attention kernel alone is in `roofline` (HIP events
around that kernel: mean, median and minimum over the timed steps).
"""
import argparse
import json
import sys
import time

import numpy as np
import torch

import paper_2605_22718_amd as wk
import wk_synth as ws

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
# HBM bytes per wk_attention launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (two runs), each
# scaled by what the counter reads for the plain calibration copy (0.500 and 1.000), per workload index;
# see profiles/hbm_traffic_lingbot_pmc.txt for the commands
MEASURED_ATTENTION_TRAFFIC = {2: (2 * 700460 + 46800) * 1024}
# shader-clock cycles one wk_attention launch on this workload takes (SQ_BUSY_CYCLES over the 32 shader engines in
# the counter runs of profiles/hbm_traffic_lingbot_pmc.txt): a property of the kernel and the workload, while the
# clock the chip holds under this load differs from box to box.  The clock reported beside the roofline is this
# count over the launch time measured here; the peak at that clock is 256 CUs x 4 SIMDs x 1,024 bf16 flop per cycle.
MEASURED_ATTENTION_CYCLES = {2: 3.848e6}
FLOP_PER_CLOCK = 256 * 4 * 1024


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=2, choices=[1, 2],
                    help="workload index: 2 = LingBot-shaped (the workload the metric is quoted on), "
                         "1 = Matrix-Game-shaped; the other configurations are parity-test cases")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-pinned", action="store_true", help="skip the pinned-host store measurement")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target CPU time of the oracle sample")
    return ap.parse_args()


def build_store(cfg, dev, n_out):
    """Fill the store by compressing M seeded chunks on the GPU (wk_compress_chunk)."""
    dt = ws.torch_dtype(cfg.dtype)
    desc = wk.make_compress_desc(cfg.H, cfg.T, cfg.F, cfg.dtype, cfg.rho, ratio_kind=cfg.ratio_kind,
                                 anchor_mode=cfg.anchor_mode, head_mode=cfg.head_mode)
    wsb = torch.empty(wk.wk_compress_workspace_bytes(desc), dtype=torch.uint8, device=dev)
    store_k = torch.empty((cfg.M, cfg.H, n_out, cfg.d), dtype=dt, device=dev)
    store_v = torch.empty_like(store_k)
    for c in range(cfg.M):
        K, V, A = ws.make_chunk(cfg, c, dev)
        wk.wk_compress_chunk(desc, K, V, A, None, store_k[c], store_v[c], wsb)
    torch.cuda.synchronize()
    return desc, wsb, store_k, store_v


def cpu_baseline(cfg, Q, Kw, Vw, N_kv, raw_chunk, store_chunks, ids, Kn, Vn, poses, cur, n_out, target_s):
    """Time the fp64 oracle (as written, never tuned) on a bounded sample of the same step: attention on a
    sample of query rows (all heads, whole window; extrapolated by rows), the other three calls in full.
    All-core times make `value`; the attention sample is also timed on one thread."""
    import oracle

    H, N_q = cfg.H, cfg.N_q
    Qc, Kc, Vc = Q.cpu(), Kw.cpu(), Vw.cpu()
    rng = np.random.default_rng(0)
    rows = np.sort(rng.choice(N_q, 4, replace=False)).astype(np.int32)
    t0 = time.perf_counter()
    oracle.attention(Qc, Kc, Vc, N_kv=N_kv, rows=rows)
    t_probe = time.perf_counter() - t0
    n_rows = int(max(4, min(N_q, 0.5 * target_s / (t_probe / 4))))
    rows = np.sort(rng.choice(N_q, n_rows, replace=False)).astype(np.int32)
    t0 = time.perf_counter()
    oracle.attention(Qc, Kc, Vc, N_kv=N_kv, rows=rows)
    t_att = time.perf_counter() - t0
    att_full = t_att * N_q / n_rows
    # one thread: a sixteenth of the rows
    threads = oracle.n_threads()
    rows1 = rows[:: 16][: max(1, n_rows // 16)]
    oracle.set_threads(1)
    t0 = time.perf_counter()
    oracle.attention(Qc, Kc, Vc, N_kv=N_kv, rows=rows1)
    att_full_1 = (time.perf_counter() - t0) * N_q / rows1.size
    oracle.set_threads(threads)
    # compress: the whole evicted chunk (Eq. 5 double loop, selection, compaction)
    Kr, Vr = raw_chunk[0].cpu(), raw_chunk[1].cpu()
    Ar = None if raw_chunk[2] is None else raw_chunk[2].cpu()
    t0 = time.perf_counter()
    oracle.compress(Kr, Vr, Ar, cfg.T, cfg.F, cfg.rho, cfg.ratio_kind, cfg.head_mode, cfg.anchor_mode)
    t_c = time.perf_counter() - t0
    t0 = time.perf_counter()
    oracle.score_chunks(poses, cur, cfg.R)
    t_s = time.perf_counter() - t0
    # gather: the oracle's window assembly from the retrieved chunks of the store, in full
    ck = [store_chunks[0][c].cpu() for c in ids]
    cv = [store_chunks[1][c].cpu() for c in ids]
    Knc, Vnc = Kn.cpu(), Vn.cpu()
    t0 = time.perf_counter()
    oracle.gather(ck, cv, np.arange(len(ids), dtype=np.int32), Knc, Vnc, N_kv)
    t_g = time.perf_counter() - t0
    step = att_full + t_c + t_s + t_g
    flops = 4.0 * N_q * N_kv * cfg.d * H
    return {
        "value": flops / step / 1e12, "unit": "TFLOP/s", "cores": threads, "kind": "oracle",
        "sample": f"fp64 oracle: attention on {n_rows} of {N_q} query rows x {H} heads over the whole window "
                  f"(extrapolated by rows); compression of one chunk, retrieval and window assembly in full",
        "attention_only_tflops": flops / att_full / 1e12,
        "attention_only_tflops_one_thread": flops / att_full_1 / 1e12,
        "ms": {"attention_extrapolated": att_full * 1e3, "attention_extrapolated_one_thread": att_full_1 * 1e3,
               "compress": t_c * 1e3, "score": t_s * 1e3, "gather": t_g * 1e3},
    }


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (the path shards by heads with no exchange "
              "between GPUs); --gpus must be 1", file=sys.stderr)
        sys.exit(2)
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    cfg = ws.get_config(a.config)
    dt = ws.torch_dtype(cfg.dtype)
    n_out, _ = wk.wk_keep_count(cfg.rho, cfg.ratio_kind, cfg.anchor_mode, cfg.F, cfg.T)
    N_kv = cfg.n_native + cfg.R * n_out

    desc, wsb, store_k, store_v = build_store(cfg, dev, n_out)
    store = wk.Store([store_k[c] for c in range(cfg.M)], [store_v[c] for c in range(cfg.M)])
    poses_np, cur = ws.make_poses(cfg.M, cfg.seed)
    poses = torch.from_numpy(poses_np).to(dev)
    Q = ws.make_queries(cfg, dev)
    Kn, Vn = ws.make_native(cfg, dev)
    evicted = ws.make_chunk(cfg, cfg.M, dev)          # the chunk leaving the window in this step
    ev_k = torch.empty((cfg.H, n_out, cfg.d), dtype=dt, device=dev)
    ev_v = torch.empty_like(ev_k)
    ev_idx = torch.empty((1, n_out), dtype=torch.int32, device=dev)
    ids = torch.empty(cfg.R, dtype=torch.int32, device=dev)
    dist = torch.empty(cfg.R, dtype=torch.float64, device=dev)
    n_found = torch.empty(1, dtype=torch.int32, device=dev)
    Kw = torch.zeros((cfg.H, N_kv, cfg.d), dtype=dt, device=dev)
    Vw = torch.zeros_like(Kw)
    Kw[:, :cfg.n_native] = Kn
    Vw[:, :cfg.n_native] = Vn
    n_win = torch.empty(1, dtype=torch.int32, device=dev)
    O = torch.empty_like(Q)
    att_ws_bytes = wk.wk_attention_workspace_bytes(cfg.H, cfg.N_q, N_kv, cfg.dtype)   # 0 for the LingBot shape
    att_ws = torch.empty(att_ws_bytes, dtype=torch.uint8, device=dev) if att_ws_bytes else None

    def step(store_desc, ev_att=None):
        wk.wk_compress_chunk(desc, evicted[0], evicted[1], evicted[2], ev_idx, ev_k, ev_v, wsb)
        wk.wk_score_chunks(poses, cfg.M, cur, wk.WK_NORM_MAX, cfg.R, ids, dist, n_found)
        # the native sliding-window rows already live at the head of the window buffer (K_native = NULL):
        # only the retrieved chunks move
        wk.wk_gather_window(store_desc, ids, n_found, cfg.R, None, None, cfg.n_native, Kw, Vw, N_kv, n_win)
        if ev_att:
            ev_att[0].record()
        wk.wk_attention(Q, Kw, Vw, O, None, N_kv=N_kv, n_kv_dev=n_win, workspace=att_ws)
        if ev_att:
            ev_att[1].record()

    for _ in range(a.warmup):
        step(store.desc)
    torch.cuda.synchronize()
    assert int(n_win.item()) == N_kv and int(n_found.item()) == cfg.R

    def ev():
        return torch.cuda.Event(enable_timing=True)

    def timed_steps(store_desc):
        """EXACTLY a.steps steps between two synchronisations; HIP events around every step and around
        the attention call inside it (on the launch stream)."""
        att_ev = [(ev(), ev()) for _ in range(a.steps)]
        step_ev = [(ev(), ev()) for _ in range(a.steps)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(a.steps):
            step_ev[i][0].record()
            step(store_desc, att_ev[i])
            step_ev[i][1].record()
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) / a.steps * 1e3
        return wall_ms, [s.elapsed_time(e) for s, e in att_ev], [s.elapsed_time(e) for s, e in step_ev]

    def stats(xs):
        return {"mean": float(np.mean(xs)), "median": float(np.median(xs)), "min": float(np.min(xs))}

    ms_step, att_list, step_list = timed_steps(store.desc)
    att_ms = float(np.mean(att_list))
    flops = 4.0 * cfg.N_q * N_kv * cfg.d * cfg.H
    att_tflops = flops / (att_ms * 1e-3) / 1e12

    # the same step captured once in a HIP graph and replayed (no per-call host work)
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step(store.desc)
    graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(a.steps):
        graph.replay()
    torch.cuda.synchronize()
    ms_step_graph = (time.perf_counter() - t0) / a.steps * 1e3
    assert int(n_win.item()) == N_kv

    # per-call times (each call alone on the stream, HIP events, mean of `steps` repetitions)
    def time_call(fn, reps):
        fn()
        torch.cuda.synchronize()
        s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        s.record()
        for _ in range(reps):
            fn()
        e.record()
        torch.cuda.synchronize()
        return s.elapsed_time(e) / reps

    reps = max(3, a.steps)
    per_call = {
        "compress": time_call(lambda: wk.wk_compress_chunk(desc, evicted[0], evicted[1], evicted[2], ev_idx, ev_k,
                                                           ev_v, wsb), reps),
        "score": time_call(lambda: wk.wk_score_chunks(poses, cfg.M, cur, wk.WK_NORM_MAX, cfg.R, ids, dist, n_found),
                           reps),
        "gather_hbm": time_call(lambda: wk.wk_gather_window(store.desc, ids, n_found, cfg.R, None, None, cfg.n_native,
                                                            Kw, Vw, N_kv, n_win), reps),
        "gather_hbm_with_native_copy": time_call(lambda: wk.wk_gather_window(store.desc, ids, n_found, cfg.R, Kn, Vn,
                                                                             cfg.n_native, Kw, Vw, N_kv, n_win), reps),
        "attention": att_ms,
    }
    if cfg.dtype == ws.configs.DT_BF16:
        # Eq. 5 as a similarity GEMM on the matrix cores (same result; reported against the MFMA peak)
        gdesc = wk.make_compress_desc(cfg.H, cfg.T, cfg.F, cfg.dtype, cfg.rho, ratio_kind=cfg.ratio_kind,
                                      anchor_mode=cfg.anchor_mode, head_mode=cfg.head_mode,
                                      score_algo=wk.WK_SCORE_GEMM)
        gws = torch.empty(wk.wk_compress_workspace_bytes(gdesc), dtype=torch.uint8, device=dev)
        per_call["compress_gemm_scoring"] = time_call(
            lambda: wk.wk_compress_chunk(gdesc, evicted[0], evicted[1], evicted[2], ev_idx, ev_k, ev_v, gws), reps)
    row_bytes = cfg.d * Q.element_size()
    gather_bytes = 2 * 2 * cfg.H * cfg.R * n_out * row_bytes   # retrieved rows of K and V, read + write
    # ceilings for the gather: a plain device-to-device copy of the same bytes (HBM store) ...
    flat = Kw.view(-1)[: (gather_bytes // 2) // Kw.element_size()]
    dst = torch.empty_like(flat)
    t_d2d = time_call(lambda: dst.copy_(flat), reps)
    del dst
    # a plain copy of a window-sized buffer that is cold in the caches: the copy of known size against which
    # the rocprofv3 FETCH_SIZE / WRITE_SIZE readings of the library's kernels are calibrated (k_copy_plain)
    cal_src = Kw.clone()
    cal_dst = torch.zeros_like(Kw)          # written after cal_src: pushes it out of the Infinity Cache
    wk.wk_calibration_copy(cal_dst, cal_src)
    del cal_src, cal_dst
    # context for the attention roofline: what the vendor library's dense bf16 GEMM reaches on this machine, on N(0,1)
    # operands like the window's (the chip is power-limited under dense matrix work, so no kernel holds the
    # nameplate peak; this is a measured reference, not the roofline's `peak`)
    gemm_tflops = None
    if cfg.dtype == ws.configs.DT_BF16:
        n_g = 8192
        ga = torch.randn(n_g, n_g, device=dev, dtype=torch.bfloat16)
        gb = torch.randn(n_g, n_g, device=dev, dtype=torch.bfloat16)
        gc = torch.empty(n_g, n_g, device=dev, dtype=torch.bfloat16)
        gemm_tflops = {   # B given row-major (k x n) / as the transpose of a row-major n x k matrix
            "b_row_major": 2.0 * n_g ** 3 / (time_call(lambda: torch.matmul(ga, gb, out=gc), reps) * 1e-3) / 1e12,
            "b_transposed": 2.0 * n_g ** 3 / (time_call(lambda: torch.matmul(ga, gb.t(), out=gc), reps) * 1e-3) / 1e12,
        }
        del ga, gb, gc
    extra = {
        "library_gemm_bf16_8192_tflops": gemm_tflops,
        "d2d_copy_ceiling_GBps": 2 * flat.numel() * flat.element_size() / (t_d2d * 1e-3) / 1e9,
        "attention_tflops": att_tflops,
        "pct_bf16_mfma_peak": 100.0 * att_tflops / PEAK_BF16_TFLOPS,
        "ms_per_chunk": per_call,
        "ms_per_step_graph_replay": ms_step_graph,
        "gather_hbm_GBps": gather_bytes / (per_call["gather_hbm"] * 1e-3) / 1e9,
    }

    if cfg.dtype == ws.configs.DT_BF16:
        # the HBM-resident store attended in place (no window copy): gather + attention as one call
        O2 = torch.empty_like(O)
        wk.wk_attention_in_place(Q, Kw, Vw, cfg.n_native, store.desc, ids, n_found, cfg.R, O2)
        torch.cuda.synchronize()
        assert (O2.float() - O.float()).abs().max().item() <= 4e-3      # same window, key tiles cut per chunk
        # both sides timed the same way (back-to-back repetitions run hotter than the step loop's attention)
        def gather_then_attend():
            wk.wk_gather_window(store.desc, ids, n_found, cfg.R, None, None, cfg.n_native, Kw, Vw, N_kv, n_win)
            wk.wk_attention(Q, Kw, Vw, O, None, N_kv=N_kv, n_kv_dev=n_win, workspace=att_ws)
        t_two = time_call(gather_then_attend, reps)
        t_ip = time_call(lambda: wk.wk_attention_in_place(Q, Kw, Vw, cfg.n_native, store.desc, ids, n_found, cfg.R,
                                                          O2), reps)
        extra["attention_in_place"] = {
            "ms": t_ip, "ms_gather_plus_attention": t_two,
            "note": "not part of `value`: the timed step assembles the window with wk_gather_window"}
        del O2

    if cfg.q_frames > 1 and N_kv >= 2 * cfg.N_q:
        # option: frame-level causal mask inside the denoising chunk, placed behind a sink chunk of the same
        # size (the window manager's layout); same window, so the flop count is that of the unmasked call
        # minus the hidden later frames
        bc_ws = torch.empty(wk.wk_attention_block_causal_workspace_bytes(cfg.H, cfg.N_q), dtype=torch.uint8,
                            device=dev)
        t_bc = time_call(lambda: wk.wk_attention_block_causal(Q, Kw, Vw, O, cfg.N_q, cfg.T, bc_ws, N_kv=N_kv,
                                                              n_kv_dev=n_win), 3)
        hidden = sum(cfg.q_frames - 1 - f for f in range(cfg.q_frames)) * cfg.T * cfg.T
        bc_flops = flops - 4.0 * hidden * cfg.d * cfg.H
        extra["attention_block_causal"] = {"ms": t_bc, "tflops": bc_flops / (t_bc * 1e-3) / 1e12,
                                           "launches": 2}
        del bc_ws

    if cfg.M > 0 and cfg.M <= wk.WK_QUERY_MAX_CHUNKS:
        # query-based retrieval (Sec. 4.2, App. C) in place of the pose distance: attention mass of the
        # current queries on every stored chunk, over a device-resident index of the chunks' anchor keys
        index_k = store_k[:, :, :cfg.T].contiguous()
        index = wk.Store([index_k[c] for c in range(cfg.M)], [index_k[c] for c in range(cfg.M)])
        n_rows = cfg.H * cfg.N_q
        lse_c = torch.empty((cfg.M, n_rows), dtype=torch.float32, device=dev)
        q_ids = torch.empty(cfg.R, dtype=torch.int32, device=dev)
        q_nf = torch.empty(1, dtype=torch.int32, device=dev)
        q_ws = torch.empty(wk.wk_score_chunks_query_workspace_bytes(cfg.M, n_rows), dtype=torch.uint8, device=dev)
        t_lse = time_call(lambda: wk.wk_chunk_lse(index.desc, Q, lse_c), 3)
        t_top = time_call(lambda: wk.wk_score_chunks_query(lse_c, cfg.M, n_rows, cfg.R, q_ids, None, q_nf, q_ws), 3)
        q_flops = 2.0 * cfg.N_q * cfg.T * cfg.d * cfg.H * cfg.M
        extra["query_retrieval"] = {
            "index": f"anchor keys of all {cfg.M} chunks ({cfg.T} per chunk), HBM-resident",
            "ms_chunk_lse": t_lse, "ms_score_chunks_query": t_top,
            "chunk_lse_tflops": q_flops / (t_lse * 1e-3) / 1e12,
            "chunk_lse_frac_bf16_mfma_peak": q_flops / (t_lse * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
        }
        del index, index_k, lse_c

    if not a.no_pinned and cfg.store == "pinned":
        # the CPU-offloaded store of the workload definition: same chunks in pinned host memory
        pk = torch.empty(store_k.shape, dtype=dt, pin_memory=True)
        pv = torch.empty(store_v.shape, dtype=dt, pin_memory=True)
        pk.copy_(store_k)
        pv.copy_(store_v)
        torch.cuda.synchronize()
        pstore = wk.Store([pk[c] for c in range(cfg.M)], [pv[c] for c in range(cfg.M)])
        t_pin = time_call(lambda: wk.wk_gather_window(pstore.desc, ids, n_found, cfg.R, None, None, cfg.n_native,
                                                      Kw, Vw, N_kv, n_win), 3)
        link_bytes = 2 * cfg.H * cfg.R * n_out * row_bytes
        # ... and a plain pinned-host to device copy of as many bytes (pinned store)
        n_link = link_bytes // pk.element_size()
        dst = torch.empty(n_link, dtype=dt, device=dev)
        t_h2d = time_call(lambda: dst.copy_(pk.view(-1)[:n_link], non_blocking=True), 3)
        extra["h2d_copy_ceiling_GBps"] = link_bytes / (t_h2d * 1e-3) / 1e9
        del dst
        extra["ms_per_chunk"]["gather_pinned_host"] = t_pin
        extra["gather_pinned_host_GBps"] = link_bytes / (t_pin * 1e-3) / 1e9
        # the whole step as the workload defines it: the store in pinned host memory, every retrieved chunk
        # crossing the host link in every step
        for _ in range(2):
            step(pstore.desc)
        ms_step_pinned, _, step_list_pinned = timed_steps(pstore.desc)
        extra["ms_per_step_pinned_store"] = ms_step_pinned
        extra["value_pinned_store"] = flops / (ms_step_pinned * 1e-3) / 1e12
        extra["step_ms_pinned_store_hip_events"] = stats(step_list_pinned)
        # in-place refresh of the retrieved slots (Sec. 4.2 window regions): only chunks that are not resident
        # yet cross the host link.  Two id sets differing in k chunks are requested in turn.
        slot_ids = torch.full((cfg.R,), -1, dtype=torch.int32, device=dev)
        n_fetched = torch.zeros(1, dtype=torch.int32, device=dev)
        u_ws = torch.empty(wk.wk_window_update_workspace_bytes(cfg.R), dtype=torch.uint8, device=dev)
        base_ids = ids.clone()
        refresh = {}
        for k in (0, 1, 2, cfg.R):
            other = base_ids.clone()
            spare = [c for c in range(cfg.M) if c not in set(base_ids.tolist())][:k]
            other[:k] = torch.tensor(spare, dtype=torch.int32, device=dev)
            sets = [base_ids, other]
            wk.wk_window_update(pstore.desc, base_ids, n_found, cfg.R, n_out, slot_ids, cfg.n_native, Kw, Vw, N_kv,
                                n_win, n_fetched, u_ws)
            torch.cuda.synchronize()
            ts = []
            for rep in range(4):
                s_ev, e_ev = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                s_ev.record()
                wk.wk_window_update(pstore.desc, sets[(rep + 1) % 2], n_found, cfg.R, n_out, slot_ids, cfg.n_native,
                                    Kw, Vw, N_kv, n_win, n_fetched, u_ws)
                e_ev.record()
                torch.cuda.synchronize()
                assert int(n_fetched.item()) == k
                ts.append(s_ev.elapsed_time(e_ev))
            refresh[f"{k}_of_{cfg.R}_chunks_change"] = float(np.median(ts))
        extra["window_update_pinned_host_ms"] = refresh
        # the pinned-store step with the retrieved region refreshed in place: compress + score + window update
        # + attention, with 1 of the R retrieved chunks changing from step to step (a smooth camera path)
        other = base_ids.clone()
        other[:1] = torch.tensor([c for c in range(cfg.M) if c not in set(base_ids.tolist())][:1],
                                 dtype=torch.int32, device=dev)
        sets = [base_ids, other]

        def step_update(i):
            wk.wk_compress_chunk(desc, evicted[0], evicted[1], evicted[2], ev_idx, ev_k, ev_v, wsb)
            wk.wk_score_chunks(poses, cfg.M, cur, wk.WK_NORM_MAX, cfg.R, ids, dist, n_found)
            wk.wk_window_update(pstore.desc, sets[i % 2], n_found, cfg.R, n_out, slot_ids, cfg.n_native, Kw, Vw, N_kv,
                                n_win, n_fetched, u_ws)
            wk.wk_attention(Q, Kw, Vw, O, None, N_kv=N_kv, n_kv_dev=n_win, workspace=att_ws)
        for i in range(2):
            step_update(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(a.steps):
            step_update(i)
        torch.cuda.synchronize()
        ms_upd = (time.perf_counter() - t0) / a.steps * 1e3
        extra["pinned_store_step_with_window_update"] = {
            "ms_per_step": ms_upd, "value": flops / (ms_upd * 1e-3) / 1e12, "chunks_changing_per_step": 1,
            "note": "wk_window_update in place of wk_gather_window: resident chunks stay, 1 of the "
                    f"{cfg.R} retrieved chunks is fetched over the host link per step"}
        wk.wk_score_chunks(poses, cfg.M, cur, wk.WK_NORM_MAX, cfg.R, ids, dist, n_found)
        # offload overlap (Sec. 7): a loop over layers (each a gather from the pinned store + attention),
        # on one stream vs with the next layer's gather on the prefetch stream into a second window buffer
        n_layers, cap_wg = 6, 64
        Kw2, Vw2 = Kw.clone(), Vw.clone()
        n_win2 = torch.empty(1, dtype=torch.int32, device=dev)
        wins = [(Kw, Vw, n_win), (Kw2, Vw2, n_win2)]

        def layers_sequential():
            for l in range(n_layers):
                kw, vw, nw = wins[l % 2]
                wk.wk_gather_window(pstore.desc, ids, n_found, cfg.R, None, None, cfg.n_native, kw, vw, N_kv, nw)
                wk.wk_attention(Q, kw, vw, O, None, N_kv=N_kv, n_kv_dev=nw, workspace=att_ws)

        pf = wk.wk_prefetch_create(2)

        def layers_overlapped():
            wk.wk_prefetch_after(pf)
            wk.wk_prefetch_gather(pf, 0, pstore.desc, ids, n_found, cfg.R, None, None, cfg.n_native, Kw, Vw, N_kv,
                                  n_win, cap_wg)
            for l in range(n_layers):
                s = l % 2
                if l + 1 < n_layers:
                    kw, vw, nw = wins[1 - s]
                    wk.wk_prefetch_gather(pf, 1 - s, pstore.desc, ids, n_found, cfg.R, None, None, cfg.n_native,
                                          kw, vw, N_kv, nw, cap_wg)
                wk.wk_prefetch_acquire(pf, s)
                kw, vw, nw = wins[s]
                wk.wk_attention(Q, kw, vw, O, None, N_kv=N_kv, n_kv_dev=nw, workspace=att_ws)
                wk.wk_prefetch_release(pf, s)

        def wall(fn, reps=2):
            fn()
            torch.cuda.synchronize()
            t = time.perf_counter()
            for _ in range(reps):
                fn()
            torch.cuda.synchronize()
            return (time.perf_counter() - t) / reps * 1e3

        t_seq = wall(layers_sequential) / n_layers
        t_ovl = wall(layers_overlapped) / n_layers
        wk.wk_prefetch_destroy(pf)
        extra["offload_overlap"] = {
            "layers": n_layers, "gather_max_workgroups": cap_wg,
            "ms_per_layer_one_stream": t_seq, "ms_per_layer_prefetch_stream": t_ovl,
            "ms_gather_alone": t_pin, "ms_attention_alone": att_ms,
            "note": "pinned-host store; per layer: gather of the retrieved chunks + attention; the overlapped "
                    "loop includes its one unhidden first gather",
        }
        del Kw2, Vw2
        # restore the window for the oracle sample below
        wk.wk_gather_window(store.desc, ids, n_found, cfg.R, None, None, cfg.n_native, Kw, Vw, N_kv, n_win)
        torch.cuda.synchronize()
        del pstore, pk, pv

    cycles = MEASURED_ATTENTION_CYCLES.get(cfg.index)
    clk = cycles / (att_ms * 1e-3) / 1e9 if cycles else None
    value = flops / (ms_step * 1e-3) / 1e12
    out = {
        "metric": "attention TFLOP/s of the whole hot-path step (4*N_q*N_kv*d*H flop of wk_attention over the time "
                  "of compress + score + gather + attend)",
        "value": value,
        "unit": "TFLOP/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg.dtype == ws.configs.DT_BF16 else "f32", "data": "synthetic",
        "config": {"workload": f"config {cfg.index} ({cfg.name}): H={cfg.H} d={cfg.d} N_q={cfg.N_q} "
                               f"N_kv={N_kv} (native {cfg.n_native} + R={cfg.R} x {n_out}), store M={cfg.M}, "
                               f"rho={cfg.rho}, one layer, one denoising step",
                   "store": "`value` and `ms_per_step`: chunk store resident in HBM (inputs in HBM when the timed "
                            "region starts); the same step over the store in pinned host memory, which is how the "
                            "workload defines the store, is `value_pinned_store` / `ms_per_step_pinned_store` "
                            "(host-link inclusive)"},
        "value_hbm_store": value,
        "step_ms_hip_events": stats(step_list),
        "roofline": {"bound": "mfma", "achieved": att_tflops, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": att_tflops / PEAK_BF16_TFLOPS,
                     "traffic": MEASURED_ATTENTION_TRAFFIC.get(cfg.index),
                     "kernel": "k_attn_bf16", "ms": att_ms, "ms_median": float(np.median(att_list)),
                     "ms_min": float(np.min(att_list)), "flop": flops,
                     "frac_best_launch": flops / (float(np.min(att_list)) * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
                     "clock_GHz_under_load": clk,
                     "frac_of_peak_at_that_clock": (att_tflops * 1e12 / (FLOP_PER_CLOCK * clk * 1e9)) if clk else None},
        **extra,
    }
    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, Q, Kw, Vw, N_kv, evicted, (store_k, store_v), ids.cpu().tolist(), Kn, Vn,
                                           poses_np, cur, n_out, a.cpu_seconds)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
