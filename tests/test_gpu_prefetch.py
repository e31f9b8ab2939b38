"""Overlapped window assembly (Sec. 7: CPU-offloaded store): a loop over layers whose gathers run on the
prefetch stream into alternating window buffers while the previous layer attends must give, layer by
layer, the oracle's window bytes and attention output -- the same as the plain one-stream sequence."""
import numpy as np
import pytest
import torch

import oracle
import paper_2605_22718_amd as wk
import wk_synth as ws
from wkt import ATT_MAX_ABS_BF16, ATT_MEAN_ABS_BF16, attention_errors, bits, dev

pytestmark = pytest.mark.gpu


def _layers(cfg, L, lens, n_native, N_q):
    """Per layer: a pinned-host store of ragged chunks, native rows, queries (all distinct)."""
    out = []
    for l in range(L):
        ks, vs = [], []
        for c, n in enumerate(lens):
            k, v = ws.make_native(cfg.with_(index=100 + 10 * l + c), n_rows=n)
            ks.append(k), vs.append(v)
        Kn, Vn = ws.make_native(cfg.with_(index=200 + l), n_rows=n_native)
        Q = ws.make_queries(cfg.with_(index=300 + l), "cpu", N_q)
        store = wk.Store([k.clone().pin_memory() for k in ks], [v.clone().pin_memory() for v in vs])
        out.append(dict(ks=ks, vs=vs, Kn=Kn, Vn=Vn, Q=Q, store=store))
    return out


@pytest.mark.parametrize("max_wg", [0, 3])
def test_layer_loop_with_prefetch_matches_oracle_and_sequential(max_wg):
    d = dev()
    cfg = ws.get_config(1).with_(H=4)
    L, R, n_native, N_q = 5, 3, 517, 300
    lens = [700, 333, 1024, 64, 901, 650]
    M = len(lens)
    layers = _layers(cfg, L, lens, n_native, N_q)
    poses, cur = ws.make_poses(M, 77)
    cap = n_native + R * max(lens)
    ids = torch.empty(R, dtype=torch.int32, device=d)
    nf = torch.empty(1, dtype=torch.int32, device=d)
    Kn = [x["Kn"].to(d) for x in layers]
    Vn = [x["Vn"].to(d) for x in layers]
    Qd = [x["Q"].to(d) for x in layers]
    win = [(torch.full((cfg.H, cap, cfg.d), 3.0, dtype=torch.bfloat16, device=d),
            torch.full((cfg.H, cap, cfg.d), 5.0, dtype=torch.bfloat16, device=d)) for _ in range(2)]
    n_win = [torch.zeros(1, dtype=torch.int32, device=d) for _ in range(2)]
    O = [torch.empty_like(q) for q in Qd]
    snap = [(torch.empty_like(win[0][0]), torch.empty_like(win[0][1])) for _ in range(L)]
    n_snap = torch.zeros(L, dtype=torch.int32, device=d)

    p = wk.wk_prefetch_create(2)
    try:
        with pytest.raises(wk.WkError):
            wk.wk_prefetch_acquire(p, 0)          # nothing was gathered into the slot yet
        wk.wk_score_chunks(torch.from_numpy(poses).to(d), M, cur, wk.WK_NORM_MAX, R, ids, None, nf)
        wk.wk_prefetch_after(p)                   # ids are final before the first gather reads them
        wk.wk_prefetch_gather(p, 0, layers[0]["store"].desc, ids, nf, R, Kn[0], Vn[0], n_native, win[0][0], win[0][1],
                              cap, n_win[0], max_wg)
        for l in range(L):
            s = l % 2
            if l + 1 < L:
                t = (l + 1) % 2
                wk.wk_prefetch_gather(p, t, layers[l + 1]["store"].desc, ids, nf, R, Kn[l + 1], Vn[l + 1], n_native,
                                      win[t][0], win[t][1], cap, n_win[t], max_wg)
            wk.wk_prefetch_acquire(p, s)
            wk.wk_attention(Qd[l], win[s][0], win[s][1], O[l], None, N_kv=cap, n_kv_dev=n_win[s])
            snap[l][0].copy_(win[s][0])           # more readers of the slot, for the byte check below
            snap[l][1].copy_(win[s][1])
            n_snap[l:l + 1].copy_(n_win[s])
            wk.wk_prefetch_release(p, s)
        torch.cuda.synchronize()
    finally:
        wk.wk_prefetch_destroy(p)

    o_ids, _, _ = oracle.score_chunks(poses, cur, R)
    np.testing.assert_array_equal(ids.cpu().numpy(), o_ids)
    for l, x in enumerate(layers):
        oK, oV, o_n = oracle.gather(x["ks"], x["vs"], o_ids, x["Kn"], x["Vn"], cap)
        assert int(n_snap[l].item()) == o_n
        assert torch.equal(bits(snap[l][0][:, :o_n].cpu()), bits(oK[:, :o_n])), l
        assert torch.equal(bits(snap[l][1][:, :o_n].cpu()), bits(oV[:, :o_n])), l
        ref = oracle.attention(x["Q"], oK, oV, N_kv=o_n)
        mx, mean = attention_errors(O[l], ref)
        assert mx <= ATT_MAX_ABS_BF16 and mean <= ATT_MEAN_ABS_BF16, (l, mx, mean)
        # the plain sequence on one stream gives the same bits
        Kw = torch.zeros_like(win[0][0])
        Vw = torch.zeros_like(Kw)
        nw = torch.zeros(1, dtype=torch.int32, device=d)
        O2 = torch.empty_like(O[l])
        wk.wk_gather_window(x["store"].desc, ids, nf, R, Kn[l], Vn[l], n_native, Kw, Vw, cap, nw)
        wk.wk_attention(Qd[l], Kw, Vw, O2, None, N_kv=cap, n_kv_dev=nw)
        torch.cuda.synchronize()
        assert torch.equal(bits(O2), bits(O[l])), l


def test_capped_grid_gather_is_byte_exact():
    """Every cap from one workgroup up walks all work units (HBM store, fp32 and bf16)."""
    d = dev()
    for dtype in (ws.configs.DT_BF16, ws.configs.DT_F32):
        cfg = ws.get_config(1).with_(H=3, dtype=dtype)
        lens = [5, 300, 77, 1, 129, 64]
        ks, vs = [], []
        for c, n in enumerate(lens):
            k, v = ws.make_native(cfg.with_(index=50 + c), n_rows=n)
            ks.append(k), vs.append(v)
        store = wk.Store([k.to(d) for k in ks], [v.to(d) for v in vs])
        Kn, Vn = ws.make_native(cfg, n_rows=131)
        cap = 131 + 4 * 300
        ids = [1, 0, 5, 2]
        oK, oV, o_n = oracle.gather(ks, vs, ids, Kn, Vn, cap)
        ids_d = torch.tensor(ids, dtype=torch.int32, device=d)
        p = wk.wk_prefetch_create(1)
        try:
            for max_wg in (1, 2, 7, 64, 100000):
                Kw = torch.full((cfg.H, cap, cfg.d), 7.0, dtype=ws.torch_dtype(dtype), device=d)
                Vw = torch.full_like(Kw, 9.0)
                nw = torch.full((1,), -1, dtype=torch.int32, device=d)
                wk.wk_prefetch_after(p)
                wk.wk_prefetch_gather(p, 0, store.desc, ids_d, None, 4, Kn.to(d), Vn.to(d), 131, Kw, Vw, cap, nw, max_wg)
                wk.wk_prefetch_acquire(p, 0)
                Kc, Vc = Kw.clone(), Vw.clone()
                wk.wk_prefetch_release(p, 0)
                torch.cuda.synchronize()
                assert int(nw.item()) == o_n
                assert torch.equal(bits(Kc[:, :o_n].cpu()), bits(oK[:, :o_n]))
                assert torch.equal(bits(Vc[:, :o_n].cpu()), bits(oV[:, :o_n]))
                assert (Kc[:, o_n:] == 7).all() and (Vc[:, o_n:] == 9).all()
        finally:
            wk.wk_prefetch_destroy(p)


def test_eviction_to_host_store_on_the_copy_stream():
    """Compression of an evicted chunk straight into mapped host memory, enqueued on the prefetch stream
    while the compute stream attends (Sec. 7), gives the oracle's compacted chunk."""
    d = dev()
    cfg = ws.get_config(1).with_(H=2, T=200)
    K, V, A = ws.make_chunk(cfg, 3)
    n_out, _ = wk.wk_keep_count(cfg.rho, cfg.ratio_kind, cfg.anchor_mode, cfg.F, cfg.T)
    desc = wk.make_compress_desc(cfg.H, cfg.T, cfg.F, cfg.dtype, cfg.rho, ratio_kind=cfg.ratio_kind,
                                 anchor_mode=cfg.anchor_mode)
    wsb = torch.empty(wk.wk_compress_workspace_bytes(desc), dtype=torch.uint8, device=d)
    Kh = torch.zeros((cfg.H, n_out, cfg.d), dtype=torch.bfloat16).pin_memory()
    Vh = torch.zeros_like(Kh).pin_memory()
    idx = torch.empty((1, n_out), dtype=torch.int32, device=d)
    Kd, Vd = K.to(d), V.to(d)                       # produced on the compute stream
    Q = ws.make_queries(cfg, d, 512)
    Kn, Vn = ws.make_native(cfg, d, 4096)
    O = torch.empty_like(Q)
    p = wk.wk_prefetch_create(1)
    try:
        wk.wk_prefetch_after(p)                     # the chunk's K/V exist before the copy stream reads them
        with torch.cuda.stream(torch.cuda.ExternalStream(wk.wk_prefetch_stream(p))):
            wk.wk_compress_chunk(desc, Kd, Vd, None, idx, Kh, Vh, wsb)
        wk.wk_attention(Q, Kn, Vn, O)               # meanwhile, on the compute stream
        torch.cuda.synchronize()
    finally:
        wk.wk_prefetch_destroy(p)
    o_idx, oK, oV, _ = oracle.compress(K, V, A, cfg.T, cfg.F, cfg.rho, cfg.ratio_kind, anchor_mode=cfg.anchor_mode)
    np.testing.assert_array_equal(idx.cpu().numpy(), o_idx)
    assert torch.equal(bits(Kh), bits(oK)) and torch.equal(bits(Vh), bits(oV))
    mx, mean = attention_errors(O, oracle.attention(Q.cpu(), Kn.cpu(), Vn.cpu()))
    assert mx <= ATT_MAX_ABS_BF16 and mean <= ATT_MEAN_ABS_BF16
