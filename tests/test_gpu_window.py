"""Window bookkeeping on the GPU (Sec. 4.2 regions): in-place refresh of the retrieved slots against the
oracle's slot policy, byte-exact, and a rolling generation loop through every entry point."""
import random

import numpy as np
import pytest
import torch

import oracle
import paper_2605_22718_amd as wk
import wk_synth as ws
from oracle.window import update_slots
from wkt import ATT_MAX_ABS_BF16, ATT_MEAN_ABS_BF16, attention_errors, bits, dev

pytestmark = pytest.mark.gpu


def _pattern(H, n, d, cid, version, dtype):
    """Chunk content as small integers (exact in bf16), different for every (chunk, version, row, column)."""
    h = torch.arange(H).view(H, 1, 1)
    r = torch.arange(n).view(1, n, 1)
    c = torch.arange(d).view(1, 1, d)
    return ((cid * 7 + version * 3 + h * 5 + r + c) % 200).to(dtype)


@pytest.mark.parametrize("dtype,pinned", [(torch.bfloat16, False), (torch.float32, False), (torch.bfloat16, True)])
def test_slot_refresh_matches_oracle_and_copies_only_newcomers(dtype, pinned):
    d = dev()
    H, slot_tokens, M, n_native = 3, 150, 12, 70
    lens = [slot_tokens] * M
    lens[4] = slot_tokens - 1          # chunks of another length cannot be placed: dropped
    lens[9] = slot_tokens + 3
    version = [0] * M
    place = (lambda t: t.pin_memory()) if pinned else (lambda t: t.to(d))
    Ks = [place(_pattern(H, lens[c], 128, c, 0, dtype)) for c in range(M)]
    Vs = [place(_pattern(H, lens[c], 128, c + 50, 0, dtype)) for c in range(M)]
    store = wk.Store(Ks, Vs, d)
    rng = random.Random(11)
    for R in (1, 4, 6):
        cap = n_native + R * slot_tokens + 9
        Kw = torch.full((H, cap, 128), 251.0, dtype=dtype, device=d)
        Vw = torch.full((H, cap, 128), 253.0, dtype=dtype, device=d)
        slot_ids = torch.full((R,), -1, dtype=torch.int32, device=d)
        n_win = torch.zeros(1, dtype=torch.int32, device=d)
        n_f = torch.zeros(1, dtype=torch.int32, device=d)
        wsb = torch.empty(wk.wk_window_update_workspace_bytes(R), dtype=torch.uint8, device=d)
        model_slots = [-1] * R
        model_rows = {}                # slot -> (K rows, V rows) as fetched
        cur = rng.sample(range(M), min(R, 3))
        for step in range(14):
            # a drifting request: mostly the previous ids, sometimes new, invalid or repeated ones
            if step % 5 == 4:
                cur = cur[: max(1, len(cur) - 2)]                      # shrinking request: may force a rebuild
            else:
                cur = [i if rng.random() < 0.7 else rng.randint(-1, M) for i in cur]
                while len(cur) < R and rng.random() < 0.6:
                    cur.append(rng.randint(0, M - 1))
            rng.shuffle(cur)
            ids = torch.tensor(cur + [0] * (R - len(cur)), dtype=torch.int32, device=d)
            n_ids = torch.tensor([len(cur)], dtype=torch.int32, device=d)
            max_wg = [0, 2, 64][step % 3]
            wk.wk_window_update(store.desc, ids, n_ids, R, slot_tokens, slot_ids, n_native, Kw, Vw, cap, n_win, n_f,
                                wsb, max_wg)
            torch.cuda.synchronize()
            valid = lambda i: 0 <= i < M and lens[i] == slot_tokens
            new_slots, fetched = update_slots(model_slots, cur, R, valid)
            assert slot_ids.cpu().tolist() == new_slots, (R, step, cur, model_slots)
            assert int(n_f.item()) == len(fetched)
            n = sum(1 for x in new_slots if x >= 0)
            assert int(n_win.item()) == n_native + n * slot_tokens
            for s, i in fetched:
                model_rows[s] = (Ks[i].clone().cpu(), Vs[i].clone().cpu())
            model_slots = new_slots
            Kc, Vc = Kw.cpu(), Vw.cpu()
            for s in range(n):
                r0 = n_native + s * slot_tokens
                assert torch.equal(bits(Kc[:, r0:r0 + slot_tokens]), bits(model_rows[s][0])), (R, step, s)
                assert torch.equal(bits(Vc[:, r0:r0 + slot_tokens]), bits(model_rows[s][1])), (R, step, s)
            assert (Kc[:, :n_native] == 251).all() and (Vc[:, :n_native] == 253).all()        # native rows untouched
            assert (Kc[:, n_native + R * slot_tokens:] == 251).all()                            # nothing past the slots
            # change the store's copy of every resident chunk: a needless re-fetch would now show up
            for i in set(x for x in model_slots if x >= 0):
                version[i] += 1
                Ks[i].copy_(_pattern(H, lens[i], 128, i, version[i], dtype))
                Vs[i].copy_(_pattern(H, lens[i], 128, i + 50, version[i], dtype))
            torch.cuda.synchronize()


def test_rolling_generation_loop_through_every_entry_point():
    """Chunks are generated one after another; the planner says where each lives and when one leaves;
    the evicted chunk is compressed into the store; poses pick the chunks to retrieve; the retrieved
    slots are refreshed in place; the denoising chunk attends over the window.  Every step's output is
    compared with the oracle run on the oracle's own bookkeeping."""
    d = dev()
    cfg = ws.get_config(1).with_(H=2, T=96)
    F, T, H = cfg.F, cfg.T, cfg.H
    n_chunks, R = 9, 3
    n_out, _ = wk.wk_keep_count(cfg.rho, cfg.ratio_kind, cfg.anchor_mode, F, T)
    wdesc = wk.wk_window_desc(T, F, 1, 1, R, n_out)
    cdesc = wk.make_compress_desc(H, T, F, cfg.dtype, cfg.rho, ratio_kind=cfg.ratio_kind, anchor_mode=cfg.anchor_mode)
    cws = torch.empty(wk.wk_compress_workspace_bytes(cdesc), dtype=torch.uint8, device=d)
    p0 = wk.wk_window_plan(wdesc, 0)
    cap = p0.win_capacity
    Kw = torch.zeros((H, cap, cfg.d), dtype=torch.bfloat16, device=d)
    Vw = torch.zeros_like(Kw)
    # the store's tables are sized for the whole rollout; n_tok = 0 marks chunks not stored yet
    sk = torch.zeros((n_chunks, H, n_out, cfg.d), dtype=torch.bfloat16, device=d)
    sv = torch.zeros_like(sk)
    store = wk.Store([sk[c] for c in range(n_chunks)], [sv[c] for c in range(n_chunks)], d)
    poses_np, _ = ws.make_poses(n_chunks, 5)          # pose of generated chunk c
    slot_ids = torch.full((R,), -1, dtype=torch.int32, device=d)
    uws = torch.empty(wk.wk_window_update_workspace_bytes(R), dtype=torch.uint8, device=d)
    ids = torch.empty(R, dtype=torch.int32, device=d)
    nf = torch.empty(1, dtype=torch.int32, device=d)
    n_win = torch.empty(1, dtype=torch.int32, device=d)
    idx = torch.empty((1, n_out), dtype=torch.int32, device=d)
    o_store_k, o_store_v, o_slots, stored_pose = [], [], [-1] * R, []
    gen = [ws.make_chunk(cfg, 40 + c) for c in range(n_chunks)]          # the K/V each new chunk brings
    for c in range(n_chunks):
        p = wk.wk_window_plan(wdesc, c)
        if p.evict:
            Ke = Kw[:, p.evict_row0:p.evict_row0 + p.denoise_rows].contiguous()
            Ve = Vw[:, p.evict_row0:p.evict_row0 + p.denoise_rows].contiguous()
            wk.wk_compress_chunk(cdesc, Ke, Ve, None, idx, sk[p.store_id], sv[p.store_id], cws)
            gK, gV, _ = gen[p.evict_chunk]
            _, oK, oV, _ = oracle.compress(gK, gV, None, T, F, cfg.rho, cfg.ratio_kind, anchor_mode=cfg.anchor_mode)
            o_store_k.append(oK), o_store_v.append(oV)
            stored_pose.append(poses_np[p.evict_chunk])
        Kc, Vc, _ = gen[c]
        Kw[:, p.denoise_row0:p.denoise_row0 + p.denoise_rows] = Kc.to(d)
        Vw[:, p.denoise_row0:p.denoise_row0 + p.denoise_rows] = Vc.to(d)
        Q = ws.make_queries(cfg.with_(index=60 + c), d, F * T)
        O = torch.empty_like(Q)
        M = p.M
        store.desc.M = M                               # chunks stored so far
        if M > 0:
            pose_tab = torch.from_numpy(np.stack(stored_pose)).to(d)
            wk.wk_score_chunks(pose_tab, M, poses_np[c], wk.WK_NORM_MAX, R, ids, None, nf)
            wk.wk_window_update(store.desc, ids, nf, R, n_out, slot_ids, p.retrieved_row0, Kw, Vw, cap, n_win, None, uws)
            wk.wk_attention(Q, Kw, Vw, O, None, N_kv=cap, n_kv_dev=n_win)
        else:
            wk.wk_attention(Q, Kw, Vw, O, None, N_kv=p.n_native)
        torch.cuda.synchronize()
        # the oracle's side of the same step
        if M > 0:
            o_ids, _, _ = oracle.score_chunks(np.stack(stored_pose), poses_np[c], R)
            o_slots, _ = update_slots(o_slots, [int(i) for i in o_ids], R, lambda i: 0 <= i < M)
            assert slot_ids.cpu().tolist() == o_slots
            order = [i for i in o_slots if i >= 0]
            native_k, native_v = Kw[:, :p.n_native].cpu(), Vw[:, :p.n_native].cpu()
            oKw, oVw, o_n = oracle.gather(o_store_k, o_store_v, order, native_k, native_v, cap)
            assert int(n_win.item()) == o_n
            assert torch.equal(bits(Kw[:, :o_n].cpu()), bits(oKw[:, :o_n])) and torch.equal(bits(Vw[:, :o_n].cpu()), bits(oVw[:, :o_n]))
        else:
            o_n = p.n_native
            oKw, oVw = Kw[:, :o_n].cpu().contiguous(), Vw[:, :o_n].cpu().contiguous()
        mx, mean = attention_errors(O, oracle.attention(Q.cpu(), oKw, oVw, N_kv=o_n))
        assert mx <= ATT_MAX_ABS_BF16 and mean <= ATT_MEAN_ABS_BF16, (c, mx, mean)
    assert len(o_store_k) == n_chunks - 3 and p.M == n_chunks - 3      # all but the sink chunk and the two in the ring


def test_slot_refresh_at_the_lingbot_window_size():
    """Config 2 at full size: 8 slots of 2,340 rows x 40 heads behind 9,360 native rows.  First fill, then a
    request that keeps five chunks and brings three new ones: only those three are copied, every slot holds its
    chunk byte for byte, the native rows stay as they were."""
    d = dev()
    cfg = ws.get_config(2)
    n_out, _ = wk.wk_keep_count(cfg.rho, cfg.ratio_kind, cfg.anchor_mode, cfg.F, cfg.T)
    M, R = 12, cfg.R
    Ks, Vs = [], []
    for c in range(M):
        k, v = ws.make_native(cfg.with_(index=300 + c), d, n_rows=n_out)
        Ks.append(k), Vs.append(v)
    store = wk.Store(Ks, Vs, d)
    cap = cfg.n_native + R * n_out
    Kn, Vn = ws.make_native(cfg, d)
    Kw = torch.zeros((cfg.H, cap, cfg.d), dtype=torch.bfloat16, device=d)
    Vw = torch.zeros_like(Kw)
    Kw[:, :cfg.n_native], Vw[:, :cfg.n_native] = Kn, Vn
    slot_ids = torch.full((R,), -1, dtype=torch.int32, device=d)
    n_win = torch.zeros(1, dtype=torch.int32, device=d)
    n_f = torch.zeros(1, dtype=torch.int32, device=d)
    wsb = torch.empty(wk.wk_window_update_workspace_bytes(R), dtype=torch.uint8, device=d)
    model = [-1] * R
    for req, expect_fetched in (([0, 1, 2, 3, 4, 5, 6, 7], 8), ([7, 9, 1, 3, 10, 5, 11, 0], 3)):
        ids = torch.tensor(req, dtype=torch.int32, device=d)
        n_ids = torch.tensor([len(req)], dtype=torch.int32, device=d)
        wk.wk_window_update(store.desc, ids, n_ids, R, n_out, slot_ids, cfg.n_native, Kw, Vw, cap, n_win, n_f, wsb)
        torch.cuda.synchronize()
        model, fetched = update_slots(model, req, R, lambda i: 0 <= i < M)
        assert slot_ids.cpu().tolist() == model
        assert int(n_f.item()) == len(fetched) == expect_fetched
        assert int(n_win.item()) == cap
        for s, c in enumerate(model):
            r0 = cfg.n_native + s * n_out
            assert torch.equal(bits(Kw[:, r0:r0 + n_out]), bits(Ks[c])) and torch.equal(bits(Vw[:, r0:r0 + n_out]), bits(Vs[c])), s
        assert torch.equal(bits(Kw[:, :cfg.n_native]), bits(Kn)) and torch.equal(bits(Vw[:, :cfg.n_native]), bits(Vn))
