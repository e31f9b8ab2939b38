"""GPU parity on seeded random shapes: attention (both element types, with and without workspace, device-side
window length), attention in place over ragged stores with skipped ids, compression in every mode, the
frame-causal mask in random window layouts, query-based and pose-based retrieval, each against the oracle.  Shapes are drawn from lists that straddle the tile sizes (32, 64, 256)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2605_22718_amd as wk
from wkt import assert_selection_matches, attention_errors, bits, dev as _dev

pytestmark = pytest.mark.gpu


def _rand(shape, dtype, g):
    return torch.randn(*shape, generator=g).to(dtype)


@pytest.mark.parametrize("seed", [1, 2])
def test_attention_random_shapes(seed):
    rng = np.random.default_rng(seed)
    dev = _dev()
    for it in range(30):
        H = int(rng.integers(1, 5))
        Nq = int(rng.choice([1, 31, 32, 33, 100, 255, 256, 257, 300, 513, 700]))
        Nkv = int(rng.choice([1, 2, 63, 64, 65, 127, 128, 129, 300, 1000, 2049, 4100]))
        stride = Nkv + int(rng.integers(0, 3))
        dtype = torch.bfloat16 if rng.random() < 0.7 else torch.float32
        g = torch.Generator().manual_seed(100 * seed + it)
        Q, K, V = _rand((H, Nq, 128), dtype, g), _rand((H, stride, 128), dtype, g), _rand((H, stride, 128), dtype, g)
        use_ws = rng.random() < 0.6
        n_dev = None if rng.random() < 0.6 else int(rng.integers(1, Nkv + 1))
        scale = float(rng.choice([0.0, 0.05, 0.3]))
        code = wk.WK_BF16 if dtype == torch.bfloat16 else wk.WK_F32
        n = wk.wk_attention_workspace_bytes(H, Nq, Nkv, code) if use_ws else 0
        wsb = torch.empty(n, dtype=torch.uint8, device=dev) if n else None
        O = torch.full(Q.shape, float("nan"), dtype=dtype, device=dev)
        lse = torch.full((H, Nq), float("nan"), dtype=torch.float32, device=dev)
        nk = None if n_dev is None else torch.tensor([n_dev], dtype=torch.int32, device=dev)
        what = f"case {it}: H={H} Nq={Nq} Nkv={Nkv} stride={stride} {dtype} ws={n} n_dev={n_dev} scale={scale}"
        wk.wk_attention(Q.to(dev), K.to(dev), V.to(dev), O, lse, N_kv=Nkv, scale=scale, n_kv_dev=nk, workspace=wsb)
        torch.cuda.synchronize()
        n_eff = Nkv if n_dev is None else min(Nkv, n_dev)
        ref, ref_lse = oracle.attention(Q, K, V, N_kv=n_eff, scale=None if scale == 0.0 else scale, want_lse=True)
        mx, mean = attention_errors(O, ref)
        # fp32: logits reach ~15 at scale 0.3, where the rounding of the 128-term dot products shows in exp
        tol = (2e-2, 2e-3) if dtype == torch.bfloat16 else (2e-5, 2e-6)
        assert mx <= tol[0] and mean <= tol[1], (what, mx, mean)
        el = np.abs(lse.cpu().numpy().astype(np.float64) - ref_lse).max()
        assert el <= (2e-2 if dtype == torch.bfloat16 else 1e-4), (what, el)


@pytest.mark.parametrize("seed", [1, 2])
def test_attention_in_place_random_stores(seed):
    rng = np.random.default_rng(10 + seed)
    dev = _dev()
    for it in range(25):
        H = int(rng.integers(1, 4))
        Nq = int(rng.choice([1, 33, 256, 300]))
        M = int(rng.integers(1, 7))
        lens = [int(rng.choice([0, 1, 5, 63, 64, 65, 128, 200, 129])) for _ in range(M)]
        n_native = int(rng.choice([0, 1, 64, 100, 131]))
        R = int(rng.integers(0, 7))
        ids = [int(rng.integers(-1, M + 1)) for _ in range(R)]          # -1 and M are not in the store
        n_ids = None if rng.random() < 0.5 else int(rng.integers(0, R + 1))
        g = torch.Generator().manual_seed(1000 * seed + it)
        ks = [_rand((H, n, 128), torch.bfloat16, g) for n in lens]
        vs = [_rand((H, n, 128), torch.bfloat16, g) for n in lens]
        # an empty chunk still needs an address: one row of backing, length 0 in the table
        dk = [(k if k.shape[1] else torch.zeros((H, 1, 128), dtype=torch.bfloat16)).to(dev) for k in ks]
        dv = [(v if v.shape[1] else torch.zeros((H, 1, 128), dtype=torch.bfloat16)).to(dev) for v in vs]
        store = wk.Store(dk, dv)
        store.n_tok.copy_(torch.tensor(lens, dtype=torch.int32, device=dev))
        Q = _rand((H, Nq, 128), torch.bfloat16, g)
        Kn, Vn = _rand((H, n_native + 2, 128), torch.bfloat16, g), _rand((H, n_native + 2, 128), torch.bfloat16, g)
        O = torch.full(Q.shape, float("nan"), dtype=torch.bfloat16, device=dev)
        lse = torch.full((H, Nq), float("nan"), dtype=torch.float32, device=dev)
        ids_d = torch.tensor(ids + [0] * (8 - len(ids)), dtype=torch.int32, device=dev)
        n_ids_d = None if n_ids is None else torch.tensor([n_ids], dtype=torch.int32, device=dev)
        what = f"case {it}: H={H} Nq={Nq} lens={lens} n_native={n_native} ids={ids} n_ids={n_ids}"
        wk.wk_attention_in_place(Q.to(dev), Kn.to(dev), Vn.to(dev), n_native, store.desc, ids_d, n_ids_d, R, O, lse)
        torch.cuda.synchronize()
        used = ids if n_ids is None else ids[:n_ids]
        valid = [i for i in used if 0 <= i < M and lens[i] > 0]
        total = n_native + sum(lens[i] for i in valid)
        if total == 0:
            assert (O == 0).all() and torch.isinf(lse).all(), what
            continue
        Knn = Kn[:, :n_native].contiguous() if n_native else None
        Vnn = Vn[:, :n_native].contiguous() if n_native else None
        Kw, Vw, n_win = oracle.gather(ks, vs, valid, Knn, Vnn, total)
        ref, ref_lse = oracle.attention(Q, Kw, Vw, want_lse=True)
        mx, mean = attention_errors(O, ref)
        assert mx <= 2e-2 and mean <= 2e-3, (what, mx, mean)
        assert np.abs(lse.cpu().numpy().astype(np.float64) - ref_lse).max() <= 2e-2, what


@pytest.mark.parametrize("seed", [1, 2])
def test_compress_random_modes(seed):
    rng = np.random.default_rng(20 + seed)
    dev = _dev()
    done = 0
    for it in range(40):
        H = int(rng.choice([1, 2, 3, 4, 5, 7, 12]))
        T = int(rng.choice([1, 7, 16, 33, 100, 250]))
        F = int(rng.integers(1, 5))
        dtype = torch.bfloat16 if rng.random() < 0.7 else torch.float32
        code = wk.WK_BF16 if dtype == torch.bfloat16 else wk.WK_F32
        ext = F == 1 or rng.random() < 0.3
        anchor_mode = wk.WK_ANCHOR_EXTERNAL if ext else wk.WK_ANCHOR_FIRST_FRAME
        head_mode = wk.WK_HEADS_INDEPENDENT if rng.random() < 0.4 else wk.WK_HEADS_SHARED
        ratio_kind = wk.WK_RATIO_NONANCHOR if rng.random() < 0.5 else wk.WK_RATIO_CHUNK
        rho = float(np.float32(rng.choice([0.0, 0.25, 0.5, 0.6, 0.75, 1.0])))
        algo = wk.WK_SCORE_GEMM if (dtype == torch.bfloat16 and rng.random() < 0.4) else wk.WK_SCORE_FACTORED
        try:
            n_out, n_keep = wk.wk_keep_count(rho, ratio_kind, anchor_mode, F, T)
        except wk.WkError:
            continue                                                       # ratio below the anchor frame
        g = torch.Generator().manual_seed(2000 * seed + it)
        K, V = _rand((H, F * T, 128), dtype, g), _rand((H, F * T, 128), dtype, g)
        Ka = _rand((H, T, 128), dtype, g) if ext else None
        desc = wk.make_compress_desc(H, T, F, code, rho, head_mode=head_mode, anchor_mode=anchor_mode,
                                     ratio_kind=ratio_kind, score_algo=algo)
        wsb = torch.empty(wk.wk_compress_workspace_bytes(desc), dtype=torch.uint8, device=dev)
        G = H if head_mode == wk.WK_HEADS_INDEPENDENT else 1
        idx = torch.full((G, n_out), -5, dtype=torch.int32, device=dev)
        Ko = torch.zeros((H, n_out, 128), dtype=dtype, device=dev)
        Vo = torch.zeros_like(Ko)
        what = (f"case {it}: H={H} T={T} F={F} {dtype} ext={ext} head_mode={head_mode} ratio_kind={ratio_kind} "
                f"rho={rho} algo={algo} n_out={n_out}")
        got = wk.wk_compress_chunk(desc, K.to(dev), V.to(dev), None if Ka is None else Ka.to(dev), idx, Ko, Vo, wsb)
        torch.cuda.synchronize()
        oidx, oK, oV, osc = oracle.compress(K, V, Ka, T, F, rho, ratio_kind, head_mode, anchor_mode)
        assert got == n_out, what
        first = 0 if ext else T
        gi = idx.cpu().numpy()
        for gg in range(G):
            if first:
                assert np.array_equal(gi[gg, :first], np.arange(first)), what
            if n_out > first:
                assert_selection_matches(gi[gg, first:] - first, oidx[gg, first:] - first, osc[gg], what)
        for h in range(H):                                  # rows copied verbatim at the indices the GPU reports
            sel = torch.as_tensor(gi[h if G > 1 else 0].astype(np.int64))
            assert torch.equal(bits(Ko[h].cpu()), bits(K[h][sel])) and torch.equal(bits(Vo[h].cpu()), bits(V[h][sel])), what
        done += 1
    assert done >= 20


@pytest.mark.parametrize("seed", [1, 2])
def test_block_causal_random_layouts(seed):
    rng = np.random.default_rng(30 + seed)
    dev = _dev()
    for it in range(24):
        H = int(rng.integers(1, 4))
        frames = int(rng.choice([1, 2, 3, 4, 9, 12]))             # 9 and 12 frames: one launch per frame
        T = int(rng.choice([1, 7, 32, 33, 100, 256, 300]))
        Nq = frames * T
        before, after = int(rng.choice([0, 1, 64, 100, 257])), int(rng.choice([0, 1, 63, 200, 513]))
        Nkv = before + Nq + after
        stride = Nkv + int(rng.integers(0, 2))
        dtype = torch.bfloat16 if rng.random() < 0.7 else torch.float32
        g = torch.Generator().manual_seed(3000 * seed + it)
        Q, K, V = _rand((H, Nq, 128), dtype, g), _rand((H, stride, 128), dtype, g), _rand((H, stride, 128), dtype, g)
        wsb = torch.empty(wk.wk_attention_block_causal_workspace_bytes(H, Nq), dtype=torch.uint8, device=dev)
        O = torch.full(Q.shape, float("nan"), dtype=dtype, device=dev)
        lse = torch.full((H, Nq), float("nan"), dtype=torch.float32, device=dev)
        what = f"case {it}: H={H} frames={frames} T={T} before={before} after={after} {dtype}"
        wk.wk_attention_block_causal(Q.to(dev), K.to(dev), V.to(dev), O, before, T, wsb, lse=lse, N_kv=Nkv)
        torch.cuda.synchronize()
        ref, ref_lse = oracle.attention_block_causal(Q, K, V, before, T, N_kv=Nkv, want_lse=True)
        mx, mean = attention_errors(O, ref)
        tol = (2e-2, 2e-3) if dtype == torch.bfloat16 else (2e-5, 2e-6)
        assert mx <= tol[0] and mean <= tol[1], (what, mx, mean)
        el = np.abs(lse.cpu().numpy().astype(np.float64) - ref_lse).max()
        assert el <= (2e-2 if dtype == torch.bfloat16 else 1e-4), (what, el)


@pytest.mark.parametrize("seed", [1, 2])
def test_query_retrieval_random_stores(seed):
    rng = np.random.default_rng(40 + seed)
    dev = _dev()
    for it in range(16):
        H = int(rng.integers(1, 4))
        Nq = int(rng.choice([1, 33, 256, 300]))
        M = int(rng.integers(1, 9))
        lens = [int(rng.choice([1, 5, 63, 64, 65, 128, 200])) for _ in range(M)]
        R = int(rng.integers(1, 10))
        dtype = torch.bfloat16 if rng.random() < 0.7 else torch.float32
        g = torch.Generator().manual_seed(4000 * seed + it)
        Q = _rand((H, Nq, 128), dtype, g)
        ks = [_rand((H, n, 128), dtype, g) for n in lens]
        store = wk.Store([k.to(dev) for k in ks], [k.to(dev) for k in ks])
        lse = torch.full((M, H, Nq), float("nan"), dtype=torch.float32, device=dev)
        what = f"case {it}: H={H} Nq={Nq} lens={lens} R={R} {dtype}"
        wk.wk_chunk_lse(store.desc, Q.to(dev), lse)
        wsb = torch.empty(wk.wk_score_chunks_query_workspace_bytes(M, H * Nq), dtype=torch.uint8, device=dev)
        ids = torch.full((R,), -7, dtype=torch.int32, device=dev)
        mass = torch.zeros(R, dtype=torch.float64, device=dev)
        nf = torch.zeros(1, dtype=torch.int32, device=dev)
        wk.wk_score_chunks_query(lse, M, H * Nq, R, ids, mass, nf, wsb)
        torch.cuda.synchronize()
        oids, _, oall = oracle.score_chunks_query(Q, ks, R)
        n = int(nf.item())
        assert n == min(R, M), what
        gm = wsb[: M * 8].view(torch.float64).cpu().numpy()
        tolm = 5e-3 if dtype == torch.bfloat16 else 1e-5        # masses are sums of exp(lse differences) of fp32 lse
        assert np.abs(gm - oall).max() <= tolm, (what, np.abs(gm - oall).max())
        gi = ids.cpu().numpy()
        for a_, b_ in zip(gi[:n], oids):                        # same ids, except between masses that tie
            assert a_ == b_ or abs(oall[a_] - oall[b_]) <= 2 * tolm, (what, gi, oids)
        assert (gi[n:] == -1).all(), what


@pytest.mark.parametrize("seed", [1, 2])
def test_pose_retrieval_random_tables(seed):
    rng = np.random.default_rng(50 + seed)
    dev = _dev()
    for it in range(30):
        M = int(rng.choice([0, 1, 2, 5, 16, 100, 1000]))
        R = int(rng.integers(1, 20))
        mode = int(rng.integers(0, 3))
        poses = np.zeros((max(M, 1), 5), np.float32)
        poses[:, :3] = rng.normal(0, 5, (max(M, 1), 3))
        poses[:, 3] = rng.uniform(-4, 4, max(M, 1))
        poses[:, 4] = rng.uniform(-1, 1, max(M, 1))
        if M > 3 and rng.random() < 0.5:
            poses[M // 2] = poses[0]                            # an exact duplicate: a tie, lower id first
        cur = poses[0] + rng.normal(0, 0.1, 5).astype(np.float32)
        ids = torch.full((R,), -7, dtype=torch.int32, device=dev)
        dist = torch.zeros(R, dtype=torch.float64, device=dev)
        nf = torch.zeros(1, dtype=torch.int32, device=dev)
        what = f"case {it}: M={M} R={R} mode={mode}"
        wk.wk_score_chunks(torch.from_numpy(poses).to(dev), M, cur, mode, R, ids, dist, nf)
        torch.cuda.synchronize()
        oids, od, oall = oracle.score_chunks(poses[:M], cur, R, mode)
        n = int(nf.item())
        assert n == min(R, M), what
        gi, gd = ids.cpu().numpy()[:n], dist.cpu().numpy()[:n]
        if n:
            assert np.abs(gd - od).max() <= 1e-9, (what, np.abs(gd - od).max())
        for a_, b_ in zip(gi, oids):
            assert a_ == b_ or abs(oall[a_] - oall[b_]) <= 1e-6, (what, gi, oids)
