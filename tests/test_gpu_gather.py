"""GPU parity of wk_gather_window against the oracle: byte-exact window assembly (Sec. 4.2)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2605_22718_amd as wk
import wk_synth as ws
from wkt import bits, dev

pytestmark = pytest.mark.gpu


def _store(cfg, lengths, pinned=False):
    ks, vs = [], []
    for c, n in enumerate(lengths):
        k, v = ws.make_native(cfg.with_(index=50 + c), n_rows=n)
        ks.append(k), vs.append(v)
    if pinned:
        place = lambda t: t.clone().pin_memory()
    else:
        place = lambda t: t.to(dev())
    return ks, vs, wk.Store([place(k) for k in ks], [place(v) for v in vs])


def _gather(cfg, store, ids, n_ids, R_max, Kn, Vn, cap, in_place=False):
    d = dev()
    Kw = torch.full((cfg.H, cap, cfg.d), 7.0, dtype=ws.torch_dtype(cfg.dtype), device=d)
    Vw = torch.full_like(Kw, 9.0)
    n_native = Kn.shape[1]
    if in_place:
        Kw[:, :n_native] = Kn.to(d)
        Vw[:, :n_native] = Vn.to(d)
    n_win = torch.full((1,), -1, dtype=torch.int32, device=d)
    ids_d = torch.tensor(list(ids) + [0] * (R_max - len(ids)), dtype=torch.int32, device=d) if R_max else None
    n_ids_d = None if n_ids is None else torch.tensor([n_ids], dtype=torch.int32, device=d)
    wk.wk_gather_window(store.desc, ids_d, n_ids_d, R_max, None if in_place else Kn.to(d),
                        None if in_place else Vn.to(d), n_native, Kw, Vw, cap, n_win)
    torch.cuda.synchronize()
    return Kw.cpu(), Vw.cpu(), int(n_win.item())


@pytest.mark.parametrize("dtype", [ws.configs.DT_BF16, ws.configs.DT_F32])
@pytest.mark.parametrize("pinned", [False, True])
def test_gather_matches_oracle(dtype, pinned):
    cfg = ws.get_config(1).with_(H=3, dtype=dtype)
    lengths = [5, 300, 77, 1, 129, 64]
    ks, vs, store = _store(cfg, lengths, pinned)
    Kn, Vn = ws.make_native(cfg, n_rows=131)
    cap = 131 + 4 * 300
    for ids in ([1, 0, 5, 2], [3], [], [4, 4, 1]):
        Kw, Vw, n_win = _gather(cfg, store, ids, len(ids), 4, Kn, Vn, cap)
        oK, oV, o_n = oracle.gather(ks, vs, ids, Kn, Vn, cap)
        assert n_win == o_n
        assert torch.equal(bits(Kw[:, :n_win]), bits(oK[:, :n_win])) and torch.equal(bits(Vw[:, :n_win]), bits(oV[:, :n_win]))
        assert (Kw[:, n_win:] == 7).all() and (Vw[:, n_win:] == 9).all()     # rows past the window untouched
    # n_ids = NULL uses all R_max ids; invalid ids are skipped
    Kw, Vw, n_win = _gather(cfg, store, [2, -1, 99, 0], None, 4, Kn, Vn, cap)
    oK, oV, o_n = oracle.gather(ks, vs, [2, 0], Kn, Vn, cap)
    assert n_win == o_n and torch.equal(bits(Kw[:, :n_win]), bits(oK[:, :n_win]))
    # native rows already in place
    Kw, Vw, n_win = _gather(cfg, store, [5, 1], 2, 4, Kn, Vn, cap, in_place=True)
    oK, oV, o_n = oracle.gather(ks, vs, [5, 1], Kn, Vn, cap)
    assert n_win == o_n and torch.equal(bits(Kw[:, :n_win]), bits(oK[:, :n_win])) and torch.equal(bits(Vw[:, :n_win]), bits(oV[:, :n_win]))


def test_no_native_rows_and_no_retrieval():
    cfg = ws.get_config(1).with_(H=2)
    ks, vs, store = _store(cfg, [40, 40])
    empty = torch.zeros((2, 0, 128), dtype=torch.bfloat16)
    Kw, Vw, n_win = _gather(cfg, store, [1, 0], 2, 2, empty, empty, 80)
    oK, oV, o_n = oracle.gather(ks, vs, [1, 0], None, None, 80)
    assert n_win == 80 and torch.equal(bits(Kw), bits(oK)) and torch.equal(bits(Vw), bits(oV))
    Kn, Vn = ws.make_native(cfg, n_rows=33)
    Kw, Vw, n_win = _gather(cfg, store, [], 0, 0, Kn, Vn, 33)     # R_max = 0: sliding window only
    assert n_win == 33 and torch.equal(bits(Kw), bits(Kn)) and torch.equal(bits(Vw), bits(Vn))


@pytest.mark.parametrize("ci,order", [(1, (4, 0, 5, 2)), (2, (9, 4, 0, 5, 2, 11, 7, 1))])
def test_config_sized_gather(ci, order):
    """Configs 1 and 2 at full size from an HBM store, in the launch the bench times (ids on the device)."""
    cfg = ws.get_config(ci)
    d = dev()
    n_out, _ = wk.wk_keep_count(cfg.rho, cfg.ratio_kind, cfg.anchor_mode, cfg.F, cfg.T)
    ks = [ws.make_native(cfg.with_(index=70 + c), d, n_rows=n_out) for c in range(12)]
    store = wk.Store([k for k, _ in ks], [v for _, v in ks])
    Kn, Vn = ws.make_native(cfg, d)
    cap = cfg.n_native + cfg.R * n_out
    Kw = torch.zeros((cfg.H, cap, cfg.d), dtype=torch.bfloat16, device=d)
    Vw = torch.zeros_like(Kw)
    ids = torch.tensor(order, dtype=torch.int32, device=d)
    n_win = torch.zeros(1, dtype=torch.int32, device=d)
    wk.wk_gather_window(store.desc, ids, None, cfg.R, Kn, Vn, cfg.n_native, Kw, Vw, cap, n_win)
    torch.cuda.synchronize()
    assert int(n_win.item()) == cap == (10560 if ci == 1 else 28080)
    expect_k = torch.cat([Kn] + [ks[i][0] for i in order], 1)
    expect_v = torch.cat([Vn] + [ks[i][1] for i in order], 1)
    assert torch.equal(bits(Kw), bits(expect_k)) and torch.equal(bits(Vw), bits(expect_v))
    # byte-exact against the oracle on one head's slice (the oracle copies on the CPU)
    oK, oV, _ = oracle.gather([k[:1].cpu() for k, _ in ks], [v[:1].cpu() for _, v in ks], list(order),
                              Kn[:1].cpu(), Vn[:1].cpu(), cap)
    assert torch.equal(bits(Kw[:1].cpu()), bits(oK)) and torch.equal(bits(Vw[:1].cpu()), bits(oV))
    # native rows already in place: only the retrieved chunks move, same window
    Kw2, Vw2 = torch.zeros_like(Kw), torch.zeros_like(Vw)
    Kw2[:, :cfg.n_native], Vw2[:, :cfg.n_native] = Kn, Vn
    wk.wk_gather_window(store.desc, ids, None, cfg.R, None, None, cfg.n_native, Kw2, Vw2, cap, n_win)
    torch.cuda.synchronize()
    assert torch.equal(bits(Kw2), bits(expect_k)) and torch.equal(bits(Vw2), bits(expect_v))


def test_calibration_copy_is_exact():
    d = dev()
    g = torch.Generator(device="cpu").manual_seed(1)
    for n in (16, 48, 32 * 1024 + 16, 5 * 1024 * 1024 + 32):
        src = torch.randint(0, 255, (n,), dtype=torch.uint8, generator=g).to(d)
        dst = torch.zeros(n + 16, dtype=torch.uint8, device=d)
        wk.wk_calibration_copy(dst[:n], src)
        torch.cuda.synchronize()
        assert torch.equal(dst[:n], src) and int(dst[n:].sum()) == 0


def test_chunks_beyond_the_descriptors_bound_are_skipped():
    """max_tok is a hard bound: a chunk whose n_tok exceeds it is skipped (its head stride is its true length,
    so it cannot be read cut short), by the gather and by attention in place alike."""
    import ctypes as C
    cfg = ws.get_config(1).with_(H=3)
    lengths = [40, 300, 77, 129]
    ks, vs, store = _store(cfg, lengths)
    tight = wk.wk_store_desc(store.K_ptr.data_ptr(), store.V_ptr.data_ptr(), store.n_tok.data_ptr(), len(lengths),
                             129, cfg.H, cfg.d, store.dtype)          # chunk 1 (300 rows) violates the bound
    Kn, Vn = ws.make_native(cfg, n_rows=70)
    ids = [3, 1, 0, 2]
    cap = 70 + 4 * 129
    d = dev()
    Kw = torch.full((cfg.H, cap, cfg.d), 7.0, dtype=torch.bfloat16, device=d)
    Vw = torch.full_like(Kw, 9.0)
    n_win = torch.full((1,), -1, dtype=torch.int32, device=d)
    ids_d = torch.tensor(ids, dtype=torch.int32, device=d)
    wk.wk_gather_window(tight, ids_d, None, 4, Kn.to(d), Vn.to(d), 70, Kw, Vw, cap, n_win)
    torch.cuda.synchronize()
    oK, oV, o_n = oracle.gather(ks, vs, [3, 0, 2], Kn, Vn, cap)
    assert int(n_win.item()) == o_n == 70 + 129 + 40 + 77
    assert torch.equal(bits(Kw.cpu()[:, :o_n]), bits(oK[:, :o_n])) and torch.equal(bits(Vw.cpu()[:, :o_n]), bits(oV[:, :o_n]))
    assert (Kw[:, o_n:] == 7).all()
    # attention in place skips the same chunk
    Q = ws.make_queries(cfg, n_q=90)
    O = torch.empty((cfg.H, 90, cfg.d), dtype=torch.bfloat16, device=d)
    lse = torch.empty((cfg.H, 90), dtype=torch.float32, device=d)
    wk.wk_attention_in_place(Q.to(d), Kn.to(d), Vn.to(d), 70, tight, ids_d, None, 4, O, lse)
    torch.cuda.synchronize()
    ref, ref_lse = oracle.attention(Q, oK, oV, N_kv=o_n, want_lse=True)
    err = np.abs(O.float().cpu().numpy().astype(np.float64) - ref)
    assert err.max() <= 2e-2 and err.mean() <= 2e-3
    assert np.abs(lse.cpu().numpy() - ref_lse).max() <= 2e-2
    # the chunk index for query-based retrieval reports such a chunk as empty
    out = torch.empty((len(lengths), cfg.H, 90), dtype=torch.float32, device=d)
    wk.wk_chunk_lse(tight, Q.to(d), out)
    torch.cuda.synchronize()
    assert torch.isinf(out[1]).all() and (out[1] < 0).all() and torch.isfinite(out[[0, 2, 3]]).all()
