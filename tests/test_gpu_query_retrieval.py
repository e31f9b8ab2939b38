"""GPU parity of query-based retrieval (Sec. 4.2, App. C): wk_attention's log-sum-exp per stored
chunk -> wk_score_chunks_query, against the oracle's joint softmax over all candidates' keys."""
import numpy as np
import pytest
import torch

import oracle
import paper_2605_22718_amd as wk
import wk_synth as ws
from wkt import TIE_BAND, dev

pytestmark = pytest.mark.gpu

# Mass of a chunk = mean over rows of exp(lse_c - L).  With fp32 inputs the kernel's lse is good to
# ~1e-6; with bf16 inputs the probabilities are rounded to bf16 before the row sum (relative 2^-9
# each, averaging down over the keys), which the attention parity tests bound by 2e-2 on lse in the
# worst case and which is ~1e-3 in practice.  A relative error e on every l_c moves a mass by at
# most ~2e of itself.
MASS_RTOL = {torch.float32: 2e-5, torch.bfloat16: 1e-2}


def _chunk_lse(Q, Ks):
    """lse [M][H*N_q] from one O = NULL attention call per chunk."""
    d = dev()
    H, N_q, _ = Q.shape
    out = torch.full((max(len(Ks), 1), H * N_q), float("nan"), dtype=torch.float32, device=d)
    Qd = Q.to(d)
    for c, K in enumerate(Ks):
        wk.wk_attention(Qd, K.to(d), None, None, out[c].view(H, N_q))
    return out


def _chunk_lse_batched(Q, Ks):
    """The same from one wk_chunk_lse launch over a store of the chunks' keys."""
    d = dev()
    H, N_q, _ = Q.shape
    Kd = [K.to(d) for K in Ks]
    store = wk.Store(Kd, Kd, d)
    out = torch.full((len(Ks), H * N_q), float("nan"), dtype=torch.float32, device=d)
    wk.wk_chunk_lse(store.desc, Q.to(d), out)
    torch.cuda.synchronize()
    return out


def _gpu_query_scores(lse, M, R):
    d = dev()
    n_rows = lse.shape[1]
    ids = torch.full((max(R, 1),), -7, dtype=torch.int32, device=d)
    mass = torch.full((max(R, 1),), -7.0, dtype=torch.float64, device=d)
    nf = torch.full((1,), -7, dtype=torch.int32, device=d)
    wsb = torch.empty(wk.wk_score_chunks_query_workspace_bytes(M, n_rows), dtype=torch.uint8, device=d)
    wk.wk_score_chunks_query(lse, M, n_rows, R, ids, mass, nf, wsb)
    torch.cuda.synchronize()
    all_mass = wsb[: 8 * M].view(torch.float64).cpu().numpy().copy()
    return ids.cpu().numpy()[:R], mass.cpu().numpy()[:R], int(nf.item()), all_mass


def _compare(Q, Ks, R):
    M = len(Ks)
    lse = _chunk_lse(Q, Ks)
    if M:
        assert torch.equal(lse, _chunk_lse_batched(Q, Ks))   # one launch over the store = one call per chunk
    ids, mass, nf, all_mass = _gpu_query_scores(lse, M, R)
    o_ids, o_sel, o_all = oracle.score_chunks_query(Q, Ks, R)
    assert nf == o_ids.size == min(R, M)
    assert np.all(ids[nf:] == -1) and np.all(np.isneginf(mass[nf:]))
    rtol = MASS_RTOL[Q.dtype]
    np.testing.assert_allclose(all_mass, o_all, rtol=rtol, atol=1e-12)
    g = ids[:nf]
    assert len(set(g.tolist())) == nf
    # what the GPU returns is exactly the ordering of its own masses, ties to the lower id ...
    order = np.lexsort((np.arange(M), -all_mass))[:nf]
    np.testing.assert_array_equal(g, order)
    np.testing.assert_array_equal(mass[:nf], all_mass[order])
    # ... and it may differ from the oracle's only between chunks whose exact masses are closer
    # than the arithmetic can resolve
    if not np.array_equal(g, o_ids):
        band = np.maximum(2 * rtol * o_sel, TIE_BAND)
        assert np.all(np.abs(o_all[g] - o_sel) <= band), (g, o_ids, o_all[g], o_sel)
    return g, o_ids, o_all


@pytest.mark.parametrize("index,H,N_q,lens", [
    (0, 2, 75, [64, 33, 1, 130, 257, 90]),             # fp32 path; ragged and one-key chunks
    (1, 3, 300, [880 + 137 * (c % 5) for c in range(12)]),   # bf16: several tiles, ragged tails
    (2, 2, 520, [1560 + 390 * (c % 4) for c in range(20)]),
])
def test_revisited_chunks_rank_by_attention_mass(index, H, N_q, lens):
    cfg = ws.get_config(index).with_(H=H)
    Q = ws.make_queries(cfg, "cpu", N_q)
    Ks, a = ws.make_revisit_keys(cfg, Q, lens)
    for R in sorted({0, 1, 3, len(lens), len(lens) + 2}):
        _compare(Q, Ks, R)


def test_lse_only_mode_matches_full_attention_lse():
    d = dev()
    for index, N_q, N_kv in [(0, 70, 150), (1, 300, 1000), (1, 256, 64), (2, 520, 4681)]:
        cfg = ws.get_config(index).with_(H=2)
        Q = ws.make_queries(cfg, d, N_q)
        K, V = ws.make_native(cfg, d, N_kv)
        O = torch.empty_like(Q)
        full = torch.empty((2, N_q), dtype=torch.float32, device=d)
        only = torch.full((2, N_q), float("nan"), dtype=torch.float32, device=d)
        wk.wk_attention(Q, K, V, O, full)
        wk.wk_attention(Q, K, None, None, only)
        torch.cuda.synchronize()
        assert torch.equal(full, only)                 # same arithmetic for the row sums
        _, ref = oracle.attention(Q.cpu(), K.cpu(), V.cpu(), want_lse=True)
        err = np.abs(only.cpu().numpy().astype(np.float64) - ref).max()
        assert err <= (1e-4 if Q.dtype == torch.float32 else 2e-2)
    # lse-only honours the device-side window length and an oversized stride
    cfg = ws.get_config(1).with_(H=2)
    Q = ws.make_queries(cfg, d, 100)
    K, V = ws.make_native(cfg, d, 500)
    nk = torch.tensor([333], dtype=torch.int32, device=d)
    only = torch.empty((2, 100), dtype=torch.float32, device=d)
    wk.wk_attention(Q, K, None, None, only, n_kv_dev=nk)
    torch.cuda.synchronize()
    _, ref = oracle.attention(Q.cpu(), K.cpu(), V.cpu(), N_kv=333, want_lse=True)
    assert np.abs(only.cpu().numpy().astype(np.float64) - ref).max() <= 2e-2


def test_query_scores_from_given_lse_exact_cases():
    d = dev()
    # every chunk the same lse: equal masses 1/M, ids come out 0,1,2,...
    lse = torch.full((5, 1000), 3.25, dtype=torch.float32, device=d)
    ids, mass, nf, all_mass = _gpu_query_scores(lse, 5, 3)
    np.testing.assert_array_equal(ids, [0, 1, 2])
    np.testing.assert_allclose(all_mass, 0.2, rtol=0, atol=1e-15)
    # lse_c = log(w_c) for every row: mass_c = w_c / sum(w)
    w = np.array([1.0, 8.0, 2.0, 4.0, 0.5, 0.25])
    lse = torch.tensor(np.log(w), dtype=torch.float32, device=d).view(-1, 1).repeat(1, 777).contiguous()
    ids, mass, nf, all_mass = _gpu_query_scores(lse, 6, 6)
    np.testing.assert_array_equal(ids, [1, 3, 2, 0, 4, 5])
    np.testing.assert_allclose(all_mass, w / w.sum(), rtol=1e-7)
    # an empty chunk (lse = -inf) gets mass 0; a row that sees no key at all is skipped
    lse = torch.zeros((3, 300), dtype=torch.float32, device=d)
    lse[1] = float("-inf")
    lse[:, 17] = float("-inf")
    ids, mass, nf, all_mass = _gpu_query_scores(lse, 3, 3)
    np.testing.assert_array_equal(ids, [0, 2, 1])
    np.testing.assert_allclose(all_mass, [0.5 * 299 / 300, 0.0, 0.5 * 299 / 300], rtol=1e-12)
    # empty store, single candidate, M at the limit, more rows than one pass of the grid covers
    ids, mass, nf, _ = _gpu_query_scores(torch.zeros((1, 10), dtype=torch.float32, device=d), 0, 2)
    assert nf == 0 and np.all(ids == -1)
    ids, mass, nf, all_mass = _gpu_query_scores(torch.randn((1, 10), device=d), 1, 2)
    assert nf == 1 and ids[0] == 0 and ids[1] == -1 and abs(all_mass[0] - 1.0) < 1e-15
    M = wk.WK_QUERY_MAX_CHUNKS
    g = torch.Generator(device="cpu").manual_seed(3)
    lse_h = torch.randn((M, 600), generator=g)
    ids, mass, nf, all_mass = _gpu_query_scores(lse_h.to(d), M, 16)
    p = torch.softmax(lse_h.double(), 0).mean(1).numpy()
    np.testing.assert_allclose(all_mass, p, rtol=1e-12)
    np.testing.assert_array_equal(ids, np.lexsort((np.arange(M), -p))[:16])
    lse_h = torch.randn((3, 1024 * 256 + 77), generator=g)
    ids, mass, nf, all_mass = _gpu_query_scores(lse_h.to(d), 3, 3)
    np.testing.assert_allclose(all_mass, torch.softmax(lse_h.double(), 0).mean(1).numpy(), rtol=1e-12)
    assert abs(all_mass.sum() - 1.0) < 1e-12


@pytest.mark.parametrize("index", [0, 1])
def test_chunk_lse_against_oracle_with_empty_and_pinned_chunks(index):
    d = dev()
    cfg = ws.get_config(index).with_(H=2)
    Q = ws.make_queries(cfg, "cpu", 301)
    lens = [64, 0, 1, 63, 65, 500, 129]
    Ks, _ = ws.make_revisit_keys(cfg, Q, lens)
    # chunk 5 lives in pinned host memory (CPU-offloaded store), the others in HBM
    Kd = [K.pin_memory() if c == 5 else K.to(d) for c, K in enumerate(Ks)]
    store = wk.Store(Kd, Kd, d)
    out = torch.full((len(Ks), 2, 301), float("nan"), dtype=torch.float32, device=d)
    wk.wk_chunk_lse(store.desc, Q.to(d), out)
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    assert np.all(np.isneginf(got[1]))
    for c, K in enumerate(Ks):
        if lens[c] == 0:
            continue
        _, ref = oracle.attention(Q, K, K, want_lse=True)
        assert np.abs(got[c] - ref).max() <= (1e-4 if Q.dtype == torch.float32 else 2e-2), c


def test_chunk_lse_and_masses_at_the_lingbot_index_size_sampled():
    """The index the bench times: anchor-frame keys (1,560 per chunk) of 120 stored chunks, 40 heads, 4,680
    queries.  Sampled (chunk, query row) entries of the log-sum-exp against the oracle on all heads, and the masses
    and ids of wk_score_chunks_query against a softmax over the GPU's own log-sum-exps taken in fp64."""
    d = dev()
    cfg = ws.get_config(2)
    M, n_anchor = cfg.M, cfg.T
    Q = ws.make_queries(cfg, d)
    keys = torch.empty((M, cfg.H, n_anchor, cfg.d), dtype=torch.bfloat16, device=d)
    for c in range(M):
        keys[c] = ws.make_native(cfg.with_(index=200 + c), d, n_rows=n_anchor)[0]
    store = wk.Store([keys[c] for c in range(M)], [keys[c] for c in range(M)], d)
    lse = torch.full((M, cfg.H, cfg.N_q), float("nan"), dtype=torch.float32, device=d)
    wk.wk_chunk_lse(store.desc, Q, lse)
    torch.cuda.synchronize()
    assert torch.isfinite(lse).all()
    rng = np.random.default_rng(7)
    rows = sorted(set([0, 255, 256, cfg.N_q - 1] + rng.integers(0, cfg.N_q, 8).tolist()))
    Qc = Q.cpu()
    for c in [0, 1, 57, M - 1]:
        Kc = keys[c].cpu()
        _, ref = oracle.attention(Qc, Kc, Kc, rows=rows, want_lse=True)
        got = lse[c][:, rows].cpu().numpy().astype(np.float64)
        assert np.abs(got - ref).max() <= 2e-2, c
    n_rows = cfg.H * cfg.N_q
    wsb = torch.empty(wk.wk_score_chunks_query_workspace_bytes(M, n_rows), dtype=torch.uint8, device=d)
    ids = torch.full((cfg.R,), -7, dtype=torch.int32, device=d)
    mass = torch.zeros(cfg.R, dtype=torch.float64, device=d)
    nf = torch.zeros(1, dtype=torch.int32, device=d)
    wk.wk_score_chunks_query(lse, M, n_rows, cfg.R, ids, mass, nf, wsb)
    torch.cuda.synchronize()
    all_mass = wsb[: M * 8].view(torch.float64).cpu().numpy()
    expect = torch.softmax(lse.view(M, n_rows).double(), 0).mean(1).cpu().numpy()
    np.testing.assert_allclose(all_mass, expect, rtol=1e-9)
    assert abs(all_mass.sum() - 1.0) < 1e-9 and int(nf.item()) == cfg.R
    np.testing.assert_array_equal(ids.cpu().numpy(), np.lexsort((np.arange(M), -expect))[: cfg.R])
