"""GPU parity of wk_compress_chunk against the oracle (World Compression, Sec. 4.3, Eq. 5).
Kept-index sets must be bit-exact outside the 1e-6 tie band; compaction is byte-exact."""
import numpy as np
import pytest
import torch

import oracle
import paper_2605_22718_amd as wk
import wk_synth as ws
from wkt import assert_selection_matches, bits, dev

pytestmark = pytest.mark.gpu
SCORE_TOL = 1e-7   # absolute; the adjacent-score gaps near the cut are a few 1e-6


def _gpu_compress(cfg, K, V, K_anchor, batch=1, head_mode=wk.WK_HEADS_SHARED, rho=None, ratio_kind=None,
                  score_algo=wk.WK_SCORE_FACTORED):
    d = dev()
    rho = cfg.rho if rho is None else rho
    ratio_kind = cfg.ratio_kind if ratio_kind is None else ratio_kind
    desc = wk.make_compress_desc(cfg.H, cfg.T, cfg.F, cfg.dtype, rho, batch=batch, head_mode=head_mode,
                                 anchor_mode=cfg.anchor_mode, ratio_kind=ratio_kind, score_algo=score_algo)
    n_out, n_keep = wk.wk_keep_count(rho, ratio_kind, cfg.anchor_mode, cfg.F, cfg.T)
    G = cfg.H if head_mode == wk.WK_HEADS_INDEPENDENT else 1
    n_cand = cfg.F * cfg.T - (0 if cfg.anchor_mode == wk.WK_ANCHOR_EXTERNAL else cfg.T)
    nbytes = wk.wk_compress_workspace_bytes(desc)
    assert nbytes > 0
    wsb = torch.zeros(nbytes, dtype=torch.uint8, device=d)
    idx = torch.full((batch, G, n_out), -1, dtype=torch.int32, device=d)
    Ko = torch.zeros((batch, cfg.H, n_out, cfg.d), dtype=K.dtype, device=d)
    Vo = torch.zeros_like(Ko)
    got = wk.wk_compress_chunk(desc, K.to(d), V.to(d), None if K_anchor is None else K_anchor.to(d), idx, Ko, Vo, wsb)
    torch.cuda.synchronize()
    assert got == n_out
    scores = wsb[: batch * G * n_cand * 8].view(torch.float64).view(batch, G, n_cand).cpu().numpy()
    return idx.cpu().numpy(), Ko.cpu(), Vo.cpu(), scores, n_out


def _compare_chunk(cfg, K, V, K_anchor, g_idx, g_K, g_V, g_scores, head_mode, rho, ratio_kind, oracle_result=None):
    o_idx, o_K, o_V, o_scores = oracle_result or oracle.compress(K, V, K_anchor, cfg.T, cfg.F, rho, ratio_kind,
                                                                 head_mode, cfg.anchor_mode)
    assert np.abs(g_scores - o_scores).max() <= SCORE_TOL, np.abs(g_scores - o_scores).max()
    first = 0 if cfg.anchor_mode == wk.WK_ANCHOR_EXTERNAL else cfg.T
    for g in range(o_idx.shape[0]):
        np.testing.assert_array_equal(g_idx[g, :first], np.arange(first))
        assert_selection_matches(g_idx[g, first:] - first, o_idx[g, first:] - first, o_scores[g], f"list {g}")
    # compaction is a verbatim copy of the rows the GPU selected ...
    for h in range(cfg.H):
        sel = torch.as_tensor(g_idx[h if head_mode == wk.WK_HEADS_INDEPENDENT else 0], dtype=torch.long)
        assert torch.equal(bits(g_K[h]), bits(K[h, sel])) and torch.equal(bits(g_V[h]), bits(V[h, sel]))
    # ... and equals the oracle's chunk whenever the index sets agree
    if np.array_equal(g_idx, o_idx):
        assert torch.equal(bits(g_K), bits(o_K)) and torch.equal(bits(g_V), bits(o_V))
    return bool(np.array_equal(g_idx, o_idx))


@pytest.mark.parametrize("dtype", [ws.configs.DT_BF16, ws.configs.DT_F32])
@pytest.mark.parametrize("head_mode", [wk.WK_HEADS_SHARED, wk.WK_HEADS_INDEPENDENT])
@pytest.mark.parametrize("H,T,F", [(3, 50, 3), (2, 17, 4), (5, 130, 2)])
def test_small_chunks(dtype, head_mode, H, T, F):
    cfg = ws.get_config(1).with_(H=H, T=T, F=F, dtype=dtype)
    K, V, _ = ws.make_chunk(cfg, 0)
    for rho, kind in [(0.5, wk.WK_RATIO_CHUNK), (0.25, wk.WK_RATIO_NONANCHOR), (0.75, wk.WK_RATIO_NONANCHOR)]:
        gi, gK, gV, gs, _ = _gpu_compress(cfg, K, V, None, head_mode=head_mode, rho=rho, ratio_kind=kind)
        _compare_chunk(cfg, K, V, None, gi[0], gK[0], gV[0], gs[0], head_mode, rho, kind)


def test_batch_of_chunks_and_external_anchor():
    cfg = ws.get_config(0).with_(H=2, T=70)       # one-frame chunks against an external anchor, fp32
    chunks = [ws.make_chunk(cfg, c) for c in range(3)]
    K = torch.stack([c[0] for c in chunks])
    V = torch.stack([c[1] for c in chunks])
    A = torch.stack([c[2] for c in chunks])
    gi, gK, gV, gs, n_out = _gpu_compress(cfg, K, V, A, batch=3)
    assert n_out == 35
    for b in range(3):
        _compare_chunk(cfg, K[b], V[b], A[b], gi[b], gK[b], gV[b], gs[b], wk.WK_HEADS_SHARED, cfg.rho, cfg.ratio_kind)


@pytest.mark.parametrize("ci,H,T,F,batch,dtype", [
    (1, 4, 300, 2, 128, ws.configs.DT_F32),      # 3 head rows per lane group, fp32
    (1, 12, 280, 3, 128, ws.configs.DT_BF16),    # 3, bf16, T not a multiple of the tokens per workgroup
    (1, 33, 200, 2, 192, ws.configs.DT_BF16),    # 10, heads not a multiple of 4
    (0, 48, 140, 1, 256, ws.configs.DT_BF16),    # 16, external anchor
])
def test_batches_that_take_the_one_pass_anchor_kernel(ci, H, T, F, batch, dtype):
    """Batches with T * batch >= 8 * 4096 tokens: anchor norms and the normalised anchor mean come from the
    one-pass kernel, in each of its three sizes.  Several chunks of the batch against the whole oracle."""
    cfg = ws.get_config(ci).with_(H=H, T=T, F=F, dtype=dtype)
    assert T * batch >= 8 * 4096
    picks = [0, 1, batch // 2, batch - 1]
    base = {c: ws.make_chunk(cfg, c) for c in picks}
    idx = [picks[b % len(picks)] for b in range(batch)]
    K = torch.stack([base[c][0] for c in idx])
    V = torch.stack([base[c][1] for c in idx])
    A = torch.stack([base[c][2] for c in idx]) if cfg.anchor_mode == wk.WK_ANCHOR_EXTERNAL else None
    gi, gK, gV, gs, _ = _gpu_compress(cfg, K, V, A, batch=batch, rho=0.75)
    for b in [0, 1, 2, 3, batch - 1]:
        _compare_chunk(cfg, K[b], V[b], None if A is None else A[b], gi[b], gK[b], gV[b], gs[b], wk.WK_HEADS_SHARED,
                       0.75, cfg.ratio_kind)
    # equal chunks of the batch give equal results, whichever workgroups served them
    for b in range(len(picks), batch):
        assert np.array_equal(gi[b], gi[b % len(picks)]) and np.array_equal(gs[b], gs[b % len(picks)])


@pytest.mark.parametrize("dtype", [ws.configs.DT_BF16, ws.configs.DT_F32])
def test_rho_one_is_identity_and_rho_zero_is_anchor_only(dtype):
    cfg = ws.get_config(1).with_(H=2, T=40, dtype=dtype)
    K, V, _ = ws.make_chunk(cfg, 2)
    gi, gK, gV, _, n_out = _gpu_compress(cfg, K, V, None, rho=1.0)
    assert n_out == cfg.F * cfg.T
    np.testing.assert_array_equal(gi[0, 0], np.arange(n_out))
    assert torch.equal(bits(gK[0]), bits(K)) and torch.equal(bits(gV[0]), bits(V))
    gi, gK, gV, _, n_out = _gpu_compress(cfg, K, V, None, rho=0.0, ratio_kind=wk.WK_RATIO_NONANCHOR)
    assert n_out == cfg.T
    np.testing.assert_array_equal(gi[0, 0], np.arange(cfg.T))
    assert torch.equal(bits(gK[0]), bits(K[:, :cfg.T]))


def test_exact_ties_go_to_the_lower_index():
    cfg = ws.get_config(1).with_(H=2, T=32, F=3)
    K, V, _ = ws.make_chunk(cfg, 3)
    # duplicate candidate tokens: equal rows give bit-equal scores on both sides
    K[:, cfg.T + 10: cfg.T + 40] = K[:, cfg.T + 5: cfg.T + 6]
    K[:, cfg.T + 50: cfg.T + 60] = K[:, cfg.T + 45: cfg.T + 46]
    for rho in (0.1, 0.3, 0.5, 0.7, 0.9):
        gi, gK, gV, gs, _ = _gpu_compress(cfg, K, V, None, rho=rho, ratio_kind=wk.WK_RATIO_NONANCHOR)
        same = _compare_chunk(cfg, K, V, None, gi[0], gK[0], gV[0], gs[0], wk.WK_HEADS_SHARED,
                              float(np.float32(rho)), wk.WK_RATIO_NONANCHOR)
        assert same
    # a zero key has score 0 on both sides
    K[:, cfg.T + 3] = 0
    gi, gK, gV, gs, _ = _gpu_compress(cfg, K, V, None)
    assert gs[0, 0, 3] == 0.0
    _compare_chunk(cfg, K, V, None, gi[0], gK[0], gV[0], gs[0], wk.WK_HEADS_SHARED, cfg.rho, cfg.ratio_kind)


@pytest.mark.parametrize("head_mode", [wk.WK_HEADS_SHARED, wk.WK_HEADS_INDEPENDENT])
@pytest.mark.parametrize("H,T,F", [(3, 50, 3), (2, 17, 4), (5, 130, 2), (2, 64, 3)])
def test_gemm_scoring_small_chunks(head_mode, H, T, F):
    """Eq. 5 as a token-by-anchor similarity GEMM on the matrix cores: same scores, same index sets."""
    cfg = ws.get_config(1).with_(H=H, T=T, F=F)
    K, V, _ = ws.make_chunk(cfg, 5)
    K[:, T + 3] = 0          # a zero candidate and a zero anchor
    K[:, 1] = 0
    for rho, kind in [(0.5, wk.WK_RATIO_CHUNK), (0.25, wk.WK_RATIO_NONANCHOR)]:
        gi, gK, gV, gs, _ = _gpu_compress(cfg, K, V, None, head_mode=head_mode, rho=rho, ratio_kind=kind,
                                          score_algo=wk.WK_SCORE_GEMM)
        _compare_chunk(cfg, K, V, None, gi[0], gK[0], gV[0], gs[0], head_mode, rho, kind)


def test_gemm_scoring_external_anchor_batch_and_fp32_refusal():
    cfg = ws.get_config(0).with_(H=2, T=70, dtype=ws.configs.DT_BF16)
    chunks = [ws.make_chunk(cfg, c) for c in range(2)]
    K = torch.stack([c[0] for c in chunks])
    V = torch.stack([c[1] for c in chunks])
    A = torch.stack([c[2] for c in chunks])
    gi, gK, gV, gs, n_out = _gpu_compress(cfg, K, V, A, batch=2, score_algo=wk.WK_SCORE_GEMM)
    for b in range(2):
        _compare_chunk(cfg, K[b], V[b], A[b], gi[b], gK[b], gV[b], gs[b], wk.WK_HEADS_SHARED, cfg.rho, cfg.ratio_kind)
    desc = wk.make_compress_desc(2, 70, 1, wk.WK_F32, 0.5, anchor_mode=wk.WK_ANCHOR_EXTERNAL, score_algo=wk.WK_SCORE_GEMM)
    assert wk.wk_compress_workspace_bytes(desc) == 0      # the matrix-core variant is bf16 only


# (config 0 is fp32; the matrix-core scoring variant is bf16 only)
@pytest.mark.parametrize("ci,algo", [(0, wk.WK_SCORE_FACTORED), (1, wk.WK_SCORE_FACTORED), (1, wk.WK_SCORE_GEMM)])
def test_config_sized_chunk_full_compare(ci, algo):
    cfg = ws.get_config(ci)
    K, V, A = ws.make_chunk(cfg, 1)
    gi, gK, gV, gs, n_out = _gpu_compress(cfg, K, V, A, score_algo=algo)
    assert n_out == {0: 440, 1: 1320}[ci]
    same = _compare_chunk(cfg, K, V, A, gi[0], gK[0], gV[0], gs[0], wk.WK_HEADS_SHARED, cfg.rho, cfg.ratio_kind)
    print(f"config{ci}: index set identical to the oracle: {same}; max score err {np.abs(gs[0] - oracle.compress_scores(K, A, cfg.T, cfg.F, anchor_mode=cfg.anchor_mode)).max():.2e}")


@pytest.mark.parametrize("algo", [wk.WK_SCORE_FACTORED, wk.WK_SCORE_GEMM])
@pytest.mark.parametrize("head_mode", [wk.WK_HEADS_SHARED, wk.WK_HEADS_INDEPENDENT])
def test_lingbot_sized_batch_sampled(head_mode, algo):
    """Config 2/4 shape (H=40, T=1560, F=3), a batch of 2 chunks at P in {0.25, 0.75}: oracle scores on
    sampled candidates, and -- valid at any size -- the kept set is exactly the n_keep lowest of the
    GPU's own scores with ties to the lower index."""
    cfg = ws.get_config(4)
    d = dev()
    chunks = [ws.make_chunk(cfg, c, d) for c in range(2)]
    K = torch.stack([c[0] for c in chunks])
    V = torch.stack([c[1] for c in chunks])
    rng = np.random.default_rng(0)
    sel = np.unique(np.concatenate([[0, 1, 3119, 1559, 1560], rng.integers(0, 3120, 40)])).astype(np.int32)
    for P in (0.25, 0.75):
        gi, gK, gV, gs, n_out = _gpu_compress(cfg, K, V, None, batch=2, head_mode=head_mode, rho=P,
                                              ratio_kind=wk.WK_RATIO_NONANCHOR, score_algo=algo)
        n_keep = n_out - cfg.T
        assert n_out == {0.25: 2340, 0.75: 3900}[P]
        for b in range(2):
            Kc, Vc = K[b].cpu(), V[b].cpu()
            for g in range(gs.shape[1]):
                order = np.lexsort((np.arange(gs.shape[2]), gs[b, g]))[:n_keep]
                np.testing.assert_array_equal(gi[b, g, cfg.T:] - cfg.T, np.sort(order))
                np.testing.assert_array_equal(gi[b, g, :cfg.T], np.arange(cfg.T))
            if b == 0 and P == 0.25:
                o = oracle.compress_scores(Kc, None, cfg.T, cfg.F, head_mode, cand_sel=sel)
                heads = range(gs.shape[1])
                err = max(np.abs(gs[b, g, sel] - o[g, sel]).max() for g in heads)
                assert err <= SCORE_TOL, err
            for h in (0, 17, 39):
                s_idx = torch.as_tensor(gi[b, h if head_mode == wk.WK_HEADS_INDEPENDENT else 0], dtype=torch.long)
                assert torch.equal(bits(gK[b, h]), bits(Kc[h, s_idx])) and torch.equal(bits(gV[b, h]), bits(Vc[h, s_idx]))


# ---- one full LingBot-sized chunk (configs 2 and 4: H = 40, T = 1,560, F = 3) against the whole oracle ----
_ORACLE_CACHE = {}


def _lingbot_chunk():
    if "chunk" not in _ORACLE_CACHE:
        cfg = ws.get_config(2)
        K, V, _ = ws.make_chunk(cfg, 3, dev())       # generated once on the GPU; both sides get these bytes
        _ORACLE_CACHE["chunk"] = (cfg, K.cpu(), V.cpu())
    return _ORACLE_CACHE["chunk"]


def _lingbot_oracle(head_mode, rho, kind):
    """oracle.compress of the whole chunk (Eq. 5 double loop over 3,120 x 1,560 x 40 heads), cached per setting."""
    key = (head_mode, rho, kind)
    if key not in _ORACLE_CACHE:
        cfg, K, V = _lingbot_chunk()
        _ORACLE_CACHE[key] = oracle.compress(K, V, None, cfg.T, cfg.F, rho, kind, head_mode)
    return _ORACLE_CACHE[key]


@pytest.mark.timeout(600)
@pytest.mark.parametrize("algo", [wk.WK_SCORE_FACTORED, wk.WK_SCORE_GEMM])
@pytest.mark.parametrize("head_mode,rho,kind,n_out", [
    (wk.WK_HEADS_SHARED, 0.5, wk.WK_RATIO_CHUNK, 2340),          # config 2's setting (3 frames -> 1.5)
    (wk.WK_HEADS_SHARED, 0.25, wk.WK_RATIO_NONANCHOR, 2340),     # the same count stated as P = 25 %
    (wk.WK_HEADS_SHARED, 0.75, wk.WK_RATIO_NONANCHOR, 3900),     # config 4's upper ratio
    (wk.WK_HEADS_INDEPENDENT, 0.25, wk.WK_RATIO_NONANCHOR, 2340),
])
def test_lingbot_sized_chunk_full_oracle_compare(head_mode, rho, kind, n_out, algo):
    """Every one of the 3,120 candidate scores (x 40 lists with per-head index sets), the kept-index sets and
    the compacted rows of a LingBot-sized chunk against oracle.compress."""
    cfg, K, V = _lingbot_chunk()
    gi, gK, gV, gs, got = _gpu_compress(cfg, K, V, None, head_mode=head_mode, rho=rho, ratio_kind=kind, score_algo=algo)
    assert got == n_out
    same = _compare_chunk(cfg, K, V, None, gi[0], gK[0], gV[0], gs[0], head_mode, rho, kind, oracle_result=_lingbot_oracle(head_mode, rho, kind))
    print(f"LingBot chunk, head_mode {head_mode}, rho {rho}, algo {algo}: index sets identical to the oracle: {same}")
