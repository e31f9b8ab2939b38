"""Pins for the oracle's World Compression (Sec. 4.3, Eq. 5) -- CPU only.

The oracle evaluates Eq. 5 as a literal double sum.  It is pinned here by hand
values, by the algebraic collapse of Eq. 5 (mean cosine = dot with the mean of
the normalised anchors), by a normalised-matrix product in numpy, by the
symmetries of the cosine, by brute-force selection on tiny inputs, and by the
token counts the paper prints.
"""
import itertools
import os

import numpy as np
import pytest
import torch

import oracle
import wk_synth as ws

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    out = []
    for line in open(os.path.join(GOLD, name)):
        line = line.strip()
        if line and not line.startswith("#"):
            out.append([float(x) for x in line.split()])
    return out


def test_eq5_hand_values():
    rows = _rows("eq5_hand.txt")
    anchors = torch.tensor([[1.0, 0.0], [0.0, 1.0]])
    cand = torch.tensor([[r[0], r[1]] for r in rows])
    K = torch.cat([anchors, cand, torch.ones(2 - len(rows) % 2, 2)], 0)  # pad to F*T with T=2
    n_tok = K.shape[0]
    assert n_tok % 2 == 0
    s = oracle.compress_scores(K.view(1, n_tok, 2).contiguous(), None, T=2, F=n_tok // 2)
    for j, r in enumerate(rows):
        assert abs(s[0, j] - r[2]) < 1e-15, (j, s[0, j], r[2])


def _factored(K64, T, first_cand):
    """s_j = khat_j . mean_i khat_i -- the algebraic collapse of Eq. 5."""
    a = K64[:T]
    c = K64[first_cand:]
    m = (a / np.linalg.norm(a, axis=1, keepdims=True)).mean(0)
    return (c / np.linalg.norm(c, axis=1, keepdims=True)) @ m


@pytest.mark.parametrize("head_mode", [oracle.HEADS_SHARED, oracle.HEADS_INDEPENDENT])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_eq5_equals_factored_and_matrix_forms(head_mode, dtype):
    H, T, F, d = 3, 37, 3, 16
    g = torch.Generator().manual_seed(5)
    K = torch.randn(H, F * T, d, generator=g).to(dtype)
    s = oracle.compress_scores(K, None, T, F, head_mode)
    K64 = K.double().numpy()
    if head_mode == oracle.HEADS_SHARED:
        groups = [np.concatenate([K64[h] for h in range(H)], axis=1)]
    else:
        groups = [K64[h] for h in range(H)]
    assert s.shape == (len(groups), (F - 1) * T)
    for gi, Kg in enumerate(groups):
        np.testing.assert_allclose(s[gi], _factored(Kg, T, T), rtol=0, atol=1e-12)
        kn = Kg / np.linalg.norm(Kg, axis=1, keepdims=True)
        cosmat = kn[T:] @ kn[:T].T            # [N_c][T] matrix of cosines
        np.testing.assert_allclose(s[gi], cosmat.mean(1), rtol=0, atol=1e-12)


def test_eq5_external_anchor_matches_first_frame():
    """A chunk [anchor | rest] scored with its first frame as anchor equals the rest scored
    against the same anchor passed separately."""
    H, T, F, d = 2, 19, 3, 8
    g = torch.Generator().manual_seed(6)
    K = torch.randn(H, F * T, d, generator=g)
    s_first = oracle.compress_scores(K, None, T, F)
    rest = K[:, T:].contiguous()
    anchor = K[:, :T].contiguous()
    # the external-anchor form treats all F' * T tokens of `rest` as candidates
    s_ext = oracle.compress_scores(rest, anchor, T, F - 1, anchor_mode=oracle.ANCHOR_EXTERNAL)
    np.testing.assert_allclose(s_first, s_ext, rtol=0, atol=1e-15)


def test_eq5_symmetries():
    H, T, F, d = 1, 11, 2, 6
    g = torch.Generator().manual_seed(7)
    K = torch.randn(H, F * T, d, generator=g, dtype=torch.float64).float()
    s0 = oracle.compress_scores(K, None, T, F)
    # positive scaling of any key leaves every score unchanged (powers of two keep it exact)
    K2 = K.clone()
    K2[0, 3] *= 4.0      # an anchor
    K2[0, T + 2] *= 0.25  # a candidate
    np.testing.assert_allclose(oracle.compress_scores(K2, None, T, F), s0, rtol=0, atol=1e-14)
    # negating a candidate flips the sign of its score only
    K3 = K.clone()
    K3[0, T + 5] *= -1.0
    s3 = oracle.compress_scores(K3, None, T, F)
    assert abs(s3[0, 5] + s0[0, 5]) < 1e-15
    mask = np.ones(T, bool)
    mask[5] = False
    np.testing.assert_array_equal(s3[0, mask], s0[0, mask])
    # all anchors equal to u: s_j = cos(k_j, u)
    u = torch.tensor([1.0, 2.0, -1.0, 0.5, 0.0, 3.0])
    K4 = K.clone()
    K4[0, :T] = u
    s4 = oracle.compress_scores(K4, None, T, F)
    c = K4[0, T:].double().numpy()
    expect = (c @ u.double().numpy()) / (np.linalg.norm(c, axis=1) * np.linalg.norm(u.double().numpy()))
    np.testing.assert_allclose(s4[0], expect, rtol=0, atol=1e-14)
    # a candidate equal to every anchor scores exactly 1 (up to rounding)
    K4[0, T + 1] = u * 2.0
    assert abs(oracle.compress_scores(K4, None, T, F)[0, 1] - 1.0) < 1e-15


def test_zero_norm_key_scores_zero():
    K = torch.ones(1, 4, 3)
    K[0, 2] = 0.0   # a zero candidate
    s = oracle.compress_scores(K, None, T=2, F=2)
    assert s[0, 0] == 0.0 and abs(s[0, 1] - 1.0) < 1e-15
    K[0, 0] = 0.0   # a zero anchor contributes 0 to the mean
    s = oracle.compress_scores(K, None, T=2, F=2)
    assert abs(s[0, 1] - 0.5) < 1e-15


def test_select_lowest_brute_force_all_tie_patterns():
    for n in range(0, 7):
        for vals in itertools.product([0.0, 1.0, 2.0], repeat=n):
            for k in range(0, n + 1):
                got = oracle.select_lowest(np.array(vals), k)
                # brute force: rank by (value, index), keep k, report ascending
                order = sorted(range(n), key=lambda i: (vals[i], i))[:k]
                assert list(got) == sorted(order), (vals, k, got)


def test_select_lowest_random_against_numpy():
    rng = np.random.default_rng(3)
    for n, k in [(64, 16), (1, 1), (100, 0), (257, 256), (1000, 250)]:
        s = rng.standard_normal(n).round(1)  # many ties
        got = oracle.select_lowest(s, k)
        order = np.lexsort((np.arange(n), s))[:k]
        np.testing.assert_array_equal(got, np.sort(order))


def test_keep_counts_printed_by_the_paper():
    for T, F, P, expect in _rows("counts.txt"):
        n_out, n_keep = oracle.keep_count(P, oracle.RATIO_NONANCHOR, oracle.ANCHOR_FIRST_FRAME, int(F), int(T))
        assert n_out == int(expect) and n_keep == n_out - int(T)
    # whole-chunk ratio 0.5 is the same point as P = 25% for F = 3
    for T in (880, 1560):
        assert oracle.keep_count(0.5, oracle.RATIO_CHUNK, oracle.ANCHOR_FIRST_FRAME, 3, T) == (3 * T // 2, T // 2)
    # one-frame chunk against an external anchor: every token is a candidate
    assert oracle.keep_count(0.5, oracle.RATIO_CHUNK, oracle.ANCHOR_EXTERNAL, 1, 880) == (440, 440)
    # window bookkeeping of Sec. 5.1: 3 + 9 + 3 + 3 = 18 frames, the 9 retrieved frames hold 6 compressed chunks
    n_out, _ = oracle.keep_count(0.25, oracle.RATIO_NONANCHOR, oracle.ANCHOR_FIRST_FRAME, 3, 880)
    assert 6 * n_out == 9 * 880 and 3 + 9 + 3 + 3 == 18
    # a whole-chunk ratio below the anchor frame is rejected
    with pytest.raises(ValueError):
        oracle.keep_count(0.25, oracle.RATIO_CHUNK, oracle.ANCHOR_FIRST_FRAME, 3, 1560)
    with pytest.raises(ValueError):
        oracle.keep_count(1.5, oracle.RATIO_NONANCHOR, oracle.ANCHOR_FIRST_FRAME, 3, 1560)
    # rounding: half away from zero
    assert oracle.keep_count(0.5, oracle.RATIO_NONANCHOR, oracle.ANCHOR_FIRST_FRAME, 2, 5)[1] == 3


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_rho_one_is_identity(dtype):
    cfg = ws.get_config(1).with_(H=2, T=24, d=16)
    K, V, _ = ws.make_chunk(cfg, 0)
    K, V = K.to(dtype), V.to(dtype)
    idx, Ko, Vo, _ = oracle.compress(K, V, None, cfg.T, cfg.F, 1.0)
    np.testing.assert_array_equal(idx[0], np.arange(cfg.F * cfg.T))
    assert torch.equal(Ko.view(torch.uint8), K.view(torch.uint8))
    assert torch.equal(Vo.view(torch.uint8), V.view(torch.uint8))


def test_keeps_the_least_similar_tokens():
    """All anchors equal u.  Candidates equal to -u (score -1) are kept before orthogonal ones
    (score 0), and copies of u (score 1) are dropped first: 'retain the bottom P%'."""
    T, F, d = 4, 3, 4
    u = torch.tensor([1.0, 0, 0, 0])
    w = torch.tensor([0.0, 1.0, 0, 0])
    K = torch.zeros(1, F * T, d)
    K[0, :T] = u
    kinds = [u, -u, w, u, -u, w, u, w]  # candidates 0..7
    for j, k in enumerate(kinds):
        K[0, T + j] = k
    V = torch.arange(F * T * d, dtype=torch.float32).view(1, F * T, d)
    idx, Ko, Vo, s = oracle.compress(K, V, None, T, F, 0.5, oracle.RATIO_NONANCHOR)
    np.testing.assert_allclose(s[0], [1, -1, 0, 1, -1, 0, 1, 0], atol=1e-15)
    # n_keep = 4: both -u tokens (1, 4) then the two lowest-index orthogonal ones (2, 5)
    np.testing.assert_array_equal(idx[0], [0, 1, 2, 3, T + 1, T + 2, T + 4, T + 5])
    assert torch.equal(Ko[0], K[0, idx[0]]) and torch.equal(Vo[0], V[0, idx[0]])
    # anchor only (3 -> 1.0)
    idx, Ko, _, _ = oracle.compress(K, V, None, T, F, 0.0, oracle.RATIO_NONANCHOR)
    np.testing.assert_array_equal(idx[0], np.arange(T))


def test_head_modes_agree_on_reshaped_input():
    """Head-shared scoring of [H][N][d] is per-head scoring of the single 'head' [1][N][H*d]."""
    H, T, F, d = 4, 13, 3, 8
    g = torch.Generator().manual_seed(11)
    K = torch.randn(H, F * T, d, generator=g)
    V = torch.randn(H, F * T, d, generator=g)
    Kcat = K.permute(1, 0, 2).reshape(1, F * T, H * d).contiguous()
    Vcat = V.permute(1, 0, 2).reshape(1, F * T, H * d).contiguous()
    i_sh, Ko, Vo, s_sh = oracle.compress(K, V, None, T, F, 0.5)
    i_in, Kc, Vc, s_in = oracle.compress(Kcat, Vcat, None, T, F, 0.5, head_mode=oracle.HEADS_INDEPENDENT)
    np.testing.assert_allclose(s_sh, s_in, rtol=0, atol=1e-15)
    np.testing.assert_array_equal(i_sh, i_in)
    assert torch.equal(Ko.permute(1, 0, 2).reshape(1, -1, H * d), Kc)
    assert torch.equal(Vo.permute(1, 0, 2).reshape(1, -1, H * d), Vc)
    # per-head mode: each head's list is that head alone
    i_h, Kh, _, s_h = oracle.compress(K, V, None, T, F, 0.5, head_mode=oracle.HEADS_INDEPENDENT)
    for h in range(H):
        i1, K1, _, s1 = oracle.compress(K[h:h + 1].contiguous(), V[h:h + 1].contiguous(), None, T, F, 0.5)
        np.testing.assert_array_equal(i_h[h], i1[0])
        np.testing.assert_array_equal(s_h[h], s1[0])
        assert torch.equal(Kh[h], K1[0])


def test_generator_copies_score_higher_on_average():
    """Sanity of the synthetic redundancy: tokens copied from the anchor have a higher mean
    Eq. 5 score than fresh ones (the shift is about 1/T, see the input recipe)."""
    cfg = ws.get_config(1).with_(H=2, T=64, d=32)
    K, V, _ = ws.make_chunk(cfg, 1)
    s = oracle.compress_scores(K, None, cfg.T, cfg.F)[0]
    # copied tokens are those nearly equal to the anchor token at the same in-frame position
    Kd = K.double()
    anchor = Kd[:, :cfg.T]
    copied = []
    for f in range(1, cfg.F):
        diff = (Kd[:, f * cfg.T:(f + 1) * cfg.T] - anchor).abs().amax(dim=(0, 2))
        copied.append(diff < 0.5)
    copied = torch.cat(copied).numpy()
    assert 0.3 < copied.mean() < 0.7
    assert s[copied].mean() > s[~copied].mean()
