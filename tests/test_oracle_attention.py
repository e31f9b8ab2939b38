"""Pins for the oracle's window assembly and attention (Sec. 4.2, Sec. 4.3) -- CPU only."""
import math

import numpy as np
import pytest
import torch

import oracle
import wk_synth as ws


def _small(seed=0, H=3, Nq=17, Nkv=45, d=16, dtype=torch.float32):
    g = torch.Generator().manual_seed(seed)
    Q = torch.randn(H, Nq, d, generator=g).to(dtype)
    K = torch.randn(H, Nkv, d, generator=g).to(dtype)
    V = torch.randn(H, Nkv, d, generator=g).to(dtype)
    return Q, K, V


def test_hand_value():
    # d = 1, scale 1: logits 0 and ln 3 give weights 1/4 and 3/4; values 0 and 4 give 3
    Q = torch.tensor([[[1.0]]])
    K = torch.tensor([[[0.0], [math.log(3.0)]]])
    V = torch.tensor([[[0.0], [4.0]]])
    O, lse = oracle.attention(Q, K, V, scale=1.0, want_lse=True)
    assert abs(O[0, 0, 0] - 3.0) < 1e-6      # float32 rounding of ln 3 in the input
    assert abs(lse[0, 0] - math.log(4.0)) < 1e-6
    # default scale is 1/sqrt(d)
    Q4 = torch.tensor([[[2.0, 0, 0, 0]]])
    K4 = torch.tensor([[[0.0, 0, 0, 0], [math.log(3.0), 9, 9, 9]]])
    V4 = torch.tensor([[[0.0, 1, 0, 0], [4.0, 1, 0, 8]]])
    O = oracle.attention(Q4, K4, V4)   # logit = 2*ln3/2 = ln 3
    np.testing.assert_allclose(O[0, 0], [3.0, 1.0, 0.0, 6.0], atol=1e-6)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_against_library_softmax_matmul(dtype):
    Q, K, V = _small(1, dtype=dtype)
    O, lse = oracle.attention(Q, K, V, want_lse=True)
    z = torch.einsum("hqd,hkd->hqk", Q.double(), K.double()) / math.sqrt(Q.shape[-1])
    ref = torch.softmax(z, -1) @ V.double()
    np.testing.assert_allclose(O, ref.numpy(), rtol=0, atol=1e-13)
    np.testing.assert_allclose(lse, torch.logsumexp(z, -1).numpy(), rtol=0, atol=1e-13)
    # rows of the softmax sum to one: exp(z - lse) sums to 1
    assert np.abs(np.exp(z.numpy() - lse[..., None]).sum(-1) - 1).max() < 1e-13
    # q and k are not swapped and V is not transposed: a non-square case with a custom scale
    O2 = oracle.attention(Q, K, V, scale=0.37)
    ref2 = torch.softmax(torch.einsum("hqd,hkd->hqk", Q.double(), K.double()) * 0.37, -1) @ V.double()
    np.testing.assert_allclose(O2, ref2.numpy(), rtol=0, atol=1e-13)


def test_bf16_inputs_are_widened_exactly():
    Q, K, V = _small(2, dtype=torch.bfloat16)
    a = oracle.attention(Q, K, V)
    b = oracle.attention(Q.float(), K.float(), V.float())
    np.testing.assert_array_equal(a, b)


def test_normalisation_cases():
    Q, K, V = _small(3)
    ones = torch.ones_like(V)
    np.testing.assert_allclose(oracle.attention(Q, K, ones), 1.0, atol=1e-14)
    # V = indicator of a key subset: the output is that subset's attention mass
    sub = torch.zeros_like(V)
    sub[:, 5:20] = 1.0
    z = torch.einsum("hqd,hkd->hqk", Q.double(), K.double()) / math.sqrt(Q.shape[-1])
    mass = torch.softmax(z, -1)[:, :, 5:20].sum(-1)
    np.testing.assert_allclose(oracle.attention(Q, K, sub)[..., 0], mass.numpy(), atol=1e-13)


def test_special_cases():
    Q, K, V = _small(4)
    # one key: the output is its value
    O = oracle.attention(Q, K[:, :1].contiguous(), V[:, :1].contiguous())
    np.testing.assert_allclose(O, V[:, :1].double().expand(-1, Q.shape[1], -1).numpy(), atol=1e-15)
    # all keys equal: uniform weights, output = mean of V
    Ke = K[:, :1].expand(-1, K.shape[1], -1).contiguous()
    np.testing.assert_allclose(oracle.attention(Q, Ke, V),
                               V.double().mean(1, keepdim=True).expand(-1, Q.shape[1], -1).numpy(), atol=1e-13)
    # adding a constant vector to every key shifts each row's logits by a constant
    K = (K * 64).round() / 64        # multiples of 2**-6, so that K + c is exact in float32
    base = oracle.attention(Q, K, V)
    c = torch.tensor([0.5, -1.0] * (K.shape[-1] // 2))
    np.testing.assert_allclose(oracle.attention(Q, (K + c).contiguous(), V), base, atol=1e-12)
    # duplicating the whole window changes nothing
    np.testing.assert_allclose(oracle.attention(Q, torch.cat([K, K], 1), torch.cat([V, V], 1)), base, atol=1e-13)
    # permuting keys together with values changes nothing
    perm = torch.randperm(K.shape[1], generator=torch.Generator().manual_seed(0))
    np.testing.assert_allclose(oracle.attention(Q, K[:, perm].contiguous(), V[:, perm].contiguous()), base, atol=1e-13)


def test_row_stride_and_row_subset():
    Q, K, V = _small(5)
    base = oracle.attention(Q, K, V)
    pad = torch.full((K.shape[0], 11, K.shape[2]), 1e4)
    Kp, Vp = torch.cat([K, pad], 1), torch.cat([V, pad], 1)
    np.testing.assert_array_equal(oracle.attention(Q, Kp, Vp, N_kv=K.shape[1]), base)
    rows = np.array([0, 16, 3, 3], np.int32)
    np.testing.assert_array_equal(oracle.attention(Q, K, V, rows=rows), base[:, rows])


def test_gather_is_verbatim_and_ordered():
    cfg = ws.get_config(1).with_(H=2, T=8, d=16)
    Kn, Vn = ws.make_native(cfg, n_rows=10)
    store_k, store_v = [], []
    for c, n in enumerate([5, 7, 3, 6]):
        k, v = ws.make_native(cfg.with_(index=10 + c), n_rows=n)
        store_k.append(k)
        store_v.append(v)
    ids = [2, 0, 3]
    Kw, Vw, n_win = oracle.gather(store_k, store_v, ids, Kn, Vn, win_capacity=40)
    assert n_win == 10 + 3 + 5 + 6
    expect_k = torch.cat([Kn] + [store_k[i] for i in ids], 1)
    expect_v = torch.cat([Vn] + [store_v[i] for i in ids], 1)
    assert torch.equal(Kw[:, :n_win].view(torch.int16), expect_k.view(torch.int16))
    assert torch.equal(Vw[:, :n_win].view(torch.int16), expect_v.view(torch.int16))
    assert (Kw[:, n_win:] == 0).all()
    # nothing retrieved: the window is the native frames
    Kw0, Vw0, n0 = oracle.gather(store_k, store_v, [], Kn, Vn, win_capacity=40)
    assert n0 == 10 and torch.equal(Kw0[:, :10], Kn) and torch.equal(Vw0[:, :10], Vn)
    with pytest.raises(ValueError):
        oracle.gather(store_k, store_v, [0, 1, 2, 3], Kn, Vn, win_capacity=20)


def test_retrieving_nothing_is_sliding_window_attention():
    cfg = ws.get_config(0).with_(H=2, T=12, d=16)
    Q = ws.make_queries(cfg)
    Kn, Vn = ws.make_native(cfg)
    Kc, Vc, _ = ws.make_chunk(cfg, 0)
    Kw, Vw, n_win = oracle.gather([Kc], [Vc], [], Kn, Vn, win_capacity=cfg.n_native + 30)
    a = oracle.attention(Q, Kw, Vw, N_kv=n_win)
    b = oracle.attention(Q, Kn, Vn)
    np.testing.assert_array_equal(a, b)


def test_retrieving_everything_uncompressed_is_full_kv_attention():
    cfg = ws.get_config(1).with_(H=2, T=10, d=16, M=5)
    Q = ws.make_queries(cfg)
    Kn, Vn = ws.make_native(cfg)
    chunks = [ws.make_chunk(cfg, c) for c in range(cfg.M)]
    comp = [oracle.compress(K, V, None, cfg.T, cfg.F, 1.0) for K, V, _ in chunks]   # rho = 1: nothing pruned
    store_k = [c[1] for c in comp]
    store_v = [c[2] for c in comp]
    poses, cur = ws.make_poses(cfg.M, cfg.seed)
    ids, _, _ = oracle.score_chunks(poses, cur, cfg.M)     # retrieve every chunk, in relevance order
    assert sorted(ids) == list(range(cfg.M))
    cap = cfg.n_native + cfg.M * cfg.chunk_tokens
    Kw, Vw, n_win = oracle.gather(store_k, store_v, ids, Kn, Vn, cap)
    assert n_win == cap
    got = oracle.attention(Q, Kw, Vw, N_kv=n_win)
    K_full = torch.cat([Kn] + [c[0] for c in chunks], 1)    # history in generation order
    V_full = torch.cat([Vn] + [c[1] for c in chunks], 1)
    np.testing.assert_allclose(got, oracle.attention(Q, K_full, V_full), rtol=0, atol=1e-13)


# ---- frame-level causal mask inside the denoising chunk (an option; the paper states no mask) ----

def _bc_setup(seed, H=2, T=5, F=3, n_before=7, n_after=9, d=16):
    g = torch.Generator().manual_seed(seed)
    N_q = F * T
    N_kv = n_before + N_q + n_after
    Q = torch.randn(H, N_q, d, generator=g)
    K = torch.randn(H, N_kv, d, generator=g)
    V = torch.randn(H, N_kv, d, generator=g)
    return Q, K, V, n_before, T, F


def test_block_causal_against_library_masked_softmax():
    for seed, (nb, na) in enumerate([(7, 9), (0, 9), (7, 0), (0, 0)]):
        Q, K, V, row0, T, F = _bc_setup(seed, n_before=nb, n_after=na)
        H, N_q, d = Q.shape
        N_kv = K.shape[1]
        O, lse = oracle.attention_block_causal(Q, K, V, row0, T, want_lse=True)
        z = torch.einsum("hqd,hkd->hqk", Q.double(), K.double()) / math.sqrt(d)
        qf = (torch.arange(N_q) // T).view(N_q, 1)
        kpos = torch.arange(N_kv).view(1, N_kv)
        inside = (kpos >= row0) & (kpos < row0 + N_q)
        hidden = inside & (((kpos - row0) // T) > qf)
        z = z.masked_fill(hidden.unsqueeze(0), float("-inf"))
        ref = torch.softmax(z, -1) @ V.double()
        np.testing.assert_allclose(O, ref.numpy(), atol=1e-13)
        np.testing.assert_allclose(lse, torch.logsumexp(z, -1).numpy(), atol=1e-13)
        # the count of visible keys per query frame: everything but the later frames of its own chunk
        vis = (~hidden).sum(1)
        assert vis.tolist() == [N_kv - (F - 1 - int(f)) * T for f in qf.view(-1)]


def test_block_causal_reduces_to_plain_attention_on_reduced_windows():
    Q, K, V, row0, T, F = _bc_setup(5)
    N_q = F * T
    O = oracle.attention_block_causal(Q, K, V, row0, T)
    for f in range(F):
        rows = np.arange(f * T, (f + 1) * T)
        # frame f sees the window with the later frames of the chunk cut out
        keep = [n for n in range(K.shape[1]) if not (row0 + (f + 1) * T <= n < row0 + N_q)]
        ref = oracle.attention(Q, K[:, keep].contiguous(), V[:, keep].contiguous(), rows=rows)
        np.testing.assert_allclose(O[:, rows], ref, atol=1e-13)
    # the last frame sees everything: plain attention
    last = np.arange((F - 1) * T, N_q)
    np.testing.assert_allclose(O[:, last], oracle.attention(Q, K, V, rows=last), atol=1e-13)
    # one frame per chunk: the mask hides nothing
    np.testing.assert_allclose(oracle.attention_block_causal(Q, K, V, row0, N_q), oracle.attention(Q, K, V), atol=1e-13)
    # frames of one token: a plain causal mask inside the chunk; the first query sees exactly one chunk key
    Qs, Ks, Vs = Q[:, :4].contiguous(), K[:, :4].contiguous(), V[:, :4].contiguous()
    O1 = oracle.attention_block_causal(Qs, Ks, Vs, 0, 1)
    np.testing.assert_allclose(O1[:, 0], Vs[:, 0].double().numpy(), atol=1e-13)
    # row subsets and lse agree with the full call
    sub = np.array([0, 4, 5, 14], np.int32)
    Os, ls = oracle.attention_block_causal(Q, K, V, row0, T, rows=sub, want_lse=True)
    Of, lf = oracle.attention_block_causal(Q, K, V, row0, T, want_lse=True)
    np.testing.assert_allclose(Os, Of[:, sub], atol=0)
    np.testing.assert_allclose(ls, lf[:, sub], atol=0)
    with pytest.raises(ValueError):
        oracle.attention_block_causal(Q, K, V, row0, 4)            # N_q not a multiple of the frame
    with pytest.raises(ValueError):
        oracle.attention_block_causal(Q, K, V, K.shape[1] - 3, T)  # chunk rows run past the window
