"""GPU parity of wk_attention_block_causal (frame-level causal mask inside the denoising chunk, an option
beside the paper's unmasked window attention) against the oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2605_22718_amd as wk
import wk_synth as ws
from wkt import (ATT_MAX_ABS_BF16, ATT_MAX_ABS_F32, ATT_MEAN_ABS_BF16, assert_attention_close_bf16, attention_errors,
                 dev, sample_rows)

pytestmark = pytest.mark.gpu


def _run(Q, K, V, row0, T, N_kv=None, n_kv_dev=None):
    d = dev()
    H, N_q, _ = Q.shape
    O = torch.full(Q.shape, float("nan"), dtype=Q.dtype, device=d)
    lse = torch.full((H, N_q), float("nan"), dtype=torch.float32, device=d)
    wsb = torch.empty(wk.wk_attention_block_causal_workspace_bytes(H, N_q), dtype=torch.uint8, device=d)
    nk = None if n_kv_dev is None else torch.tensor([n_kv_dev], dtype=torch.int32, device=d)
    wk.wk_attention_block_causal(Q.to(d), K.to(d), V.to(d), O, row0, T, wsb, lse=lse, N_kv=N_kv, n_kv_dev=nk)
    torch.cuda.synchronize()
    return O, lse


def _check(Q, O, lse, ref, ref_lse, full_size=False):
    if full_size:
        return assert_attention_close_bf16(O, ref, lse, ref_lse, full_size=True)[0]
    mx, mean = attention_errors(O, ref)
    err_l = np.abs(lse.cpu().numpy().astype(np.float64) - ref_lse).max()
    if Q.dtype == torch.float32:
        assert mx <= ATT_MAX_ABS_F32 and err_l <= 1e-4, (mx, err_l)
    else:
        assert mx <= ATT_MAX_ABS_BF16 and mean <= ATT_MEAN_ABS_BF16 and err_l <= 2e-2, (mx, mean, err_l)
    return mx


@pytest.mark.parametrize("index", [0, 1])
@pytest.mark.parametrize("T,F,n_before,n_after", [
    (130, 3, 0, 700),      # chunk first in the window
    (130, 3, 517, 333),    # chunk in the middle (ring slot of the window manager), ragged everywhere
    (130, 3, 517, 0),      # chunk last: nothing behind it
    (64, 4, 256, 128),     # everything tile-aligned
    (1, 5, 40, 9),         # one-token frames: a plain causal mask inside the chunk
    (300, 1, 100, 100),    # one frame: the mask hides nothing
])
def test_block_causal_matches_oracle(index, T, F, n_before, n_after):
    cfg = ws.get_config(index).with_(H=2)
    N_q = T * F
    N_kv = n_before + N_q + n_after
    Q = ws.make_queries(cfg, "cpu", N_q)
    K, V = ws.make_native(cfg, "cpu", N_kv)
    O, lse = _run(Q, K, V, n_before, T)
    ref, ref_lse = oracle.attention_block_causal(Q, K, V, n_before, T, want_lse=True)
    _check(Q, O, lse, ref, ref_lse)
    if F == 1:   # then it is plain attention
        mx, _ = attention_errors(O, oracle.attention(Q, K, V))
        assert mx <= (ATT_MAX_ABS_F32 if Q.dtype == torch.float32 else ATT_MAX_ABS_BF16)


def test_block_causal_with_device_side_window_length_and_stride():
    cfg = ws.get_config(1).with_(H=3)
    T, F, row0 = 100, 3, 64
    N_q = T * F
    Q = ws.make_queries(cfg, "cpu", N_q)
    K, V = ws.make_native(cfg, "cpu", 1000)           # stride 1000, capacity passed 900, 777 rows valid
    O, lse = _run(Q, K, V, row0, T, N_kv=900, n_kv_dev=777)
    ref, ref_lse = oracle.attention_block_causal(Q, K, V, row0, T, N_kv=777, want_lse=True)
    _check(Q, O, lse, ref, ref_lse)
    # the window ends exactly behind the chunk
    O, lse = _run(Q, K, V, row0, T, N_kv=900, n_kv_dev=row0 + N_q)
    ref, ref_lse = oracle.attention_block_causal(Q, K, V, row0, T, N_kv=row0 + N_q, want_lse=True)
    _check(Q, O, lse, ref, ref_lse)


def test_block_causal_config2_size_sampled_rows():
    """LingBot shape in the window manager's layout: sink chunk, ring (the chunk being denoised in ring
    slot 0, the recent chunk behind it), then 8 retrieved slots."""
    d = dev()
    cfg = ws.get_config(2)
    T, F = cfg.T, 3
    N_q = T * F
    row0 = N_q                                       # behind the sink chunk
    N_kv = 3 * N_q + 8 * 2340
    Q = ws.make_queries(cfg, d)
    K, V = ws.make_native(cfg, d, N_kv)
    O, lse = _run(Q, K, V, row0, T)
    rows = np.unique(np.concatenate([sample_rows(N_q, 256, 64, seed=4), np.array([T - 1, T, 2 * T - 1, 2 * T], np.int32)]))
    ref, ref_lse = oracle.attention_block_causal(Q.cpu(), K.cpu(), V.cpu(), row0, T, rows=rows, want_lse=True)
    sel = torch.as_tensor(rows, dtype=torch.long)
    mx = _check(Q, O[:, sel], lse[:, sel], ref, ref_lse, full_size=True)
    print(f"block-causal config-2 size: max-abs {mx:.2e} on {rows.size} rows x {cfg.H} heads")
    assert torch.isfinite(O.float()).all()


def test_block_causal_many_frames_uses_separate_launches():
    """More frames than the one-grid table holds (9 > 7): the per-range launches give the same answer."""
    cfg = ws.get_config(1).with_(H=2)
    T, F, row0 = 40, 9, 100
    Q = ws.make_queries(cfg, "cpu", T * F)
    K, V = ws.make_native(cfg, "cpu", row0 + T * F + 150)
    O, lse = _run(Q, K, V, row0, T)
    ref, ref_lse = oracle.attention_block_causal(Q, K, V, row0, T, want_lse=True)
    _check(Q, O, lse, ref, ref_lse)
