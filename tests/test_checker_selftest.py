"""Self-test of the full-size attention checker (tests/wkt.py), CPU only: a correct result (the oracle's
output rounded to bf16, the precision the kernel stores) must pass, and a reference computed on a window
with one 64-key tile missing -- the mistake the absolute 2e-2 / 2e-3 bars cannot see at 28,080 keys --
must fail the scale-aware bars."""
import numpy as np
import pytest
import torch

import oracle
from wkt import (ATT_MAX_ABS_BF16, ATT_MEAN_ABS_BF16, assert_attention_close_bf16)

N_KV = 28080          # the LingBot-shaped window


@pytest.fixture(scope="module")
def window():
    g = torch.Generator().manual_seed(5)
    H, N_q = 2, 48
    Q = torch.randn(H, N_q, 128, generator=g).to(torch.bfloat16)
    K = torch.randn(H, N_KV, 128, generator=g).to(torch.bfloat16)
    V = torch.randn(H, N_KV, 128, generator=g).to(torch.bfloat16)
    ref, lse = oracle.attention(Q, K, V, want_lse=True)
    return Q, K, V, ref, lse


def test_a_correctly_rounded_result_passes(window):
    Q, K, V, ref, lse = window
    got = torch.from_numpy(ref).to(torch.bfloat16)
    assert_attention_close_bf16(got, ref, lse.astype(np.float32), lse, full_size=True)


@pytest.mark.parametrize("tile", [0, 137, N_KV // 64 - 1])
def test_a_lost_key_tile_fails_the_scale_aware_bars_only(window, tile):
    Q, K, V, ref, lse = window
    keep = np.r_[0:64 * tile, 64 * (tile + 1):N_KV]
    wrong, wrong_lse = oracle.attention(Q, K[:, keep].contiguous(), V[:, keep].contiguous(), want_lse=True)
    got = torch.from_numpy(wrong).to(torch.bfloat16)       # what a kernel that skips one tile would return
    err = np.abs(got.float().numpy().astype(np.float64) - ref)
    assert err.max() <= ATT_MAX_ABS_BF16 and err.mean() <= ATT_MEAN_ABS_BF16   # invisible to the absolute bars
    assert_attention_close_bf16(got, ref)                                      # ... so the plain check passes
    with pytest.raises(AssertionError):
        assert_attention_close_bf16(got, ref, full_size=True)
    with pytest.raises(AssertionError):                                        # the log-sum-exp alone gives it away too
        assert_attention_close_bf16(torch.from_numpy(ref).to(torch.bfloat16), ref, wrong_lse, lse, full_size=True)


def test_a_tile_counted_twice_fails(window):
    Q, K, V, ref, lse = window
    idx = np.r_[0:N_KV, 64 * 200:64 * 201]
    wrong = oracle.attention(Q, K[:, idx].contiguous(), V[:, idx].contiguous())
    with pytest.raises(AssertionError):
        assert_attention_close_bf16(torch.from_numpy(wrong).to(torch.bfloat16), ref, full_size=True)
