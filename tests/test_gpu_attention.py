"""GPU parity of wk_attention against the fp64 oracle (attention over the assembled window,
Sec. 4.2 / Sec. 4.3).  Tolerances: fp32 1e-5 max-abs; bf16 2e-2 max-abs and 2e-3 mean-abs."""
import math

import numpy as np
import pytest
import torch

import oracle
import paper_2605_22718_amd as wk
import wk_synth as ws
from wkt import (ATT_MAX_ABS_BF16, ATT_MAX_ABS_F32, ATT_MEAN_ABS_BF16, assert_attention_close_bf16, attention_errors,
                 dev, sample_rows)

pytestmark = pytest.mark.gpu


def _rand(H, Nq, Nkv, dtype, seed, stride=None):
    g = torch.Generator().manual_seed(seed)
    stride = Nkv if stride is None else stride
    Q = torch.randn(H, Nq, 128, generator=g).to(dtype)
    K = torch.randn(H, stride, 128, generator=g).to(dtype)
    V = torch.randn(H, stride, 128, generator=g).to(dtype)
    return Q, K, V


def _workspace(H, N_q, N_kv, dtype):
    n = wk.wk_attention_workspace_bytes(H, N_q, N_kv, wk.WK_BF16 if dtype == torch.bfloat16 else wk.WK_F32)
    return torch.empty(n, dtype=torch.uint8, device=dev()) if n else None


def _run(Q, K, V, N_kv=None, scale=0.0, n_kv_dev=None, want_lse=True, split=True):
    d = dev()
    O = torch.full(Q.shape, float("nan"), dtype=Q.dtype, device=d)
    lse = torch.full(Q.shape[:2], float("nan"), dtype=torch.float32, device=d) if want_lse else None
    nk = None if n_kv_dev is None else torch.tensor([n_kv_dev], dtype=torch.int32, device=d)
    wsb = _workspace(Q.shape[0], Q.shape[1], K.shape[1] if N_kv is None else N_kv, Q.dtype) if split else None
    wk.wk_attention(Q.to(d), K.to(d), V.to(d), O, lse, N_kv=N_kv, scale=scale, n_kv_dev=nk, workspace=wsb)
    torch.cuda.synchronize()
    return O, lse


def _check(Q, K, V, O, lse, N_kv=None, scale=None, rows=None, f32_tol=ATT_MAX_ABS_F32, full_size=False):
    """full_size: also the scale-aware bars (per-row relative error, max-abs against the rows' rms, tight lse)."""
    ref, ref_lse = oracle.attention(Q, K, V, N_kv=N_kv, scale=scale, rows=rows, want_lse=True)
    Og = O if rows is None else O[:, torch.as_tensor(rows, dtype=torch.long)]
    lg = None
    if lse is not None:
        lg = lse.cpu().numpy().astype(np.float64)
        lg = lg if rows is None else lg[:, rows]
    if Q.dtype == torch.float32:
        mx, mean = attention_errors(Og, ref)
        assert mx <= f32_tol, mx
        if lg is not None:
            assert np.abs(lg - ref_lse).max() <= 1e-4
        return mx, mean
    return assert_attention_close_bf16(Og, ref, lg, ref_lse if lg is not None else None, full_size=full_size)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("H,Nq,Nkv", [(2, 200, 300), (1, 1, 1), (3, 129, 64), (2, 33, 65), (1, 257, 127), (2, 300, 333)])
def test_small_shapes_full_compare(dtype, H, Nq, Nkv):
    Q, K, V = _rand(H, Nq, Nkv, dtype, seed=Nq * 1000 + Nkv)
    O, lse = _run(Q, K, V)
    _check(Q, K, V, O, lse)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_rows_past_the_window_are_ignored(dtype):
    Q, K, V = _rand(2, 70, 150, dtype, seed=7, stride=200)
    K[:, 150:] = float("nan")      # must never be read into the result
    V[:, 150:] = float("inf")
    O, lse = _run(Q, K, V, N_kv=150)
    _check(Q, K, V, O, lse, N_kv=150)
    # the device-side length overrides the host bound when smaller
    O2, lse2 = _run(Q, K, V, N_kv=200, n_kv_dev=150)
    assert torch.equal(O2.view(torch.int32 if dtype == torch.float32 else torch.int16),
                       O.view(torch.int32 if dtype == torch.float32 else torch.int16))
    O3, lse3 = _run(Q, K, V, N_kv=200, n_kv_dev=0)
    assert (O3 == 0).all() and torch.isinf(lse3).all() and (lse3 < 0).all()


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_normalisation_and_special_cases(dtype):
    Q, K, V = _rand(2, 100, 500, dtype, seed=11)
    ones = torch.ones_like(V)
    O, _ = _run(Q, K, ones, want_lse=False)
    assert (O.float() - 1).abs().max().item() <= (5e-6 if dtype == torch.float32 else 1e-2)
    # all keys equal: output is the mean of V
    Ke = K[:, :1].expand(-1, K.shape[1], -1).contiguous()
    O, _ = _run(Q, Ke, V, want_lse=False)
    ref = V.double().mean(1, keepdim=True).expand(-1, Q.shape[1], -1).numpy()
    mx, _ = attention_errors(O, ref)
    assert mx <= (1e-5 if dtype == torch.float32 else 2e-2)
    # custom scale; large logits exercise the running-max rescale.  Logits reach ~1e2 here, so the
    # fp32 rounding of the 128-term dot products (~|z| * 2^-23) shows up in exp(z): the fp32 bar is
    # scaled accordingly (the 1e-5 bar is for unit-variance inputs)
    Qb = (Q.float() * 6).to(dtype)
    O, lse = _run(Qb, K, V, scale=0.25)
    _check(Qb, K, V, O, lse, scale=0.25, f32_tol=2e-4)
    # keys sorted by increasing logit for query 0 force a rescale in every tile
    order = torch.argsort((Q[:, :1].float() @ K.float().transpose(1, 2))[:, 0], dim=1)
    Ks = torch.stack([K[h, order[h]] for h in range(K.shape[0])])
    Vs = torch.stack([V[h, order[h]] for h in range(V.shape[0])])
    O, lse = _run(Qb, Ks, Vs)
    _check(Qb, Ks, Vs, O, lse, f32_tol=2e-4)


@pytest.mark.parametrize("H,Nq,Nkv,n_dev", [(1, 64, 4000, None), (2, 300, 2048, None), (1, 33, 4096, 100),
                                            (1, 40, 4096, 0), (3, 257, 1111, 1000)])
def test_split_key_range_matches_oracle_and_unsplit(H, Nq, Nkv, n_dev):
    """Few workgroups and a long window: the key range is split over workgroups and merged."""
    Q, K, V = _rand(H, Nq, Nkv, torch.bfloat16, seed=Nkv + Nq)
    assert (wk.wk_attention_workspace_bytes(H, Nq, Nkv, wk.WK_BF16) > 0) == (Nkv >= 2048)   # shorter: 128-query workgroups
    O, lse = _run(Q, K, V, n_kv_dev=n_dev)
    O1, lse1 = _run(Q, K, V, n_kv_dev=n_dev, split=False)
    if n_dev == 0:
        assert (O == 0).all() and torch.isinf(lse).all() and (O1 == 0).all()
        return
    n_eff = Nkv if n_dev is None else n_dev
    _check(Q, K, V, O, lse, N_kv=n_eff)
    _check(Q, K, V, O1, lse1, N_kv=n_eff)
    assert (O.float() - O1.float()).abs().max().item() <= 4e-3     # same math, different fp32 summation order


@pytest.mark.parametrize("H,Nq,Nkv,n_dev", [(10, 7500, 1000, None), (5, 15000, 520, 500), (12, 2640, 3000, None),
                                            (9, 7400, 700, 64)])
def test_more_items_than_compute_units_with_and_without_workspace(H, Nq, Nkv, n_dev):
    """Grids of more (head, query tile) items than compute units that fill their last round badly, with short
    windows: whatever the library does with the workspace, the result must be that of the plain launch."""
    Q, K, V = _rand(H, Nq, Nkv, torch.bfloat16, seed=Nkv + Nq)
    O, lse = _run(Q, K, V, n_kv_dev=n_dev)
    O1, lse1 = _run(Q, K, V, n_kv_dev=n_dev, split=False)
    assert not torch.isnan(O.float()).any() and not torch.isnan(lse).any()
    assert (O.float() - O1.float()).abs().max().item() <= 4e-3     # same math, different fp32 summation order
    assert (lse - lse1).abs().max().item() <= 2e-3     # row sums of bf16-rounded weights, taken against different running maxima
    rng = np.random.default_rng(Nq)
    rows = sorted(set([0, 255, 256, Nq - 1] + rng.integers(0, Nq, 60).tolist()))
    _check(Q, K, V, O, lse, N_kv=Nkv if n_dev is None else n_dev, rows=rows)


@pytest.mark.parametrize("Nkv", [1024, 1100, 1160, 1217, 1285, 1344, 2049])
def test_eight_wave_loop_every_ring_phase(Nkv):
    """A grid that takes the 256-query workgroups (32 heads x 8 query tiles), windows of 16 .. 33 tiles: the
    hand-scheduled groups of four steps are followed by 3, 1, 2, 3, 0, 0 and 0 left-over steps, the last tile is
    whole or ragged, and every ring position holds the last tile once."""
    H, Nq = 32, 2048
    Q, K, V = _rand(H, Nq, Nkv, torch.bfloat16, seed=7 * Nkv)
    O, lse = _run(Q, K, V, split=False)
    assert not torch.isnan(O.float()).any() and not torch.isnan(lse).any()
    rng = np.random.default_rng(Nkv)
    rows = sorted(set([0, 31, 32, 255, 256, Nq - 1] + rng.integers(0, Nq, 42).tolist()))
    _check(Q, K, V, O, lse, rows=rows, full_size=True)


@pytest.mark.parametrize("case", ["overflow", "underflow", "mixed"])
def test_logits_far_outside_the_range_of_exp2(case):
    """Rows whose logits reach the hundreds, or lie far below zero for every key, or both kinds of row in one
    workgroup: the running maximum must keep every exponent in range."""
    H, Nq, Nkv = 2, 300, 700
    Q, K, V = _rand(H, Nq, Nkv, torch.bfloat16, seed=77)
    if case == "overflow":
        scale = 20.0                                   # logits of several hundred either sign
    elif case == "underflow":
        base = torch.randn(H, 1, 128, generator=torch.Generator().manual_seed(5))
        Q = (base + 0.05 * Q.float()).to(torch.bfloat16)
        K = (-8.0 * base + 0.05 * K.float()).to(torch.bfloat16)
        scale = 0.0                                    # default 1/sqrt(d): every logit near -90
    else:
        scale = 0.0
        Q = Q.clone()
        Q[:, 7] = (Q[:, 7].float() * 300).to(torch.bfloat16)      # one row with huge logits, in two workgroups' tiles
        Q[:, 290] = (Q[:, 290].float() * 300).to(torch.bfloat16)
    for split in (False, True):
        O, lse = _run(Q, K, V, scale=scale, split=split)
        assert not torch.isnan(O.float()).any() and torch.isfinite(lse).all()
        _check(Q, K, V, O, lse, scale=None if scale == 0.0 else scale)


def test_config0_tiny_fp32_full():
    cfg = ws.get_config(0)
    Q = ws.make_queries(cfg)
    K, V = ws.make_native(cfg, n_rows=2640)
    O, lse = _run(Q, K, V)
    mx, mean = _check(Q, K, V, O, lse)
    print(f"config0 fp32: max-abs {mx:.2e} mean-abs {mean:.2e}")


@pytest.mark.parametrize("ci,n_random", [(1, 256), (2, 256), (3, 64)])
def test_full_size_configs_sampled_rows(ci, n_random):
    """Full BASELINE shapes in the launch configuration the benchmark times; the oracle checks the first and
    last row of every 256-query tile plus n_random random rows, of every head, against the contract's
    absolute bars and against the scale-aware ones (a lost or doubled key tile fails those)."""
    cfg = ws.get_config(ci)
    d = dev()
    N_kv = cfg.n_kv_override or (cfg.n_native + cfg.R * wk.wk_keep_count(cfg.rho, cfg.ratio_kind, cfg.anchor_mode,
                                                                         cfg.F, cfg.T)[0])
    assert N_kv == {1: 10560, 2: 28080, 3: 211200}[ci]
    Q = ws.make_queries(cfg, d)
    K, V = ws.make_native(cfg, d, n_rows=N_kv)
    O = torch.empty_like(Q)
    lse = torch.empty(Q.shape[:2], dtype=torch.float32, device=d)
    wsb = _workspace(cfg.H, cfg.N_q, N_kv, Q.dtype)      # config 3 splits the key range, config 1 runs 128-query workgroups, config 2 neither
    assert (wsb is None) == (ci != 3)
    wk.wk_attention(Q, K, V, O, lse, workspace=wsb)
    torch.cuda.synchronize()
    rows = sample_rows(cfg.N_q, 256, n_random, seed=ci)
    mx, mean = _check(Q.cpu(), K.cpu(), V.cpu(), O, lse, rows=rows, full_size=True)
    print(f"config{ci}: {len(rows)} rows/head, max-abs {mx:.2e} mean-abs {mean:.2e}")
    # properties that hold at any size: finite everywhere, V = 1 gives exactly-normalised rows
    assert torch.isfinite(O.float()).all()
    if ci != 3:
        wk.wk_attention(Q, K, torch.ones_like(V), O, None, workspace=wsb)
        assert (O.float() - 1).abs().max().item() <= 1e-2
