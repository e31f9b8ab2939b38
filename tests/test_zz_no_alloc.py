"""wk_compress_chunk_noalloc (the entry point for callers that cannot allocate) against
wk_compress_chunk: same kernels on the library's built-in scratch array instead of a caller's
workspace, so index lists and compacted rows must be bit-identical.  Two calls in a row, the second on
a smaller input, so that the second runs over what the first left in the array."""
import pytest
import torch

import paper_2605_22718_amd as wk
import wk_synth as ws
from wkt import bits, dev

pytestmark = pytest.mark.gpu


def _both(cfg, chunk_id, rho, kind, head_mode, algo):
    d = dev()
    K, V, A = ws.make_chunk(cfg, chunk_id, d)
    desc = wk.make_compress_desc(cfg.H, cfg.T, cfg.F, cfg.dtype, rho, head_mode=head_mode,
                                 anchor_mode=cfg.anchor_mode, ratio_kind=kind, score_algo=algo)
    n_out, _ = wk.wk_keep_count(rho, kind, cfg.anchor_mode, cfg.F, cfg.T)
    G = cfg.H if head_mode == wk.WK_HEADS_INDEPENDENT else 1
    need = wk.wk_compress_workspace_bytes(desc)
    assert 0 < need <= wk.wk_compress_scratch_bytes()
    out = []
    for noalloc in (False, True):
        idx = torch.full((1, G, n_out), -7, dtype=torch.int32, device=d)
        Ko = torch.zeros((cfg.H, n_out, cfg.d), dtype=K.dtype, device=d)
        Vo = torch.zeros_like(Ko)
        if noalloc:
            got = wk.wk_compress_chunk_noalloc(desc, K, V, A, idx, Ko, Vo)
        else:
            wsb = torch.zeros(need, dtype=torch.uint8, device=d)
            got = wk.wk_compress_chunk(desc, K, V, A, idx, Ko, Vo, wsb)
        torch.cuda.synchronize()
        assert got == n_out
        out.append((idx.cpu(), Ko.cpu(), Vo.cpu()))
    (i0, k0, v0), (i1, k1, v1) = out
    assert torch.equal(i0, i1), "index lists differ"
    assert torch.equal(bits(k0), bits(k1)) and torch.equal(bits(v0), bits(v1)), "compacted rows differ"
    return n_out


@pytest.mark.parametrize("head_mode,algo", [(wk.WK_HEADS_SHARED, wk.WK_SCORE_FACTORED),
                                            (wk.WK_HEADS_INDEPENDENT, wk.WK_SCORE_FACTORED),
                                            (wk.WK_HEADS_SHARED, wk.WK_SCORE_GEMM)])
def test_two_calls_in_a_row_second_smaller(head_mode, algo):
    big = ws.get_config(2)                               # LingBot-sized chunk: 40 heads, 3 x 1,560 tokens
    small = ws.get_config(1).with_(H=5, T=130, F=2)
    assert _both(big, 0, 0.5, wk.WK_RATIO_CHUNK, head_mode, algo) == 2340
    _both(small, 1, 0.25, wk.WK_RATIO_NONANCHOR, head_mode, algo)


def test_external_anchor_fp32_then_smaller():
    cfg = ws.get_config(0)                               # one-frame fp32 chunks against an external anchor
    assert _both(cfg, 0, cfg.rho, cfg.ratio_kind, wk.WK_HEADS_SHARED, wk.WK_SCORE_FACTORED) == 440
    _both(cfg.with_(H=2, T=70), 1, cfg.rho, cfg.ratio_kind, wk.WK_HEADS_INDEPENDENT, wk.WK_SCORE_FACTORED)


def test_request_beyond_the_built_in_scratch_is_refused():
    d = dev()
    cfg = ws.get_config(4)
    desc = wk.make_compress_desc(cfg.H, cfg.T, cfg.F, cfg.dtype, 0.25, batch=8, ratio_kind=wk.WK_RATIO_NONANCHOR,
                                 score_algo=wk.WK_SCORE_GEMM)
    assert wk.wk_compress_workspace_bytes(desc) > wk.wk_compress_scratch_bytes()
    t = torch.zeros(16, dtype=torch.bfloat16, device=d)   # never touched: the size check comes before any launch
    with pytest.raises(wk.WkError) as e:
        wk.wk_compress_chunk_noalloc(desc, t, t, None, None, t, t)
    assert e.value.status == wk.WK_ERR_WORKSPACE
