"""CPU-only checks of the C-ABI library: it loads, exports every symbol the header declares,
rejects bad arguments before launching anything, and its host-side helpers agree with the oracle."""
import ctypes as C
import math
import os
import re

import numpy as np
import pytest

import oracle
import paper_2605_22718_amd as wk
import wk_synth as ws

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "wk.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(wk_[a-z_]+)\s*\(", header))
    assert declared == set(wk.EXPORTS), declared ^ set(wk.EXPORTS)
    L = wk.lib()
    for name in declared:
        assert getattr(L, name) is not None


def test_status_strings():
    seen = {wk.status_string(s) for s in range(7)}
    assert len(seen) == 7 and "ok" in seen


def test_keep_count_matches_oracle_and_paper_counts():
    for T in (880, 1560, 7, 1):
        for F in (1, 2, 3, 4):
            for kind in (wk.WK_RATIO_CHUNK, wk.WK_RATIO_NONANCHOR):
                for anchor in (wk.WK_ANCHOR_FIRST_FRAME, wk.WK_ANCHOR_EXTERNAL):
                    for rho in (0.0, 0.125, 0.25, 0.3, 0.5, 0.75, 1.0):
                        rho32 = float(np.float32(rho))
                        try:
                            expect = oracle.keep_count(rho32, kind, anchor, F, T)
                        except ValueError:
                            with pytest.raises(wk.WkError) as e:
                                wk.wk_keep_count(rho32, kind, anchor, F, T)
                            assert e.value.status == wk.WK_ERR_RATIO
                            continue
                        assert wk.wk_keep_count(rho32, kind, anchor, F, T) == expect
    assert wk.wk_keep_count(0.25, wk.WK_RATIO_NONANCHOR, wk.WK_ANCHOR_FIRST_FRAME, 3, 880) == (1320, 440)
    assert wk.wk_keep_count(0.5, wk.WK_RATIO_CHUNK, wk.WK_ANCHOR_FIRST_FRAME, 3, 1560) == (2340, 780)
    with pytest.raises(wk.WkError):
        wk.wk_keep_count(1.01, wk.WK_RATIO_CHUNK, wk.WK_ANCHOR_FIRST_FRAME, 3, 880)
    with pytest.raises(wk.WkError):
        wk.wk_keep_count(float("nan"), wk.WK_RATIO_CHUNK, wk.WK_ANCHOR_FIRST_FRAME, 3, 880)


def test_accumulate_actions_matches_oracle():
    step, dangle, lim = (float(np.float32(x)) for x in (1.0, math.radians(15.0), math.radians(60.0)))
    for n, seed in [(0, 1), (1, 2), (50, 3), (1000, 4)]:
        labels = ws.make_action_labels(n, seed)
        got = wk.wk_accumulate_actions(labels, step, dangle, lim).numpy()
        ref = oracle.accumulate_actions(labels, step, dangle, lim)
        np.testing.assert_array_equal(got, ref)
    with pytest.raises(wk.WkError) as e:
        wk.wk_accumulate_actions(np.array([0, 9], np.int32))
    assert e.value.status == wk.WK_ERR_INVALID_ARG


def test_workspace_size_and_descriptor_validation():
    d = wk.make_compress_desc(12, 880, 3, wk.WK_BF16, 0.5)
    n = wk.wk_compress_workspace_bytes(d)
    assert n >= 1760 * 8 + 880 * 8 + 12 * 128 * 4 and n % 256 == 0
    bad = wk.make_compress_desc(12, 880, 3, wk.WK_BF16, 0.5, d=64)
    assert wk.wk_compress_workspace_bytes(bad) == 0
    L = wk.lib()
    one = C.c_void_p(256)   # never dereferenced: every call below fails validation first
    n_out = C.c_int32(-7)
    assert L.wk_compress_chunk(C.byref(bad), one, one, None, None, one, one, C.byref(n_out), one, 1 << 30, None) \
        == wk.WK_ERR_UNSUPPORTED
    assert L.wk_compress_chunk(C.byref(d), None, one, None, None, one, one, C.byref(n_out), one, 1 << 30, None) \
        == wk.WK_ERR_INVALID_ARG
    assert L.wk_compress_chunk(C.byref(d), one, one, None, None, one, one, C.byref(n_out), one, 16, None) \
        == wk.WK_ERR_WORKSPACE
    assert L.wk_compress_chunk(C.byref(d), one, one, None, None, one, one, C.byref(n_out), C.c_void_p(8), 1 << 30, None) \
        == wk.WK_ERR_WORKSPACE      # misaligned
    assert L.wk_compress_chunk(C.byref(d), one, one, one, None, one, one, C.byref(n_out), one, 1 << 30, None) \
        == wk.WK_ERR_INVALID_ARG    # anchor given in first-frame mode
    low = wk.make_compress_desc(40, 1560, 3, wk.WK_BF16, 0.25)   # below the anchor frame
    assert L.wk_compress_chunk(C.byref(low), one, one, None, None, one, one, C.byref(n_out), one, 1 << 30, None) \
        == wk.WK_ERR_RATIO
    assert n_out.value == -7    # outputs untouched on error


def test_argument_validation_of_the_other_calls():
    L = wk.lib()
    one = C.c_void_p(256)
    cur = (C.c_float * 5)()
    assert L.wk_score_chunks(one, -1, cur, 0, 1, one, None, one, None) == wk.WK_ERR_INVALID_ARG
    assert L.wk_score_chunks(one, 5, cur, 7, 1, one, None, one, None) == wk.WK_ERR_INVALID_ARG
    assert L.wk_score_chunks(one, 5, cur, 0, 1, one, None, None, None) == wk.WK_ERR_INVALID_ARG
    assert L.wk_score_chunks(one, wk.WK_SCORE_MAX_CHUNKS + 1, cur, 0, 1, one, None, one, None) == wk.WK_ERR_UNSUPPORTED
    # attention
    args = dict(H=2, N_q=8, N_kv=8, d=128, stride=8, dtype=wk.WK_BF16)
    def attn(**kw):
        a = dict(args, **kw)
        return L.wk_attention(one, one, one, one, None, a["H"], a["N_q"], a["N_kv"], a["d"], a["stride"],
                              a["dtype"], 0.0, None, None, 0, None)
    assert attn(d=64) == wk.WK_ERR_UNSUPPORTED
    assert attn(N_kv=0) == wk.WK_ERR_SHAPE
    assert attn(N_kv=9) == wk.WK_ERR_SHAPE
    assert attn(dtype=5) == wk.WK_ERR_INVALID_ARG
    assert attn(H=0) == wk.WK_ERR_INVALID_ARG
    assert L.wk_attention(None, one, one, one, None, 2, 8, 8, 128, 8, 1, 0.0, None, None, 0, None) == wk.WK_ERR_INVALID_ARG
    # bf16 windows beyond what the kernels' 32-bit byte offsets reach are refused, not wrapped around
    big = (1 << 24) - 511
    assert attn(N_kv=big, stride=big) == wk.WK_ERR_UNSUPPORTED
    assert attn(N_kv=1 << 26, stride=1 << 26) == wk.WK_ERR_UNSUPPORTED
    # O == NULL asks for the log-sum-exp only and then needs lse
    assert L.wk_attention(one, one, None, None, None, 2, 8, 8, 128, 8, 1, 0.0, None, None, 0, None) == wk.WK_ERR_INVALID_ARG
    # query-based retrieval
    assert wk.wk_score_chunks_query_workspace_bytes(wk.WK_QUERY_MAX_CHUNKS + 1, 100) == 0
    need = wk.wk_score_chunks_query_workspace_bytes(120, 40 * 4680)
    assert need >= 120 * 8 * 2 and need % 256 == 0
    def sq(**kw):
        a = dict(dict(lse=one, M=4, n_rows=64, R=2, ids=one, n_found=one, ws=one, ws_bytes=1 << 20), **kw)
        return L.wk_score_chunks_query(a["lse"], a["M"], a["n_rows"], a["R"], a["ids"], None, a["n_found"],
                                       a["ws"], a["ws_bytes"], None)
    assert sq(M=-1) == wk.WK_ERR_INVALID_ARG
    assert sq(n_rows=0) == wk.WK_ERR_INVALID_ARG
    assert sq(lse=None) == wk.WK_ERR_INVALID_ARG
    assert sq(ids=None) == wk.WK_ERR_INVALID_ARG
    assert sq(n_found=None) == wk.WK_ERR_INVALID_ARG
    assert sq(M=wk.WK_QUERY_MAX_CHUNKS + 1) == wk.WK_ERR_UNSUPPORTED
    assert sq(ws=None) == wk.WK_ERR_WORKSPACE
    assert sq(ws_bytes=16) == wk.WK_ERR_WORKSPACE
    assert sq(ws=C.c_void_p(264)) == wk.WK_ERR_WORKSPACE
    sd = wk.wk_store_desc(256, 256, 256, 4, 10, 2, 128, wk.WK_BF16)
    assert L.wk_chunk_lse(None, one, 8, 0.0, one, None) == wk.WK_ERR_INVALID_ARG
    assert L.wk_chunk_lse(C.byref(sd), None, 8, 0.0, one, None) == wk.WK_ERR_INVALID_ARG
    assert L.wk_chunk_lse(C.byref(sd), one, 8, 0.0, None, None) == wk.WK_ERR_INVALID_ARG
    assert L.wk_chunk_lse(C.byref(sd), one, -1, 0.0, one, None) == wk.WK_ERR_INVALID_ARG
    assert L.wk_chunk_lse(C.byref(sd), one, 8, -1.0, one, None) == wk.WK_ERR_INVALID_ARG
    sd64 = wk.wk_store_desc(256, 256, 256, 4, 10, 2, 64, wk.WK_BF16)
    assert L.wk_chunk_lse(C.byref(sd64), one, 8, 0.0, one, None) == wk.WK_ERR_UNSUPPORTED
    sd_big = wk.wk_store_desc(256, 256, 256, 4, (1 << 24) - 511, 2, 128, wk.WK_BF16)
    assert L.wk_chunk_lse(C.byref(sd_big), one, 8, 0.0, one, None) == wk.WK_ERR_UNSUPPORTED   # 32-bit byte offsets
    sd0 = wk.wk_store_desc(None, None, None, 0, 0, 2, 128, wk.WK_BF16)
    assert L.wk_chunk_lse(C.byref(sd0), one, 8, 0.0, one, None) == wk.WK_OK      # empty store: nothing to do
    # attention in place over the store
    def ip(store=sd, Q=one, Kn=one, Vn=one, n_native=4, stride=4, ids=one, R=2, O=one, N_q=8, scale=0.0):
        return L.wk_attention_in_place(Q, Kn, Vn, n_native, stride, C.byref(store) if store is not None else None, ids,
                                       None, R, O, None, N_q, scale, None)
    assert ip(store=None) == wk.WK_ERR_INVALID_ARG
    assert ip(Q=None) == wk.WK_ERR_INVALID_ARG
    assert ip(O=None) == wk.WK_ERR_INVALID_ARG
    assert ip(Kn=None) == wk.WK_ERR_INVALID_ARG          # native rows announced but not given
    assert ip(ids=None) == wk.WK_ERR_INVALID_ARG
    assert ip(R=-1) == wk.WK_ERR_INVALID_ARG
    assert ip(scale=-1.0) == wk.WK_ERR_INVALID_ARG
    assert ip(n_native=5) == wk.WK_ERR_SHAPE             # more native rows than the stride
    assert ip(R=33) == wk.WK_ERR_UNSUPPORTED
    assert ip(store=sd64) == wk.WK_ERR_UNSUPPORTED
    assert ip(store=wk.wk_store_desc(256, 256, 256, 4, 10, 2, 128, wk.WK_F32)) == wk.WK_ERR_UNSUPPORTED
    assert ip(N_q=0) == wk.WK_OK                         # nothing to do
    # prefetch handle: argument checks that need no device
    h = C.c_void_p()
    assert L.wk_prefetch_create(None, 2) == wk.WK_ERR_INVALID_ARG
    assert L.wk_prefetch_create(C.byref(h), 0) == wk.WK_ERR_INVALID_ARG
    assert L.wk_prefetch_create(C.byref(h), 9) == wk.WK_ERR_INVALID_ARG
    assert L.wk_prefetch_destroy(None) == wk.WK_OK
    assert L.wk_prefetch_stream(None) is None
    assert L.wk_prefetch_after(None, None) == wk.WK_ERR_INVALID_ARG
    assert L.wk_prefetch_acquire(None, 0, None) == wk.WK_ERR_INVALID_ARG
    assert L.wk_prefetch_release(None, 0, None) == wk.WK_ERR_INVALID_ARG
    assert L.wk_prefetch_gather(None, 0, C.byref(sd), one, None, 2, one, one, 5, one, one, 64, None, 0) == wk.WK_ERR_INVALID_ARG
    # block-causal attention
    def bc(**kw):
        a = dict(dict(N_q=6, N_kv=20, row0=4, T=3, ws=one, ws_bytes=1 << 20, d=128), **kw)
        return L.wk_attention_block_causal(one, one, one, one, None, 2, a["N_q"], a["N_kv"], a["d"], 32, 1, 0.0, None,
                                           a["row0"], a["T"], a["ws"], a["ws_bytes"], None)
    assert bc(T=0) == wk.WK_ERR_INVALID_ARG
    assert bc(row0=-1) == wk.WK_ERR_INVALID_ARG
    assert bc(d=64) == wk.WK_ERR_UNSUPPORTED
    assert bc(T=4) == wk.WK_ERR_SHAPE             # N_q is not a multiple of the frame
    assert bc(row0=15) == wk.WK_ERR_SHAPE         # the chunk's rows run past the window
    assert bc(N_kv=40) == wk.WK_ERR_SHAPE         # beyond the row stride
    assert L.wk_attention_block_causal(one, one, one, one, None, 2, 6, 1 << 24, 128, 1 << 24, 1, 0.0, None, 4, 3, one,
                                       1 << 20, None) == wk.WK_ERR_UNSUPPORTED               # 32-bit byte offsets
    assert bc(ws=None) == wk.WK_ERR_WORKSPACE
    assert bc(ws_bytes=100) == wk.WK_ERR_WORKSPACE
    assert wk.wk_attention_block_causal_workspace_bytes(2, 6) >= 2 * 2 * 6 * (128 + 2) * 4
    # calibration copy
    assert L.wk_calibration_copy(None, one, 32, None) == wk.WK_ERR_INVALID_ARG
    assert L.wk_calibration_copy(one, one, 24, None) == wk.WK_ERR_INVALID_ARG           # not a multiple of 16
    assert L.wk_calibration_copy(C.c_void_p(264), one, 32, None) == wk.WK_ERR_INVALID_ARG  # misaligned
    assert L.wk_calibration_copy(one, one, 0, None) == wk.WK_OK
    # key-range splits are only proposed when the plain grid would leave compute units idle
    assert wk.wk_attention_workspace_bytes(40, 4680, 28080, wk.WK_BF16) == 0
    assert wk.wk_attention_workspace_bytes(12, 2640, 211200, wk.WK_BF16) > 12 * 2640 * 128 * 4   # few items, long window
    assert wk.wk_attention_workspace_bytes(12, 2640, 10560, wk.WK_BF16) == 0     # short window: 128-query workgroups instead
    assert wk.wk_attention_workspace_bytes(4, 880, 2640, wk.WK_F32) > 4 * 880 * 128 * 4       # the tiny fp32 case splits
    assert wk.wk_attention_workspace_bytes(40, 4680 * 8, 28080, wk.WK_F32) == 0              # enough workgroups as it is
    assert wk.wk_attention_workspace_bytes(4, 880, 2640, 7) == 0                              # unknown element type
    assert wk.wk_attention_workspace_bytes(1, 64, 128, wk.WK_BF16) == 0      # too short to split
    # gather
    sd = wk.wk_store_desc(256, 256, 256, 4, 10, 2, 128, wk.WK_BF16)
    assert L.wk_gather_window(C.byref(sd), one, None, 2, one, one, 5, one, one, 24, None, None) == wk.WK_ERR_SHAPE
    assert L.wk_gather_window(C.byref(sd), None, None, 2, one, one, 5, one, one, 25, None, None) == wk.WK_ERR_INVALID_ARG
    assert L.wk_gather_window(C.byref(sd), one, None, 2, one, None, 5, one, one, 25, None, None) == wk.WK_ERR_INVALID_ARG
    assert L.wk_gather_window(C.byref(sd), one, None, 2000, one, one, 5, one, one, 1 << 30, None, None) \
        == wk.WK_ERR_UNSUPPORTED
    sd64 = wk.wk_store_desc(256, 256, 256, 4, 10, 2, 64, wk.WK_BF16)
    assert L.wk_gather_window(C.byref(sd64), one, None, 2, one, one, 5, one, one, 25, None, None) == wk.WK_ERR_UNSUPPORTED
    # window update: slots longer than any chunk the store's bound allows
    need = wk.wk_window_update_workspace_bytes(2)
    assert L.wk_window_update(C.byref(sd), one, None, 2, 11, one, 5, one, one, 64, None, None, one, need, 0, None) \
        == wk.WK_ERR_SHAPE
    assert L.wk_host_device_pointer(None, None) == wk.WK_ERR_INVALID_ARG


def test_window_plan_matches_the_rolling_window_simulation():
    """The planner's row arithmetic, applied to a label array standing for the window rows, must put
    every generated chunk exactly where the oracle's simulation says it lives (Sec. 4.2 regions)."""
    from oracle.window import RollingWindow
    for sink_chunks, recent_chunks, frames, T in [(1, 1, 3, 5), (1, 2, 3, 4), (2, 1, 2, 3), (0, 1, 3, 2), (1, 0, 1, 7)]:
        desc = wk.wk_window_desc(T, frames, sink_chunks, recent_chunks, 6, 11)
        sim = RollingWindow(sink_chunks, recent_chunks)
        rows = None
        stored = []
        for c in range(30):
            p = wk.wk_window_plan(desc, c)
            region, slot, evicted = sim.step(c)
            chunk_rows = frames * T
            if rows is None:
                rows = np.full(p.win_capacity, -1, np.int64)
                assert p.win_capacity == (sink_chunks + recent_chunks + 1) * chunk_rows + 6 * 11
                assert p.retrieved_row0 == (sink_chunks + recent_chunks + 1) * chunk_rows
            assert p.denoise_rows == chunk_rows
            if p.evict:
                assert evicted is not None and p.evict_chunk == evicted
                assert np.all(rows[p.evict_row0:p.evict_row0 + chunk_rows] == evicted)   # it is still there
                assert p.store_id == len(stored)
                stored.append(evicted)
            else:
                assert evicted is None and p.store_id == -1 and p.evict_chunk == -1
                assert np.all(rows[p.denoise_row0:p.denoise_row0 + chunk_rows] == -1)    # never overwrite unsaved rows
            rows[p.denoise_row0:p.denoise_row0 + chunk_rows] = c
            assert stored == sim.store and p.M == len(sim.store)
            # the valid native rows are a prefix and hold exactly sink + ring
            live = sorted(set(rows[:p.n_native].tolist()))
            assert live == sorted(list(sim.sink) + list(sim.ring))
            assert np.all(rows[p.n_native:p.retrieved_row0] == -1)
            if p.M > 0:
                assert p.n_native == p.retrieved_row0        # retrieval starts only once the ring is full
    # paper shape: 18 frames of 880 tokens with 6 slots of 1.5 frames
    desc = wk.wk_window_desc(880, 3, 1, 1, 6, 1320)
    p = wk.wk_window_plan(desc, 10)
    assert p.win_capacity == 18 * 880 and p.n_native == 9 * 880 and p.M == 8
    L = wk.lib()
    assert L.wk_window_plan(None, 0, C.byref(p)) == wk.WK_ERR_INVALID_ARG
    assert L.wk_window_plan(C.byref(desc), -1, C.byref(p)) == wk.WK_ERR_INVALID_ARG
    assert L.wk_window_plan(C.byref(wk.wk_window_desc(0, 3, 1, 1, 6, 10)), 0, C.byref(p)) == wk.WK_ERR_INVALID_ARG
    assert L.wk_window_plan(C.byref(wk.wk_window_desc(1 << 20, 1 << 10, 1, 1, 6, 10)), 0, C.byref(p)) == wk.WK_ERR_UNSUPPORTED
    # wk_window_update argument checks
    one = C.c_void_p(256)
    sd = wk.wk_store_desc(256, 256, 256, 4, 10, 2, 128, wk.WK_BF16)
    def upd(**kw):
        a = dict(dict(R=2, slot=10, slots=one, n_native=5, cap=64, ws=one, ws_bytes=1 << 16, ids=one), **kw)
        return L.wk_window_update(C.byref(sd), a["ids"], None, a["R"], a["slot"], a["slots"], a["n_native"], one, one,
                                  a["cap"], None, None, a["ws"], a["ws_bytes"], 0, None)
    assert upd(R=-1) == wk.WK_ERR_INVALID_ARG
    assert upd(slot=0) == wk.WK_ERR_INVALID_ARG
    assert upd(slots=None) == wk.WK_ERR_INVALID_ARG
    assert upd(ids=None) == wk.WK_ERR_INVALID_ARG
    assert upd(R=1025) == wk.WK_ERR_UNSUPPORTED
    assert upd(cap=24) == wk.WK_ERR_SHAPE
    assert upd(ws=None) == wk.WK_ERR_WORKSPACE
    assert upd(ws_bytes=8) == wk.WK_ERR_WORKSPACE
    assert wk.wk_window_update_workspace_bytes(1025) == 0 and wk.wk_window_update_workspace_bytes(6) >= 256 + 48


C_PROGRAM = r"""
#include <stdio.h>
#include <stddef.h>
#include <string.h>
#include "wk.h"
int main(void) {
    int32_t n_out = 0, n_keep = 0;
    if (wk_keep_count(0.25f, WK_RATIO_NONANCHOR, WK_ANCHOR_FIRST_FRAME, 3, 880, &n_out, &n_keep) != WK_OK) return 1;
    printf("keep %d %d\n", (int)n_out, (int)n_keep);
    printf("status %s\n", wk_status_string(WK_ERR_WORKSPACE));
    printf("sizes %d %d %d %d\n", (int)sizeof(wk_compress_desc), (int)sizeof(wk_store_desc), (int)sizeof(wk_window_desc),
           (int)sizeof(wk_window_step));
    printf("offsets %d %d %d\n", (int)offsetof(wk_store_desc, M), (int)offsetof(wk_window_step, evict_chunk),
           (int)offsetof(wk_window_step, win_capacity));
    wk_window_desc w = {1560, 3, 1, 1, 6, 2340};
    for (long long c = 0; c < 6; ++c) {
        wk_window_step s;
        if (wk_window_plan(&w, c, &s) != WK_OK) return 2;
        printf("plan %lld %d %d %d %d %d %d %lld %d %d %d\n", c, (int)s.denoise_row0, (int)s.denoise_rows, (int)s.n_native,
               (int)s.evict, (int)s.evict_row0, (int)s.store_id, (long long)s.evict_chunk, (int)s.M, (int)s.retrieved_row0,
               (int)s.win_capacity);
    }
    /* argument errors come back as status codes, before anything touches a device */
    if (wk_attention(NULL, NULL, NULL, NULL, NULL, 1, 1, 1, 128, 1, WK_BF16, 0.f, NULL, NULL, 0, NULL) != WK_ERR_INVALID_ARG)
        return 3;
    return 0;
}
"""


def test_header_is_c99_and_a_c_program_sees_what_the_binding_sees(tmp_path):
    """include/wk.h compiles as strict C99; a C program linked against libwk.so gets the same counts, structure
    layouts and window plans as the ctypes binding."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no C compiler")
    src = tmp_path / "abi.c"
    src.write_text(C_PROGRAM)
    libdir = os.path.dirname(wk.lib()._name)
    exe = tmp_path / "abi"
    cmd = ["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"), str(src),
           wk.lib()._name, "-Wl,-rpath," + libdir, "-Wl,-rpath-link,/opt/rocm/lib",
           "-Wl,--allow-shlib-undefined",    # a host-sanitizer build of the library leaves its runtime to a preload
           "-o", str(exe)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    r = subprocess.run([str(exe)], capture_output=True, text=True)
    assert r.returncode == 0, (r.returncode, r.stdout, r.stderr)
    lines = r.stdout.split("\n")
    assert lines[0] == "keep 1320 440"
    assert lines[1] == "status " + wk.status_string(wk.WK_ERR_WORKSPACE)
    assert lines[2] == "sizes %d %d %d %d" % (C.sizeof(wk.wk_compress_desc), C.sizeof(wk.wk_store_desc),
                                               C.sizeof(wk.wk_window_desc), C.sizeof(wk.wk_window_step))
    assert lines[3] == "offsets %d %d %d" % (wk.wk_store_desc.M.offset, wk.wk_window_step.evict_chunk.offset,
                                             wk.wk_window_step.win_capacity.offset)
    w = wk.wk_window_desc(1560, 3, 1, 1, 6, 2340)
    for c in range(6):
        s = wk.wk_window_plan(w, c)
        assert lines[4 + c] == "plan %d %d %d %d %d %d %d %d %d %d %d" % (
            c, s.denoise_row0, s.denoise_rows, s.n_native, s.evict, s.evict_row0, s.store_id, s.evict_chunk, s.M,
            s.retrieved_row0, s.win_capacity)


def test_the_hand_scheduled_attention_loop_is_what_its_generator_writes():
    """csrc/wk_attn_loop_gfx950.inc is committed as written by csrc/gen_attn_loop.py: regenerate and compare."""
    import importlib.util
    csrc = os.path.join(ROOT, "paper_2605_22718_amd", "csrc")
    spec = importlib.util.spec_from_file_location("gen_attn_loop", os.path.join(csrc, "gen_attn_loop.py"))
    gen = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(gen)
    assert gen.render() == open(os.path.join(csrc, "wk_attn_loop_gfx950.inc")).read()
    lines = gen.generate()
    # four steps of 32 matrix instructions; the products kept back by the last step stand behind the loop once more
    assert sum(l.startswith("v_mfma") for l in lines) == 4 * 32 + gen.DEFER
    assert sum(l == "s_barrier" for l in lines) == 4
