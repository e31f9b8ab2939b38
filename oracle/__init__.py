"""ctypes front-end of the CPU oracle (oracle/wk_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  The HIP product path never imports this package
and this package never imports the HIP package.
"""
import ctypes as C
import math
import os

import numpy as np
import torch

from . import build as _build

_LIB = None

F32, BF16 = 0, 1
HEADS_SHARED, HEADS_INDEPENDENT = 0, 1
ANCHOR_FIRST_FRAME, ANCHOR_EXTERNAL = 0, 1
RATIO_CHUNK, RATIO_NONANCHOR = 0, 1
NORM_MAX, NORM_MINMAX, NORM_MEAN = 0, 1, 2


def lib():
    global _LIB
    if _LIB is None:
        # WK_ORACLE_LIB: an already built library to load instead (the sanitizer run of the oracle's pins)
        path = os.environ.get("WK_ORACLE_LIB") or _build.build(force=False)
        L = C.CDLL(path)
        L.wko_geodesic.restype = C.c_double
        L.wko_geodesic.argtypes = [C.c_double] * 4
        _LIB = L
    return _LIB


def n_threads() -> int:
    """OpenMP threads the oracle will use (OMP_NUM_THREADS or the core count)."""
    v = os.environ.get("OMP_NUM_THREADS")
    return int(v) if v else (os.cpu_count() or 1)


def set_threads(n: int) -> None:
    """Number of OpenMP threads for the following oracle calls (the library links libgomp)."""
    lib()
    C.CDLL("libgomp.so.1").omp_set_num_threads(int(n))
    os.environ["OMP_NUM_THREADS"] = str(int(n))


def _code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"oracle takes float32 or bfloat16 tensors, got {t.dtype}")


def _chk(t: torch.Tensor) -> torch.Tensor:
    assert t.device.type == "cpu" and t.is_contiguous()
    return t


def _p(t):
    if t is None:
        return C.c_void_p(0)
    if isinstance(t, torch.Tensor):
        return C.c_void_p(t.data_ptr())
    return C.c_void_p(t.ctypes.data)


def keep_count(rho, ratio_kind, anchor_mode, F, T):
    n_out, n_keep = C.c_int64(), C.c_int64()
    rc = lib().wko_keep_count(C.c_double(rho), ratio_kind, anchor_mode, F, T, C.byref(n_out), C.byref(n_keep))
    if rc != 0:
        raise ValueError("ratio out of range for this chunk")
    return n_out.value, n_keep.value


def compress_scores(K, K_anchor, T, F, head_mode=HEADS_SHARED, anchor_mode=ANCHOR_FIRST_FRAME, cand_sel=None):
    """Eq. 5 scores [G][N_c]; with cand_sel only those candidate indices are evaluated (others are NaN)."""
    _chk(K)
    H, n_tok, d = K.shape
    assert n_tok == F * T
    n_cand = n_tok if anchor_mode == ANCHOR_EXTERNAL else n_tok - T
    G = H if head_mode == HEADS_INDEPENDENT else 1
    out = np.zeros((G, n_cand), np.float64)
    n_sel = 0
    if cand_sel is not None:
        cand_sel = np.ascontiguousarray(cand_sel, np.int32)
        n_sel = cand_sel.size
        out[:] = np.nan
    rc = lib().wko_compress_scores(_p(K), _p(K_anchor), _code(K), H, d, T, F, head_mode, anchor_mode,
                                   _p(cand_sel), C.c_int64(n_sel), _p(out))
    assert rc == 0, rc
    return out


def select_lowest(scores, n_keep):
    s = np.ascontiguousarray(scores, np.float64)
    out = np.zeros(n_keep, np.int32)
    rc = lib().wko_select_lowest(_p(s), C.c_int64(s.size), C.c_int64(n_keep), _p(out))
    assert rc == 0, rc
    return out


def compress(K, V, K_anchor, T, F, rho, ratio_kind=RATIO_CHUNK, head_mode=HEADS_SHARED,
             anchor_mode=ANCHOR_FIRST_FRAME):
    """Returns kept_idx [G][n_out] int32, K_out, V_out [H][n_out][d], scores [G][N_c]."""
    _chk(K), _chk(V)
    H, n_tok, d = K.shape
    n_out, _ = keep_count(rho, ratio_kind, anchor_mode, F, T)
    n_cand = n_tok if anchor_mode == ANCHOR_EXTERNAL else n_tok - T
    G = H if head_mode == HEADS_INDEPENDENT else 1
    idx = np.zeros((G, n_out), np.int32)
    K_out = torch.empty((H, n_out, d), dtype=K.dtype)
    V_out = torch.empty((H, n_out, d), dtype=V.dtype)
    scores = np.zeros((G, n_cand), np.float64)
    rc = lib().wko_compress(_p(K), _p(V), _p(K_anchor), _code(K), H, d, T, F, head_mode, anchor_mode,
                            C.c_double(rho), ratio_kind, _p(idx), _p(K_out), _p(V_out), _p(scores))
    assert rc == 0, rc
    return idx, K_out, V_out, scores


def geodesic(yaw_a, pitch_a, yaw_b, pitch_b) -> float:
    return lib().wko_geodesic(yaw_a, pitch_a, yaw_b, pitch_b)


def score_chunks(poses, cur, R, norm_mode=NORM_MAX):
    """Returns ids [min(R,M)] int32, D_sel, D_all [M]."""
    poses = np.ascontiguousarray(poses, np.float32).reshape(-1, 5)
    cur = np.ascontiguousarray(cur, np.float32)
    M = poses.shape[0]
    ids = np.zeros(max(R, 1), np.int32)
    d_sel = np.zeros(max(R, 1), np.float64)
    d_all = np.zeros(max(M, 1), np.float64)
    n = C.c_int32()
    rc = lib().wko_score_chunks(_p(poses), M, _p(cur), norm_mode, R, _p(ids), _p(d_sel), _p(d_all), C.byref(n))
    assert rc == 0, rc
    return ids[: n.value].copy(), d_sel[: n.value].copy(), d_all[:M].copy()


def accumulate_actions(labels, step=1.0, dangle=math.radians(15.0), pitch_limit=math.radians(60.0)):
    labels = np.ascontiguousarray(labels, np.int32)
    out = np.zeros((labels.size, 5), np.float32)
    rc = lib().wko_accumulate_actions(_p(labels), labels.size, C.c_double(step), C.c_double(dangle),
                                      C.c_double(pitch_limit), _p(out))
    if rc != 0:
        raise ValueError("action label out of range")
    return out


def gather(K_chunks, V_chunks, ids, K_native, V_native, win_capacity):
    """K_chunks/V_chunks: lists of [H][n_c][d] CPU tensors (the store). Returns K_win, V_win, n_win."""
    ref = K_native if K_native is not None else K_chunks[0]
    H, _, d = ref.shape
    n_native = 0 if K_native is None else K_native.shape[1]
    Mc = len(K_chunks)
    kp = (C.c_void_p * max(Mc, 1))(*[c.data_ptr() for c in K_chunks])
    vp = (C.c_void_p * max(Mc, 1))(*[c.data_ptr() for c in V_chunks])
    n_tok = np.array([c.shape[1] for c in K_chunks] or [0], np.int32)
    ids = np.ascontiguousarray(ids, np.int32)
    K_win = torch.zeros((H, win_capacity, d), dtype=ref.dtype)
    V_win = torch.zeros((H, win_capacity, d), dtype=ref.dtype)
    n_win = C.c_int32()
    rc = lib().wko_gather(kp, vp, _p(n_tok), _p(ids), ids.size, _p(K_native), _p(V_native), n_native,
                          H, d, _code(ref), _p(K_win), _p(V_win), win_capacity, C.byref(n_win))
    if rc != 0:
        raise ValueError(f"gather failed ({rc})")
    return K_win, V_win, n_win.value


def attention(Q, K, V, N_kv=None, scale=None, rows=None, want_lse=False):
    """fp64 softmax attention. Q [H][N_q][d], K/V [H][stride][d]. Returns O [H][n_rows][d] float64."""
    _chk(Q), _chk(K), _chk(V)
    H, N_q, d = Q.shape
    stride = K.shape[1]
    N_kv = stride if N_kv is None else N_kv
    scale = 1.0 / math.sqrt(d) if scale is None else scale
    if rows is not None:
        rows = np.ascontiguousarray(rows, np.int32)
        n_rows = rows.size
    else:
        n_rows = N_q
    O = np.zeros((H, n_rows, d), np.float64)
    lse = np.zeros((H, n_rows), np.float64)
    rc = lib().wko_attention(_p(Q), _p(K), _p(V), _code(Q), H, C.c_int64(N_q), C.c_int64(N_kv), d,
                             C.c_int64(stride), C.c_double(scale), _p(rows), C.c_int64(n_rows), _p(O), _p(lse))
    assert rc == 0, rc
    return (O, lse) if want_lse else O


def attention_block_causal(Q, K, V, denoise_row0, frame_T, N_kv=None, scale=None, rows=None, want_lse=False):
    """fp64 attention with the frame-level causal mask inside the denoising chunk, whose keys are window
    rows [denoise_row0, denoise_row0 + N_q)."""
    _chk(Q), _chk(K), _chk(V)
    H, N_q, d = Q.shape
    stride = K.shape[1]
    N_kv = stride if N_kv is None else N_kv
    scale = 1.0 / math.sqrt(d) if scale is None else scale
    if rows is not None:
        rows = np.ascontiguousarray(rows, np.int32)
        n_rows = rows.size
    else:
        n_rows = N_q
    O = np.zeros((H, n_rows, d), np.float64)
    lse = np.zeros((H, n_rows), np.float64)
    rc = lib().wko_attention_block_causal(_p(Q), _p(K), _p(V), _code(Q), H, C.c_int64(N_q), C.c_int64(N_kv), d,
                                          C.c_int64(stride), C.c_double(scale), C.c_int64(denoise_row0),
                                          C.c_int64(frame_T), _p(rows), C.c_int64(n_rows), _p(O), _p(lse))
    if rc != 0:
        raise ValueError(f"attention_block_causal failed ({rc})")
    return (O, lse) if want_lse else O


def score_chunks_query(Q, K_chunks, R, scale=None):
    """Query-based retrieval: ids [min(R,M)], mass_sel, mass_all [M] (attention mass per stored chunk)."""
    _chk(Q)
    H, N_q, d = Q.shape
    M = len(K_chunks)
    scale = 1.0 / math.sqrt(d) if scale is None else scale
    kp = (C.c_void_p * max(M, 1))(*[_chk(c).data_ptr() for c in K_chunks])
    n_tok = np.array([c.shape[1] for c in K_chunks] or [0], np.int32)
    ids = np.zeros(max(R, 1), np.int32)
    m_sel = np.zeros(max(R, 1), np.float64)
    m_all = np.zeros(max(M, 1), np.float64)
    n = C.c_int32()
    rc = lib().wko_score_chunks_query(_p(Q), kp, _p(n_tok), M, _code(Q), H, C.c_int64(N_q), d, C.c_double(scale), R,
                                      _p(ids), _p(m_sel), _p(m_all), C.byref(n))
    assert rc == 0, rc
    return ids[: n.value].copy(), m_sel[: n.value].copy(), m_all[:M].copy()
