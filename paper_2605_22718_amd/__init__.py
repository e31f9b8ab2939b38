"""Thin Python binding of libwk (include/wk.h): argument marshalling only.

Every function has the name and the meaning of the C entry point it calls; all
arithmetic happens in the HIP kernels of libwk.so.  PyTorch is used for device
memory and the current HIP stream.  There is no CPU fallback: if the library is
missing, importing a function raises.
"""
import ctypes as C
import math
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libwk.so")

WK_OK, WK_ERR_INVALID_ARG, WK_ERR_SHAPE, WK_ERR_RATIO, WK_ERR_WORKSPACE, WK_ERR_UNSUPPORTED, WK_ERR_HIP = range(7)
WK_F32, WK_BF16 = 0, 1
WK_HEADS_SHARED, WK_HEADS_INDEPENDENT = 0, 1
WK_ANCHOR_FIRST_FRAME, WK_ANCHOR_EXTERNAL = 0, 1
WK_RATIO_CHUNK, WK_RATIO_NONANCHOR = 0, 1
WK_SCORE_FACTORED, WK_SCORE_GEMM = 0, 1
WK_NORM_MAX, WK_NORM_MINMAX, WK_NORM_MEAN = 0, 1, 2
WK_SCORE_MAX_CHUNKS = 4096
WK_QUERY_MAX_CHUNKS = 1024

EXPORTS = [
    "wk_keep_count", "wk_compress_workspace_bytes", "wk_compress_chunk", "wk_compress_chunk_noalloc",
    "wk_compress_scratch_bytes", "wk_score_chunks",
    "wk_score_chunks_query", "wk_score_chunks_query_workspace_bytes", "wk_chunk_lse",
    "wk_attention_block_causal", "wk_attention_block_causal_workspace_bytes",
    "wk_window_plan", "wk_window_update", "wk_window_update_workspace_bytes",
    "wk_prefetch_create", "wk_prefetch_destroy", "wk_prefetch_stream", "wk_prefetch_after", "wk_prefetch_gather",
    "wk_prefetch_acquire", "wk_prefetch_release",
    "wk_accumulate_actions", "wk_gather_window", "wk_attention", "wk_attention_workspace_bytes",
    "wk_attention_in_place",
    "wk_host_device_pointer", "wk_calibration_copy",
    "wk_status_string",
]


class WkError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (wk_status {status})")


class wk_compress_desc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("H", "d", "T", "F", "batch", "dtype", "head_mode", "anchor_mode", "ratio_kind", "score_algo")]
    _fields_.append(("rho", C.c_float))


class wk_store_desc(C.Structure):
    _fields_ = [("K_ptr", C.c_void_p), ("V_ptr", C.c_void_p), ("n_tok", C.c_void_p),
                ("M", C.c_int32), ("max_tok", C.c_int32), ("H", C.c_int32), ("d", C.c_int32),
                ("dtype", C.c_int32)]


class wk_window_desc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("T", "chunk_frames", "sink_chunks", "recent_chunks", "R", "slot_tokens")]


class wk_window_step(C.Structure):
    _fields_ = [("denoise_row0", C.c_int32), ("denoise_rows", C.c_int32), ("n_native", C.c_int32),
                ("evict", C.c_int32), ("evict_row0", C.c_int32), ("store_id", C.c_int32),
                ("evict_chunk", C.c_int64), ("M", C.c_int32), ("retrieved_row0", C.c_int32),
                ("win_capacity", C.c_int32)]


_lib = None


def lib():
    """The loaded C-ABI library.  Raises if it has not been built."""
    global _lib
    if _lib is None:
        # WK_LIB: another build of the same library to load instead (the host-sanitizer run of the host tests)
        path = os.environ.get("WK_LIB") or _LIB_PATH
        if not os.path.exists(path):
            raise ImportError(f"{path} is missing: run `python -c 'import __graft_entry__ as g; g.build()'`")
        L = C.CDLL(path)
        vp, i32, f32 = C.c_void_p, C.c_int32, C.c_float
        L.wk_keep_count.restype = C.c_int
        L.wk_keep_count.argtypes = [f32, i32, i32, i32, i32, C.POINTER(i32), C.POINTER(i32)]
        L.wk_compress_workspace_bytes.restype = C.c_size_t
        L.wk_compress_workspace_bytes.argtypes = [C.POINTER(wk_compress_desc)]
        L.wk_compress_chunk.restype = C.c_int
        L.wk_compress_chunk.argtypes = [C.POINTER(wk_compress_desc), vp, vp, vp, vp, vp, vp, C.POINTER(i32),
                                        vp, C.c_size_t, vp]
        L.wk_compress_chunk_noalloc.restype = C.c_int
        L.wk_compress_chunk_noalloc.argtypes = [C.POINTER(wk_compress_desc), vp, vp, vp, vp, vp, vp, C.POINTER(i32), vp]
        L.wk_compress_scratch_bytes.restype = C.c_size_t
        L.wk_compress_scratch_bytes.argtypes = []
        L.wk_score_chunks.restype = C.c_int
        L.wk_score_chunks.argtypes = [vp, i32, C.POINTER(f32), i32, i32, vp, vp, vp, vp]
        L.wk_attention_in_place.restype = C.c_int
        L.wk_attention_in_place.argtypes = [vp, vp, vp, i32, i32, C.POINTER(wk_store_desc), vp, vp, i32, vp, vp, i32,
                                            f32, vp]
        L.wk_score_chunks_query.restype = C.c_int
        L.wk_score_chunks_query.argtypes = [vp, i32, C.c_int64, i32, vp, vp, vp, vp, C.c_size_t, vp]
        L.wk_score_chunks_query_workspace_bytes.restype = C.c_size_t
        L.wk_score_chunks_query_workspace_bytes.argtypes = [i32, C.c_int64]
        L.wk_accumulate_actions.restype = C.c_int
        L.wk_accumulate_actions.argtypes = [vp, i32, f32, f32, f32, vp]
        L.wk_gather_window.restype = C.c_int
        L.wk_gather_window.argtypes = [C.POINTER(wk_store_desc), vp, vp, i32, vp, vp, i32, vp, vp, i32, vp, vp]
        L.wk_attention.restype = C.c_int
        L.wk_attention.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, f32, vp, vp, C.c_size_t, vp]
        L.wk_chunk_lse.restype = C.c_int
        L.wk_chunk_lse.argtypes = [C.POINTER(wk_store_desc), vp, i32, f32, vp, vp]
        L.wk_window_plan.restype = C.c_int
        L.wk_window_plan.argtypes = [C.POINTER(wk_window_desc), C.c_int64, C.POINTER(wk_window_step)]
        L.wk_window_update.restype = C.c_int
        L.wk_window_update.argtypes = [C.POINTER(wk_store_desc), vp, vp, i32, i32, vp, i32, vp, vp, i32, vp, vp, vp,
                                       C.c_size_t, i32, vp]
        L.wk_window_update_workspace_bytes.restype = C.c_size_t
        L.wk_window_update_workspace_bytes.argtypes = [i32]
        L.wk_prefetch_create.restype = C.c_int
        L.wk_prefetch_create.argtypes = [C.POINTER(vp), i32]
        L.wk_prefetch_destroy.restype = C.c_int
        L.wk_prefetch_destroy.argtypes = [vp]
        L.wk_prefetch_stream.restype = vp
        L.wk_prefetch_stream.argtypes = [vp]
        L.wk_prefetch_after.restype = C.c_int
        L.wk_prefetch_after.argtypes = [vp, vp]
        L.wk_prefetch_gather.restype = C.c_int
        L.wk_prefetch_gather.argtypes = [vp, i32, C.POINTER(wk_store_desc), vp, vp, i32, vp, vp, i32, vp, vp, i32, vp,
                                         i32]
        L.wk_prefetch_acquire.restype = C.c_int
        L.wk_prefetch_acquire.argtypes = [vp, i32, vp]
        L.wk_prefetch_release.restype = C.c_int
        L.wk_prefetch_release.argtypes = [vp, i32, vp]
        L.wk_attention_block_causal.restype = C.c_int
        L.wk_attention_block_causal.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, f32, vp, i32, i32,
                                                vp, C.c_size_t, vp]
        L.wk_attention_block_causal_workspace_bytes.restype = C.c_size_t
        L.wk_attention_block_causal_workspace_bytes.argtypes = [i32, i32]
        L.wk_attention_workspace_bytes.restype = C.c_size_t
        L.wk_attention_workspace_bytes.argtypes = [i32, i32, i32, i32]
        L.wk_calibration_copy.restype = C.c_int
        L.wk_calibration_copy.argtypes = [vp, vp, C.c_size_t, vp]
        L.wk_host_device_pointer.restype = C.c_int
        L.wk_host_device_pointer.argtypes = [vp, C.POINTER(vp)]
        L.wk_status_string.restype = C.c_char_p
        L.wk_status_string.argtypes = [C.c_int]
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().wk_status_string(status).decode()


def _check(status: int, where: str):
    if status != WK_OK:
        raise WkError(status, where)


def dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return WK_F32
    if t.dtype == torch.bfloat16:
        return WK_BF16
    raise TypeError(f"float32 or bfloat16 expected, got {t.dtype}")


def _dev(t, name, dtype=None):
    """Pointer of a contiguous tensor kernels can address (device, or pinned host)."""
    if t is None:
        return None
    if not isinstance(t, torch.Tensor):
        raise TypeError(f"{name}: tensor expected")
    if not t.is_contiguous():
        raise ValueError(f"{name}: must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"{name}: {dtype} expected, got {t.dtype}")
    if t.is_cuda:
        return t.data_ptr()
    if t.is_pinned():
        return wk_host_device_pointer(t)
    raise ValueError(f"{name}: must live on the GPU or in pinned host memory")


def _stream():
    return torch.cuda.current_stream().cuda_stream


def wk_host_device_pointer(t: torch.Tensor) -> int:
    """wk_host_device_pointer: device-visible address of a pinned host tensor."""
    out = C.c_void_p()
    _check(lib().wk_host_device_pointer(t.data_ptr(), C.byref(out)), "wk_host_device_pointer")
    return out.value


def wk_keep_count(rho, ratio_kind, anchor_mode, F, T):
    """wk_keep_count -> (n_out, n_keep)."""
    n_out, n_keep = C.c_int32(), C.c_int32()
    _check(lib().wk_keep_count(rho, ratio_kind, anchor_mode, F, T, C.byref(n_out), C.byref(n_keep)), "wk_keep_count")
    return n_out.value, n_keep.value


def make_compress_desc(H, T, F, dtype, rho, batch=1, d=128, head_mode=WK_HEADS_SHARED,
                       anchor_mode=WK_ANCHOR_FIRST_FRAME, ratio_kind=WK_RATIO_CHUNK,
                       score_algo=WK_SCORE_FACTORED) -> wk_compress_desc:
    return wk_compress_desc(H, d, T, F, batch, dtype, head_mode, anchor_mode, ratio_kind, score_algo, rho)


def wk_compress_workspace_bytes(desc: wk_compress_desc) -> int:
    return lib().wk_compress_workspace_bytes(C.byref(desc))


def wk_compress_chunk(desc: wk_compress_desc, K, V, K_anchor, kept_idx, K_out, V_out, workspace) -> int:
    """wk_compress_chunk.  All tensors are caller-allocated; returns n_out."""
    n_out = C.c_int32()
    st = lib().wk_compress_chunk(C.byref(desc), _dev(K, "K"), _dev(V, "V"), _dev(K_anchor, "K_anchor"),
                                 _dev(kept_idx, "kept_idx", torch.int32), _dev(K_out, "K_out"), _dev(V_out, "V_out"),
                                 C.byref(n_out), _dev(workspace, "workspace"),
                                 0 if workspace is None else workspace.numel() * workspace.element_size(), _stream())
    _check(st, "wk_compress_chunk")
    return n_out.value


def wk_compress_scratch_bytes() -> int:
    return lib().wk_compress_scratch_bytes()


def wk_compress_chunk_noalloc(desc: wk_compress_desc, K, V, K_anchor, kept_idx, K_out, V_out) -> int:
    """wk_compress_chunk_noalloc: wk_compress_chunk on the library's built-in scratch array; returns n_out."""
    n_out = C.c_int32()
    st = lib().wk_compress_chunk_noalloc(C.byref(desc), _dev(K, "K"), _dev(V, "V"), _dev(K_anchor, "K_anchor"),
                                         _dev(kept_idx, "kept_idx", torch.int32), _dev(K_out, "K_out"),
                                         _dev(V_out, "V_out"), C.byref(n_out), _stream())
    _check(st, "wk_compress_chunk_noalloc")
    return n_out.value


def wk_score_chunks(poses, M, cur_pose, norm_mode, R, ids_out, dist_out, n_found):
    """wk_score_chunks.  poses: device float32 [M][5]; cur_pose: 5 host floats."""
    cur = (C.c_float * 5)(*[float(x) for x in cur_pose])
    st = lib().wk_score_chunks(_dev(poses, "poses", torch.float32), M, cur, norm_mode, R,
                               _dev(ids_out, "ids_out", torch.int32), _dev(dist_out, "dist_out", torch.float64),
                               _dev(n_found, "n_found", torch.int32), _stream())
    _check(st, "wk_score_chunks")


def wk_score_chunks_query_workspace_bytes(M, n_rows) -> int:
    return lib().wk_score_chunks_query_workspace_bytes(M, n_rows)


def wk_score_chunks_query(lse, M, n_rows, R, ids_out, mass_out, n_found, workspace):
    """wk_score_chunks_query.  lse: device float32 [M][n_rows]; workspace: device, its first M doubles
    hold every chunk's mass afterwards."""
    st = lib().wk_score_chunks_query(_dev(lse, "lse", torch.float32), M, n_rows, R,
                                     _dev(ids_out, "ids_out", torch.int32),
                                     _dev(mass_out, "mass_out", torch.float64),
                                     _dev(n_found, "n_found", torch.int32), _dev(workspace, "workspace"),
                                     0 if workspace is None else workspace.numel() * workspace.element_size(),
                                     _stream())
    _check(st, "wk_score_chunks_query")


def wk_accumulate_actions(labels, step=1.0, dangle=math.radians(15.0), pitch_limit=math.radians(60.0)):
    """wk_accumulate_actions (host).  labels: int32 numpy array or CPU tensor -> float32 CPU tensor [n][5]."""
    lab = torch.as_tensor(labels, dtype=torch.int32).contiguous()
    out = torch.zeros((lab.numel(), 5), dtype=torch.float32)
    st = lib().wk_accumulate_actions(lab.data_ptr(), lab.numel(), step, dangle, pitch_limit, out.data_ptr())
    _check(st, "wk_accumulate_actions")
    return out


class Store:
    """Device-side tables describing a chunk store (wk_store_desc) built from lists of tensors."""

    def __init__(self, K_chunks, V_chunks, device="cuda"):
        assert len(K_chunks) == len(V_chunks)
        self.K_chunks, self.V_chunks = list(K_chunks), list(V_chunks)  # keep the memory alive
        ref = K_chunks[0]
        self.H, self.d = ref.shape[0], ref.shape[2]
        self.dtype = dtype_code(ref)
        n_tok = [k.shape[1] for k in K_chunks]
        self.max_tok = max(n_tok)
        kp = [_dev(k, "K chunk") for k in K_chunks]
        vp = [_dev(v, "V chunk") for v in V_chunks]
        self.K_ptr = torch.tensor(kp, dtype=torch.int64, device=device)
        self.V_ptr = torch.tensor(vp, dtype=torch.int64, device=device)
        self.n_tok = torch.tensor(n_tok, dtype=torch.int32, device=device)
        self.desc = wk_store_desc(self.K_ptr.data_ptr(), self.V_ptr.data_ptr(), self.n_tok.data_ptr(),
                                  len(K_chunks), self.max_tok, self.H, self.d, self.dtype)


def wk_gather_window(store_desc: wk_store_desc, ids, n_ids, R_max, K_native, V_native, n_native, K_win, V_win,
                  win_capacity, n_win):
    """wk_gather_window."""
    st = lib().wk_gather_window(C.byref(store_desc), _dev(ids, "ids", torch.int32),
                                _dev(n_ids, "n_ids", torch.int32), R_max, _dev(K_native, "K_native"),
                                _dev(V_native, "V_native"), n_native, _dev(K_win, "K_win"), _dev(V_win, "V_win"),
                                win_capacity, _dev(n_win, "n_win", torch.int32), _stream())
    _check(st, "wk_gather_window")


def wk_attention_block_causal_workspace_bytes(H, N_q) -> int:
    return lib().wk_attention_block_causal_workspace_bytes(H, N_q)


def wk_attention_block_causal(Q, K_win, V_win, O, denoise_row0, frame_T, workspace, lse=None, N_kv=None, scale=0.0,
                              n_kv_dev=None):
    """wk_attention_block_causal.  The chunk's own keys are window rows [denoise_row0, denoise_row0 + N_q)."""
    H, N_q, d = Q.shape
    stride = K_win.shape[1]
    N_kv = stride if N_kv is None else N_kv
    st = lib().wk_attention_block_causal(_dev(Q, "Q"), _dev(K_win, "K_win", Q.dtype), _dev(V_win, "V_win", Q.dtype),
                                         _dev(O, "O", Q.dtype), _dev(lse, "lse", torch.float32), H, N_q, N_kv, d,
                                         stride, dtype_code(Q), scale, _dev(n_kv_dev, "n_kv_dev", torch.int32),
                                         denoise_row0, frame_T, _dev(workspace, "workspace"),
                                         0 if workspace is None else workspace.numel() * workspace.element_size(),
                                         _stream())
    _check(st, "wk_attention_block_causal")
    return O


def wk_chunk_lse(store_desc: wk_store_desc, Q, lse_out, scale=0.0):
    """wk_chunk_lse.  Q [H][N_q][d]; lse_out device float32 [M][H][N_q]."""
    st = lib().wk_chunk_lse(C.byref(store_desc), _dev(Q, "Q"), Q.shape[1], scale,
                            _dev(lse_out, "lse_out", torch.float32), _stream())
    _check(st, "wk_chunk_lse")
    return lse_out


def wk_attention_in_place(Q, K_native, V_native, n_native, store_desc: wk_store_desc, ids, n_ids, R_max, O, lse=None,
                          scale=0.0):
    """wk_attention_in_place.  K_native/V_native [H][stride][d] (or None with n_native = 0); ids/n_ids device int32."""
    stride = K_native.shape[1] if K_native is not None else 0
    st = lib().wk_attention_in_place(_dev(Q, "Q"), _dev(K_native, "K_native"), _dev(V_native, "V_native"), n_native,
                                     stride, C.byref(store_desc), _dev(ids, "ids", torch.int32),
                                     _dev(n_ids, "n_ids", torch.int32), R_max, _dev(O, "O"),
                                     _dev(lse, "lse", torch.float32), Q.shape[1], scale, _stream())
    _check(st, "wk_attention_in_place")
    return O


def wk_window_plan(desc: wk_window_desc, chunk_index: int) -> wk_window_step:
    """wk_window_plan (host)."""
    out = wk_window_step()
    _check(lib().wk_window_plan(C.byref(desc), chunk_index, C.byref(out)), "wk_window_plan")
    return out


def wk_window_update_workspace_bytes(R) -> int:
    return lib().wk_window_update_workspace_bytes(R)


def wk_window_update(store_desc: wk_store_desc, ids, n_ids, R, slot_tokens, slot_ids, n_native, K_win, V_win,
                     win_capacity, n_win, n_fetched, workspace, max_workgroups=0):
    """wk_window_update."""
    st = lib().wk_window_update(C.byref(store_desc), _dev(ids, "ids", torch.int32), _dev(n_ids, "n_ids", torch.int32),
                                R, slot_tokens, _dev(slot_ids, "slot_ids", torch.int32), n_native,
                                _dev(K_win, "K_win"), _dev(V_win, "V_win"), win_capacity,
                                _dev(n_win, "n_win", torch.int32), _dev(n_fetched, "n_fetched", torch.int32),
                                _dev(workspace, "workspace"),
                                0 if workspace is None else workspace.numel() * workspace.element_size(),
                                max_workgroups, _stream())
    _check(st, "wk_window_update")


def wk_prefetch_create(n_slots=2) -> int:
    """wk_prefetch_create -> opaque handle (an integer address)."""
    h = C.c_void_p()
    _check(lib().wk_prefetch_create(C.byref(h), n_slots), "wk_prefetch_create")
    return h.value


def wk_prefetch_destroy(p):
    _check(lib().wk_prefetch_destroy(p), "wk_prefetch_destroy")


def wk_prefetch_stream(p) -> int:
    """The copy stream as a raw hipStream_t; wrap with torch.cuda.ExternalStream to enqueue torch work."""
    return lib().wk_prefetch_stream(p)


def wk_prefetch_after(p, stream=None):
    _check(lib().wk_prefetch_after(p, _stream() if stream is None else stream), "wk_prefetch_after")


def wk_prefetch_gather(p, slot, store_desc: wk_store_desc, ids, n_ids, R_max, K_native, V_native, n_native, K_win,
                       V_win, win_capacity, n_win, max_workgroups=0):
    st = lib().wk_prefetch_gather(p, slot, C.byref(store_desc), _dev(ids, "ids", torch.int32),
                                  _dev(n_ids, "n_ids", torch.int32), R_max, _dev(K_native, "K_native"),
                                  _dev(V_native, "V_native"), n_native, _dev(K_win, "K_win"), _dev(V_win, "V_win"),
                                  win_capacity, _dev(n_win, "n_win", torch.int32), max_workgroups)
    _check(st, "wk_prefetch_gather")


def wk_prefetch_acquire(p, slot, stream=None):
    _check(lib().wk_prefetch_acquire(p, slot, _stream() if stream is None else stream), "wk_prefetch_acquire")


def wk_prefetch_release(p, slot, stream=None):
    _check(lib().wk_prefetch_release(p, slot, _stream() if stream is None else stream), "wk_prefetch_release")


def wk_calibration_copy(dst, src):
    """wk_calibration_copy: plain device copy of src into dst (same byte size)."""
    n = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() == n
    _check(lib().wk_calibration_copy(_dev(dst, "dst"), _dev(src, "src"), n, _stream()), "wk_calibration_copy")


def wk_attention_workspace_bytes(H, N_q, N_kv, dtype) -> int:
    return lib().wk_attention_workspace_bytes(H, N_q, N_kv, dtype)


def wk_attention(Q, K_win, V_win, O, lse=None, N_kv=None, scale=0.0, n_kv_dev=None, workspace=None):
    """wk_attention.  Q [H][N_q][d]; K_win/V_win [H][stride][d]; O like Q (written in place).
    O = None (then V_win may be None too) asks for lse only."""
    H, N_q, d = Q.shape
    stride = K_win.shape[1]
    N_kv = stride if N_kv is None else N_kv
    st = lib().wk_attention(_dev(Q, "Q"), _dev(K_win, "K_win", Q.dtype),
                            None if V_win is None else _dev(V_win, "V_win", Q.dtype),
                            None if O is None else _dev(O, "O", Q.dtype), _dev(lse, "lse", torch.float32), H, N_q, N_kv, d, stride,
                            dtype_code(Q), scale, _dev(n_kv_dev, "n_kv_dev", torch.int32),
                            _dev(workspace, "workspace"),
                            0 if workspace is None else workspace.numel() * workspace.element_size(), _stream())
    _check(st, "wk_attention")
    return O
