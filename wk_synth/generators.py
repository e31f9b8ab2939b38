"""Counter-based seeded generators (torch ops, run on CPU or on the GPU).

Every tensor is a pure function of (seed, stream, element index), so a slice
of a large tensor can be regenerated without the rest and the same call gives
the same bits on the same device type.  Tests always hand the *same bytes* to
the oracle and to the HIP path (generate once, copy), so CPU/GPU differences
in libm rounding never matter.
"""
import math

import numpy as np
import torch

from .configs import (ANCHOR_EXTERNAL, DT_BF16, DT_F32, WkConfig)

_M32 = 0xFFFFFFFF
_C1 = 0x7FEB352D  # odd multipliers below 2**31 keep every int64 product exact
_C2 = 0x31848BAB
_C3 = 0x632BE5AB


def torch_dtype(dt: int) -> torch.dtype:
    return {DT_F32: torch.float32, DT_BF16: torch.bfloat16}[dt]


def _mix_int(x: int) -> int:
    x &= _M32
    x ^= x >> 16
    x = (x * _C1) & _M32
    x ^= x >> 15
    x = (x * _C2) & _M32
    x ^= x >> 16
    return x


def _stream_key(seed: int, stream) -> int:
    """Fold a seed and a tuple of small integers into a 32-bit key."""
    k = _mix_int(seed ^ 0x5BD1E995)
    if isinstance(stream, int):
        stream = (stream,)
    for s in stream:
        k = _mix_int(k * 31 + int(s) + 0x9E3779B1)
    return k


def _mix_t(x: torch.Tensor) -> torch.Tensor:
    # x: int64 holding values in [0, 2**32)
    x = x ^ (x >> 16)
    x = (x * _C1) & _M32
    x = x ^ (x >> 15)
    x = (x * _C2) & _M32
    x = x ^ (x >> 16)
    return x


def _u32(seed: int, stream, counters: torch.Tensor) -> torch.Tensor:
    """32-bit hash of int64 counters (values below 2**62)."""
    key = _stream_key(seed, stream)
    lo = counters & _M32
    hi = counters >> 32
    h = _mix_t(lo ^ key)
    h = _mix_t((h + hi * _C3 + (key >> 7)) & _M32)
    return h


def uniform(seed: int, stream, shape, device="cpu") -> torch.Tensor:
    """U[0,1) float32, one value per element index."""
    n = int(np.prod(shape)) if len(shape) else 1
    idx = torch.arange(n, dtype=torch.int64, device=device)
    h = _u32(seed, stream, idx)
    return (h.to(torch.float32) * (1.0 / 4294967296.0)).clamp_(max=1.0 - 2.0 ** -24).reshape(shape)


def normal(seed: int, stream, shape, device="cpu", block: int = 1 << 24) -> torch.Tensor:
    """N(0,1) float32 by Box-Muller on two hashed uniforms per element."""
    n = int(np.prod(shape)) if len(shape) else 1
    out = torch.empty(n, dtype=torch.float32, device=device)
    for s in range(0, n, block):
        e = min(n, s + block)
        idx = torch.arange(s, e, dtype=torch.int64, device=device)
        h1 = _u32(seed, stream, idx * 2)
        h2 = _u32(seed, stream, idx * 2 + 1)
        u1 = (h1.to(torch.float32) + 1.0) * (1.0 / 4294967296.0)   # (0, 1]
        u2 = h2.to(torch.float32) * (1.0 / 4294967296.0)
        r = torch.sqrt(-2.0 * torch.log(u1))
        out[s:e] = r * torch.cos((2.0 * math.pi) * u2)
    return out.reshape(shape)


# stream tags
_S_Q, _S_NATK, _S_NATV = 1, 2, 3
_S_ANCK, _S_ANCV, _S_FRK, _S_FRV, _S_NOK, _S_NOV, _S_MASK = 10, 11, 12, 13, 14, 15, 16
_S_POSE, _S_ACT = 20, 21
_S_REVK, _S_REVA = 30, 31


def make_queries(cfg: WkConfig, device="cpu", n_q=None) -> torch.Tensor:
    """Q [H][N_q][d] ~ N(0,1), rounded to the config dtype."""
    n_q = cfg.N_q if n_q is None else n_q
    return normal(cfg.seed, _S_Q, (cfg.H, n_q, cfg.d), device).to(torch_dtype(cfg.dtype))


def make_native(cfg: WkConfig, device="cpu", n_rows=None):
    """Native sliding-window frames: K, V [H][n_native][d] ~ N(0,1)."""
    n = cfg.n_native if n_rows is None else n_rows
    dt = torch_dtype(cfg.dtype)
    k = normal(cfg.seed, _S_NATK, (cfg.H, n, cfg.d), device).to(dt)
    v = normal(cfg.seed, _S_NATV, (cfg.H, n, cfg.d), device).to(dt)
    return k, v


def make_chunk(cfg: WkConfig, chunk_id: int, device="cpu", sigma: float = 0.05, p_copy: float = 0.5):
    """One evicted chunk with temporal redundancy.

    Returns (K, V, K_anchor) where K, V are [H][F*T][d].  With the first-frame
    anchor the anchor is frame 0 of K and K_anchor is None; with an external
    anchor (one-frame chunks) K_anchor is a separate [H][T][d] tensor and every
    chunk token is a candidate.  Each non-anchor token at in-frame position p
    is, with probability p_copy (one draw per token, shared by all heads and by
    K and V), the anchor token at p plus N(0, sigma) noise; otherwise fresh N(0,1).
    """
    H, T, F, d = cfg.H, cfg.T, cfg.F, cfg.d
    dt = torch_dtype(cfg.dtype)
    anc_k = normal(cfg.seed, (_S_ANCK, chunk_id), (H, T, d), device)
    anc_v = normal(cfg.seed, (_S_ANCV, chunk_id), (H, T, d), device)
    external = cfg.anchor_mode == ANCHOR_EXTERNAL
    frames_k, frames_v = ([], []) if external else ([anc_k], [anc_v])
    first = 0 if external else 1
    for f in range(first, F):
        fk = normal(cfg.seed, (_S_FRK, chunk_id, f), (H, T, d), device)
        fv = normal(cfg.seed, (_S_FRV, chunk_id, f), (H, T, d), device)
        nk = normal(cfg.seed, (_S_NOK, chunk_id, f), (H, T, d), device) * sigma
        nv = normal(cfg.seed, (_S_NOV, chunk_id, f), (H, T, d), device) * sigma
        m = (uniform(cfg.seed, (_S_MASK, chunk_id, f), (T,), device) < p_copy).view(1, T, 1)
        frames_k.append(torch.where(m, anc_k + nk, fk))
        frames_v.append(torch.where(m, anc_v + nv, fv))
    K = torch.cat(frames_k, dim=1).to(dt).contiguous()
    V = torch.cat(frames_v, dim=1).to(dt).contiguous()
    K_anchor = anc_k.to(dt).contiguous() if external else None
    return K, V, K_anchor


def make_revisit_keys(cfg: WkConfig, Q: torch.Tensor, lens, device="cpu"):
    """Stored key chunks for query-based retrieval, some of which "see" what the current queries see.

    Chunk c has lens[c] keys per head: N(0,1) noise plus a_c times a query row (row (7*j + c) mod N_q
    for key j), with a_c drawn uniformly from [0, 0.6] per chunk -- a revisited viewpoint has keys
    aligned with the current queries (a_c large), an unrelated one has not (a_c near 0).  Returns the
    list of [H][lens[c]][d] tensors in the config dtype and the numpy array of the a_c.
    """
    H, N_q, d = Q.shape
    a = uniform(cfg.seed, _S_REVA, (len(lens),), "cpu").double().numpy() * 0.6
    out = []
    Qf = Q.to(device=device, dtype=torch.float32)
    for c, n in enumerate(lens):
        rows = (7 * torch.arange(n, device=device) + c) % N_q
        k = normal(cfg.seed, (_S_REVK, c), (H, n, d), device) + float(a[c]) * Qf[:, rows]
        out.append(k.to(torch_dtype(cfg.dtype)).contiguous())
    return out, a


def make_poses(M: int, seed: int):
    """Looping camera trajectory: poses [M][5] float32 (x, y, z, yaw, pitch; radians) and
    the current pose [5].

    A random walk of ceil(M/2) steps (unit step along the heading, yaw jitter
    10 deg, pitch jitter 3 deg clamped to +-30 deg) followed by the same poses
    retraced in reverse with small jitter, so the walk ends where it began; the
    current pose is pose 0 plus jitter.  The chunks nearest to the current pose
    are therefore chunk 0 and chunk M-1 (a planted loop closure).
    """
    if M == 0:
        return np.zeros((0, 5), np.float32), np.zeros(5, np.float32)
    half = (M + 1) // 2
    g = normal(seed, _S_POSE, (half, 2), "cpu").double().numpy()
    jit = normal(seed, (_S_POSE, 1), (M + 1, 5), "cpu").double().numpy() * 0.01
    x = y = z = yaw = pitch = 0.0
    fwd = np.zeros((half, 5))
    for i in range(half):
        fwd[i] = (x, y, z, yaw, pitch)
        yaw += math.radians(10.0) * g[i, 0]
        pitch = float(np.clip(pitch + math.radians(3.0) * g[i, 1], -math.radians(30), math.radians(30)))
        x += math.sin(yaw)
        z += math.cos(yaw)
        y += 0.1 * math.sin(pitch)
    poses = np.zeros((M, 5))
    poses[:half] = fwd
    for i in range(half, M):
        poses[i] = fwd[M - 1 - i] + jit[i]
    cur = fwd[0] + jit[M] * 0.1
    return poses.astype(np.float32), cur.astype(np.float32)


def make_action_labels(n: int, seed: int, n_classes: int = 8) -> np.ndarray:
    """n discrete action labels, uniform over n_classes, int32."""
    u = uniform(seed, _S_ACT, (n,), "cpu").double().numpy()
    return np.minimum((u * n_classes).astype(np.int32), n_classes - 1)
