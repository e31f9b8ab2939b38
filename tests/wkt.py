"""Helpers shared by the GPU parity tests (no arithmetic of the method lives here)."""
import numpy as np
import torch

TIE_BAND = 1e-6     # selections may differ from the oracle only among scores closer than this
ATT_MAX_ABS_BF16, ATT_MEAN_ABS_BF16 = 2e-2, 2e-3   # bf16 inputs, fp32 accumulation
ATT_MAX_ABS_F32 = 1e-5
# Scale-aware bars for bf16 attention at the full-size windows, where the outputs themselves are small
# (rms ~ sqrt(e / N_kv) for i.i.d. inputs) and the absolute bars above would let a lost key tile pass.
# One rounding of O to bf16 and the bf16-rounded weights each give a relative error of rms ~1e-3 per
# element; measured on every full-size window: row-relative L2 error 2.4e-3 (max 3.1e-3), max-abs 0.013-0.019
# of the rows' rms, lse 2.5e-5 .. 1.2e-4.
ATT_ROW_REL_L2_BF16 = 6e-3      # per (head, row): |o_gpu - o_ref|_2 / |o_ref|_2
ATT_MAX_ABS_OVER_RMS_BF16 = 5e-2
ATT_LSE_ABS_BF16_FULL = 5e-4


def dev():
    return torch.device("cuda:0")


def bits(t: torch.Tensor) -> torch.Tensor:
    """Reinterpret as integers for byte-exact comparison."""
    return t.contiguous().view(torch.int16 if t.element_size() == 2 else torch.int32)


def assert_selection_matches(gpu_idx, oracle_idx, oracle_scores, what=""):
    """Bit-exact index sets, except members whose fp64 scores lie within TIE_BAND of the cut.

    gpu_idx / oracle_idx: ascending indices into the scored list; oracle_scores: fp64 per item."""
    g, o = np.asarray(gpu_idx), np.asarray(oracle_idx)
    assert g.size == o.size, f"{what}: kept {g.size} items, oracle kept {o.size}"
    assert np.all(np.diff(g) > 0), f"{what}: indices not strictly ascending"
    if np.array_equal(g, o):
        return
    s = np.asarray(oracle_scores, np.float64)
    kept_max = s[o].max()
    dropped = np.setdiff1d(np.arange(s.size), o)
    dropped_min = s[dropped].min()
    extra = np.setdiff1d(g, o)      # taken by the GPU, dropped by the oracle
    missing = np.setdiff1d(o, g)    # kept by the oracle, dropped by the GPU
    assert np.all(s[extra] - kept_max < TIE_BAND), f"{what}: GPU kept an item clearly above the cut"
    assert np.all(dropped_min - s[missing] < TIE_BAND), f"{what}: GPU dropped an item clearly below the cut"


def attention_errors(O_gpu: torch.Tensor, ref: np.ndarray):
    got = O_gpu.detach().float().cpu().numpy().astype(np.float64)
    err = np.abs(got - ref)
    return float(err.max()), float(err.mean())


def sample_rows(N_q: int, tile: int, n_random: int, seed: int) -> np.ndarray:
    """First and last row of every `tile`-row block plus n_random random rows (sorted, unique)."""
    edges = [r for t in range(0, N_q, tile) for r in (t, min(t + tile, N_q) - 1)]
    rng = np.random.default_rng(seed)
    rnd = rng.integers(0, N_q, n_random).tolist()
    return np.unique(np.array(edges + rnd, np.int32))


def scale_aware_errors(got: np.ndarray, ref: np.ndarray):
    """(worst row-relative L2 error, max-abs error over the rms of ref) of outputs [H][rows][d]."""
    err = got - ref
    row_rel = np.sqrt((err ** 2).sum(-1) / np.maximum((ref ** 2).sum(-1), 1e-300))
    rms = float(np.sqrt((ref ** 2).mean()))
    return float(row_rel.max()), float(np.abs(err).max() / rms)


def assert_attention_close_bf16(got, ref, lse_got=None, lse_ref=None, full_size=False, what=""):
    """bf16 attention outputs against the oracle: the contract's absolute bars, and for the full-size windows
    the scale-aware ones (per-row relative error, max-abs against the rows' rms, tight lse).
    got: tensor or array [H][rows][d]; ref: float64 array of the same shape."""
    if isinstance(got, torch.Tensor):
        got = got.detach().float().cpu().numpy()
    got = np.asarray(got, np.float64)
    err = np.abs(got - ref)
    mx, mean = float(err.max()), float(err.mean())
    assert mx <= ATT_MAX_ABS_BF16 and mean <= ATT_MEAN_ABS_BF16, (what, mx, mean)
    if full_size:
        row_rel, max_rms = scale_aware_errors(got, ref)
        assert row_rel <= ATT_ROW_REL_L2_BF16, (what, "row-relative L2 error", row_rel)
        assert max_rms <= ATT_MAX_ABS_OVER_RMS_BF16, (what, "max-abs / rms", max_rms)
    if lse_got is not None:
        if isinstance(lse_got, torch.Tensor):
            lse_got = lse_got.detach().float().cpu().numpy()
        le = float(np.abs(np.asarray(lse_got, np.float64) - lse_ref).max())
        assert le <= (ATT_LSE_ABS_BF16_FULL if full_size else 2e-2), (what, "lse", le)
    return mx, mean
