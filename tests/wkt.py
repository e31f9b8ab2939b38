"""Helpers shared by the GPU parity tests (no arithmetic of the method lives here)."""
import numpy as np
import torch

TIE_BAND = 1e-6     # selections may differ from the oracle only among scores closer than this
ATT_MAX_ABS_BF16, ATT_MEAN_ABS_BF16 = 2e-2, 2e-3   # bf16 inputs, fp32 accumulation
ATT_MAX_ABS_F32 = 1e-5


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
