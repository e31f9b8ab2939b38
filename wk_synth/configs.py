"""The five synthetic workloads (shapes only; no arithmetic of the method)."""
from dataclasses import dataclass, replace

# enum values mirror include/wk.h (plain integers so that neither the oracle
# nor the HIP binding has to import the other to read a config)
DT_F32, DT_BF16 = 0, 1
HEADS_SHARED, HEADS_INDEPENDENT = 0, 1
ANCHOR_FIRST_FRAME, ANCHOR_EXTERNAL = 0, 1
RATIO_CHUNK, RATIO_NONANCHOR = 0, 1


@dataclass(frozen=True)
class WkConfig:
    name: str
    index: int
    H: int                 # attention heads
    d: int                 # head dimension
    T: int                 # tokens per latent frame
    F: int                 # latent frames per stored chunk
    dtype: int             # DT_F32 / DT_BF16
    q_frames: int          # frames in the denoising (query) chunk
    native_frames: int     # frames of the native sliding window
    M: int                 # chunks in the store
    R: int                 # retrieval budget
    rho: float             # keep ratio
    ratio_kind: int        # RATIO_CHUNK: rho of the whole chunk; RATIO_NONANCHOR: P of Sec. 4.3
    anchor_mode: int
    head_mode: int = HEADS_SHARED
    store: str = "device"  # "device" or "pinned"
    n_kv_override: int = 0  # config 3: plain attention over this many keys

    @property
    def seed(self) -> int:
        return 22718 * 100 + self.index

    @property
    def N_q(self) -> int:
        return self.q_frames * self.T

    @property
    def n_native(self) -> int:
        return self.native_frames * self.T

    @property
    def chunk_tokens(self) -> int:
        return self.F * self.T

    def with_(self, **kw) -> "WkConfig":
        return replace(self, **kw)


CONFIGS = [
    # 0: tiny fp32 case the oracle finishes in seconds
    WkConfig("tiny_f32", 0, H=4, d=128, T=880, F=1, dtype=DT_F32, q_frames=1, native_frames=2,
             M=16, R=2, rho=0.5, ratio_kind=RATIO_CHUNK, anchor_mode=ANCHOR_EXTERNAL),
    # 1: Matrix-Game-2.0-shaped
    WkConfig("matrix_game", 1, H=12, d=128, T=880, F=3, dtype=DT_BF16, q_frames=3, native_frames=6,
             M=60, R=4, rho=0.5, ratio_kind=RATIO_CHUNK, anchor_mode=ANCHOR_FIRST_FRAME),
    # 2: LingBot-World-Fast-shaped, store in pinned host memory
    WkConfig("lingbot", 2, H=40, d=128, T=1560, F=3, dtype=DT_BF16, q_frames=3, native_frames=6,
             M=120, R=8, rho=0.5, ratio_kind=RATIO_CHUNK, anchor_mode=ANCHOR_FIRST_FRAME,
             store="pinned"),
    # 3: full-KV attention after a one-minute rollout (240 frames x 880 tokens)
    WkConfig("full_kv", 3, H=12, d=128, T=880, F=3, dtype=DT_BF16, q_frames=3, native_frames=240,
             M=0, R=0, rho=1.0, ratio_kind=RATIO_CHUNK, anchor_mode=ANCHOR_FIRST_FRAME,
             n_kv_override=240 * 880),
    # 4: compression / retrieval stress at the LingBot shape
    WkConfig("stress", 4, H=40, d=128, T=1560, F=3, dtype=DT_BF16, q_frames=3, native_frames=0,
             M=1000, R=16, rho=0.25, ratio_kind=RATIO_NONANCHOR, anchor_mode=ANCHOR_FIRST_FRAME,
             store="pinned"),
]


def get_config(i: int) -> WkConfig:
    return CONFIGS[i]
