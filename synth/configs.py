"""Shapes of the five benchmark configurations (synthetic stand-ins for the paper's
video-QA workloads: one carrier token after N visual tokens per frame, a cache of
[text prefix | one carrier row per earlier frame])."""
from dataclasses import dataclass


@dataclass(frozen=True)
class AttnShape:
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    dtype: str  # "f32" or "bf16"

    @property
    def scale(self) -> float:
        return float(self.head_dim) ** -0.5

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads


QWEN7B = AttnShape(28, 4, 128, "bf16")

CONFIGS = {
    # tiny fp32 single layer: 16 retained rows, one frame of 49 visual tokens + carrier
    "cfg1": dict(shape=AttnShape(4, 1, 64, "f32"), seed=0, prefix=16, n_visual=49, hidden=256,
                 frames=1, layers=1, sigma=1.0),
    # single layer, 200-row text prefix, 64 frames of 169+1 tokens streamed with compaction
    "cfg2": dict(shape=QWEN7B, seed=1, prefix=200, n_visual=169, frames=64, layers=1, sigma=0.5),
    # long stream: 28 layers, 200 prefix + 4096 carrier rows already retained, 256 more frames
    "cfg3": dict(shape=QWEN7B, seed=2, prefix=200 + 4096, n_visual=169, frames=256, layers=28,
                 sigma=0.5),
    # decode: 16 ragged streams, carrier cache U[512,8192] + 128 text rows, 64 steps, 28 layers
    "cfg4": dict(shape=QWEN7B, seed=3, streams=16, carrier_lo=512, carrier_hi=8192, text_hist=128,
                 steps=64, layers=28, sigma=0.5),
    # uncompressed contrast: dense cache of 64*169 visual rows + 200 prefix vs 264 carrier-only rows
    "cfg5": dict(shape=QWEN7B, seed=4, dense_rows=64 * 169 + 200, compact_rows=264, n_visual=169,
                 layers=1, sigma=0.5),
}
