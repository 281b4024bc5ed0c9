"""The five synthetic workloads (shapes, length distributions, pool sizes) and scaled-down variants.

Each config is a recipe, not data: ``make_sessions`` / ``make_attn_inputs`` turn it into arrays with
``numpy.random.default_rng(1000 + index)``.  Where the benchmark spec leaves a size open (pool sizes of
configs 3-5) the value chosen here is the one stated in the design notes.
"""
from __future__ import annotations

import dataclasses
import math
from dataclasses import dataclass
from typing import Optional, Tuple


@dataclass(frozen=True)
class WorkloadConfig:
    name: str
    index: int                      # 0-based position in the benchmark's config list
    dtype: str                      # "bf16" or "fp32"
    n_layers: int                   # layers moved by pack / unpack
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    block_size: int
    n_blocks: int                   # physical blocks in each per-layer K pool and V pool
    n_sessions: int
    # ("const", n) | ("uniform", lo, hi) | ("geometric", mean, lo, hi)  [geometric forces a partial last block]
    prefix_dist: Tuple
    # ("const", n) | ("lognormal", median, sigma, lo, hi) | ("mixed", n_decode, median, sigma, lo, hi)
    new_dist: Tuple
    sigma: float                    # std-dev of Q, K, V
    scale: float                    # softmax scale
    attn_layer: int = 0             # which layer the one-layer attention runs on
    fresh_tables: bool = True       # also draw a destination table from unused blocks
    note: str = ""

    @property
    def elem_bytes(self) -> int:
        return 2 if self.dtype == "bf16" else 4

    @property
    def row_elems(self) -> int:
        """Elements of one token's K (or V) for one layer."""
        return self.n_kv_heads * self.head_dim

    @property
    def block_elems(self) -> int:
        return self.block_size * self.row_elems

    @property
    def layer_elems(self) -> int:
        return self.n_blocks * self.block_elems

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def seed(self) -> int:
        return 1000 + self.index

    def kv_bytes_per_token(self) -> int:
        """K and V of every layer for one token."""
        return 2 * self.n_layers * self.row_elems * self.elem_bytes


_8B = dict(n_q_heads=32, n_kv_heads=8, head_dim=128, block_size=16, dtype="bf16", scale=1.0 / math.sqrt(128.0))

CONFIGS = (
    WorkloadConfig(
        name="tiny_fp32", index=0, dtype="fp32", n_layers=1, n_q_heads=4, n_kv_heads=2, head_dim=64,
        block_size=16, n_blocks=48, n_sessions=1, prefix_dist=("const", 256), new_dist=("const", 32),
        sigma=1.0, scale=0.125, fresh_tables=True,
        note="1 session owns 16 of 48 blocks (first 16 of a seeded permutation)"),
    WorkloadConfig(
        name="llama8b", index=1, n_layers=32, n_blocks=65536, n_sessions=16,
        prefix_dist=("uniform", 1024, 8192), new_dist=("lognormal", 128.0, 1.0, 16, 1024),
        sigma=0.5, note="fragmented 64K-block pool; the configuration the headline metric is quoted on", **_8B),
    WorkloadConfig(
        name="llama70b_long", index=2, dtype="bf16", n_layers=80, n_q_heads=64, n_kv_heads=8, head_dim=128,
        block_size=16, n_blocks=8192, n_sessions=1, prefix_dist=("const", 32768), new_dist=("const", 512),
        sigma=1.0, scale=1.0 / math.sqrt(128.0), note="pool size chosen: 8192 blocks (40 GiB)"),
    WorkloadConfig(
        name="many_short", index=3, n_layers=32, n_blocks=32768, n_sessions=256,
        prefix_dist=("geometric", 600.0, 16, 4096), new_dist=("const", 64),
        sigma=1.0, note="pool size chosen: 32768 blocks so that a fresh destination list fits", **_8B),
    WorkloadConfig(
        name="mixed_resume", index=4, n_layers=1, n_blocks=81920, n_sessions=128,
        prefix_dist=("uniform", 512, 16384), new_dist=("mixed", 96, 256.0, 0.8, 2, 2048),
        sigma=1.0, fresh_tables=False, note="attention batch over a one-layer pool of 80Ki blocks", **_8B),
)

# The eight sessions that arrive while config 5's attention runs: unpack only.
MIXED_RESUME_INCOMING = WorkloadConfig(
    name="mixed_resume_incoming", index=4, n_layers=32, n_blocks=4096, n_sessions=8,
    prefix_dist=("const", 4096), new_dist=("const", 0), sigma=1.0, fresh_tables=True,
    note="8 incoming sessions x 4096 tokens, 32 layers, pool of 4096 blocks (8 GiB)", **_8B)

_BY_NAME = {c.name: c for c in CONFIGS}
_BY_NAME[MIXED_RESUME_INCOMING.name] = MIXED_RESUME_INCOMING


def get_config(key) -> WorkloadConfig:
    """Look a config up by name or by 0-based index."""
    if isinstance(key, int):
        return CONFIGS[key]
    return _BY_NAME[key]


def _scale_dist(dist: Tuple, f: float, floor: int) -> Tuple:
    kind = dist[0]
    s = lambda v: max(floor, int(round(v * f)))
    if kind == "const":
        return ("const", s(dist[1]) if dist[1] > 0 else 0)
    if kind == "uniform":
        return ("uniform", s(dist[1]), max(s(dist[1]), s(dist[2])))
    if kind == "geometric":
        return ("geometric", max(1.0, dist[1] * f), dist[2], max(dist[2] + 1, s(dist[3])))
    if kind == "lognormal":
        lo = s(dist[3])
        return ("lognormal", max(1.0, dist[1] * f), dist[2], lo, max(lo, s(dist[4])))
    if kind == "mixed":
        return ("mixed", dist[1], max(1.0, dist[2] * f), dist[3], dist[4], max(dist[4], s(dist[5])))
    raise ValueError(kind)


def scaled_config(cfg: WorkloadConfig, *, n_layers: Optional[int] = None, n_sessions: Optional[int] = None,
                  prefix_scale: float = 1.0, new_scale: float = 1.0, n_blocks: Optional[int] = None,
                  n_decode: Optional[int] = None) -> WorkloadConfig:
    """Same recipe, smaller numbers: the parity tests run the oracle on these in seconds."""
    new_dist = _scale_dist(cfg.new_dist, new_scale, 1)
    if new_dist[0] == "mixed" and n_decode is not None:
        new_dist = ("mixed", n_decode) + tuple(new_dist[2:])
    return dataclasses.replace(
        cfg,
        name=cfg.name + "_scaled",
        n_layers=n_layers if n_layers is not None else cfg.n_layers,
        n_sessions=n_sessions if n_sessions is not None else cfg.n_sessions,
        n_blocks=n_blocks if n_blocks is not None else cfg.n_blocks,
        prefix_dist=_scale_dist(cfg.prefix_dist, prefix_scale, 1),
        new_dist=new_dist,
        attn_layer=min(cfg.attn_layer, (n_layers if n_layers is not None else cfg.n_layers) - 1),
    )
