"""The five synthetic workloads: shapes, scale schedules, roles and budgets.

These tables are *inputs* to the hot path.  The paper measures on Infinity-2B
and Infinity-8B with real prompts; neither the weights nor the prompts exist
here, so every workload below is a seeded stand-in that keeps the model's
shape (layers, heads, head_dim), the multi-scale token schedule (each scale k
adds h_k*w_k tokens, Sec. 3.1 and the introduction's cache-growth argument)
and the drafter/refiner budget asymmetry (Sec. 3.3, Eq. 4: B_d >> B_r).

Nothing here performs scoring, selection or attention.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Sequence, Tuple

_M64 = (1 << 64) - 1


def _mix64(x: int) -> int:
    """splitmix64 output function on a Python int (mod 2^64)."""
    x &= _M64
    x = ((x ^ (x >> 30)) * 0xBF58476D1CE4E5B9) & _M64
    x = ((x ^ (x >> 27)) * 0x94D049BB133111EB) & _M64
    return (x ^ (x >> 31)) & _M64


def stream_key(seed: int, tensor_id: int, layer: int = 0, scale: int = 0, extra: int = 0) -> int:
    """64-bit key naming one random stream; every tensor gets its own."""
    k = _mix64(seed + 0x9E3779B97F4A7C15)
    for part in (tensor_id, layer, scale, extra):
        k = _mix64(k ^ _mix64(part + 0x632BE59BD9B4E019))
    return k


@dataclass(frozen=True)
class WorkloadConfig:
    name: str
    dtype: str                 # "f32" | "bf16" storage dtype of Q/K/V
    n_seq: int                 # batch rows; classifier-free-guidance pairs are separate rows
    n_layer: int
    n_head: int
    head_dim: int
    prefix: int                # text-prefix tokens already cached before scale 1
    sides: Tuple[int, ...]     # side length of each scale's square token map
    window: int                # observation-window size N (Sec. 3.3: typically 16)
    recipe: str                # value distribution, see generator.py
    n_drafter: int             # drafter layers per scale
    drafter_frac: float = 0.0  # budget as a fraction of the uncompressed cache length
    refiner_frac: float = 0.0
    drafter_abs: int = 0       # absolute budgets (config 0); used when > 0
    refiner_abs: int = 0
    fixed_roles: Tuple[int, ...] = ()   # if set: layer ids that are drafters at every scale
    first_compressed_scale: int = 3     # 1-based; earlier scales keep everything
    seed: int = 0

    @property
    def n_scale(self) -> int:
        return len(self.sides)

    def n_tokens(self, k: int) -> int:
        """h_k * w_k tokens of scale k (1-based)."""
        return self.sides[k - 1] ** 2

    @property
    def image_tokens(self) -> int:
        return sum(s * s for s in self.sides)

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2


_SIDES_512 = (1, 2, 4, 6, 8, 12, 16, 20, 24, 32)
_SIDES_1024 = (1, 2, 4, 6, 8, 12, 16, 20, 24, 32, 40, 48, 64)

CONFIGS = {
    # configs[0]: the CPU-seconds case.
    "tiny": WorkloadConfig(
        name="tiny", dtype="f32", n_seq=1, n_layer=2, n_head=2, head_dim=64, prefix=16,
        sides=(1, 2, 4, 8), window=8, recipe="iid_small", n_drafter=1,
        drafter_abs=32, refiner_abs=8, fixed_roles=(0,)),
    # configs[1]: Infinity-2B-shaped 512^2, batch 1.
    "2b_512": WorkloadConfig(
        name="2b_512", dtype="bf16", n_seq=1, n_layer=32, n_head=16, head_dim=128, prefix=64,
        sides=_SIDES_512, window=16, recipe="lowrank8", n_drafter=8,
        drafter_frac=0.20, refiner_frac=0.05),
    # configs[2]: Infinity-2B-shaped 1024^2, batch 8 with CFG rows -> 16 sequences. Main bench.
    # 8 drafters at 25 % and 24 refiners at 5 % give (8*25 + 24*5)/32 = 10 % retained overall.
    "2b_1024": WorkloadConfig(
        name="2b_1024", dtype="bf16", n_seq=16, n_layer=32, n_head=16, head_dim=128, prefix=64,
        sides=_SIDES_1024, window=16, recipe="lowrank8", n_drafter=8,
        drafter_frac=0.25, refiner_frac=0.05),
    # configs[3]: 8B-class shape, heavy-tailed keys.
    "8b_1024": WorkloadConfig(
        name="8b_1024", dtype="bf16", n_seq=16, n_layer=40, n_head=32, head_dim=128, prefix=128,
        sides=_SIDES_1024, window=16, recipe="student_t3", n_drafter=10,
        drafter_frac=0.25, refiner_frac=0.05),
    # configs[4]: only the 64x64 scale of the 2b_1024 shape against a generated prefix.
    "final_scale": WorkloadConfig(
        name="final_scale", dtype="bf16", n_seq=16, n_layer=1, n_head=16, head_dim=128, prefix=64,
        sides=_SIDES_1024, window=16, recipe="dominant", n_drafter=0),
    # small bf16 case for the calibrated-policy chain (ASI -> drafter set -> budgets -> steps):
    # few enough units that the fp64 oracle can follow every one of them.
    "calib_small": WorkloadConfig(
        name="calib_small", dtype="bf16", n_seq=2, n_layer=6, n_head=4, head_dim=128, prefix=32,
        sides=(1, 2, 4, 6, 8, 12, 16), window=16, recipe="lowrank8", n_drafter=2,
        drafter_frac=0.25, refiner_frac=0.05),
}

FINAL_SCALE_BUDGET_FRACS = (0.05, 0.10, 0.20, 1.00)


def get_config(name: str) -> WorkloadConfig:
    return CONFIGS[name]


def c_full(cfg: WorkloadConfig, k: int) -> int:
    """Cache length entering scale k (1-based) when nothing was ever evicted:
    the text prefix plus every earlier token map (introduction: each scale
    contributes h_k x w_k entries)."""
    return cfg.prefix + sum(cfg.n_tokens(j) for j in range(1, k))


def round_half_up(x: float) -> int:
    return int(x + 0.5)


def layer_roles(cfg: WorkloadConfig, k: int) -> List[bool]:
    """is_drafter per layer at scale k.  The paper ranks (layer, scale) pairs
    by a calibrated statistic (Eq. 3); calibration needs the trained model, so
    the drafter set of each scale is a seeded draw of the configured size."""
    if cfg.fixed_roles:
        return [l in cfg.fixed_roles for l in range(cfg.n_layer)]
    ranked = sorted(range(cfg.n_layer), key=lambda l: stream_key(cfg.seed, 0x701E, l, k))
    chosen = set(ranked[: cfg.n_drafter])
    return [l in chosen for l in range(cfg.n_layer)]


def budget_table(cfg: WorkloadConfig) -> List[List[int]]:
    """budget[l][k-1] in tokens per head (the unit of Sec. 4.3's "650 tokens
    per head/layer").  Scales before `first_compressed_scale` get a budget that
    is >= the cache length, i.e. keep everything."""
    table = [[0] * cfg.n_scale for _ in range(cfg.n_layer)]
    for k in range(1, cfg.n_scale + 1):
        roles = layer_roles(cfg, k)
        full = c_full(cfg, k)
        for l in range(cfg.n_layer):
            if k < cfg.first_compressed_scale:
                b = full
            elif cfg.drafter_abs > 0:
                b = cfg.drafter_abs if roles[l] else cfg.refiner_abs
            else:
                frac = cfg.drafter_frac if roles[l] else cfg.refiner_frac
                b = max(1, round_half_up(frac * full))
            table[l][k - 1] = b
    return table


def window_indices(cfg: WorkloadConfig, n_k: int) -> List[int]:
    """Observation window = the last min(N, n_k) tokens of the scale in raster
    order (the paper's patch-centroid sampling is replaced by this fixed list;
    the hot path takes the window as an explicit index list either way)."""
    n = min(cfg.window, n_k)
    return list(range(n_k - n, n_k))


@dataclass
class StepPlan:
    layer: int
    scale: int          # 1-based
    n_cur: int
    budget: int
    is_drafter: bool
    window: List[int] = field(default_factory=list)


def step_plans(cfg: WorkloadConfig) -> List[StepPlan]:
    """All (scale, layer) calls in execution order: scales outermost."""
    table = budget_table(cfg)
    plans = []
    for k in range(1, cfg.n_scale + 1):
        roles = layer_roles(cfg, k)
        n_k = cfg.n_tokens(k)
        for l in range(cfg.n_layer):
            plans.append(StepPlan(l, k, n_k, table[l][k - 1], roles[l], window_indices(cfg, n_k)))
    return plans


def dst_capacity(cfg: WorkloadConfig) -> int:
    """Rows a per-layer cache buffer must hold: max over scales of
    min(budget, C_full) + n_k (an upper bound on keep + n_k)."""
    table = budget_table(cfg)
    cap = 0
    for k in range(1, cfg.n_scale + 1):
        for l in range(cfg.n_layer):
            cap = max(cap, min(table[l][k - 1], c_full(cfg, k)) + cfg.n_tokens(k))
    return cap


def final_scale_budgets(cfg: WorkloadConfig) -> Sequence[int]:
    full = c_full(cfg, cfg.n_scale)
    return [max(1, round_half_up(f * full)) for f in FINAL_SCALE_BUDGET_FRACS]
