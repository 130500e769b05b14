"""Seeded generators for synthetic MoE layers shaped like the paper's models.

Shapes follow the paper's model table (Section 7, "Model configurations":
Mixtral-8x22B h=6144 E=8 top-2 h'=16384; DBRX h=6144 E=16 top-4 h'=10752) plus a
tiny fp32 layer and a fine-grained many-expert layer. The paper measured on a
private production trace; these inputs stand in for it:

* activations x ~ N(0, 1)
* router logits ~ N(0, 1) (near-uniform expert load), optionally plus a
  per-expert bias -s*ln(rank_e) with rank a seeded permutation of 1..E, which
  makes expert popularity roughly Zipf(s) (the paper reports strongly skewed
  expert load in production, Section 8 "Expert load balance")
* router and expert weights ~ N(0, 1/fan_in)

Every tensor has its own random stream, keyed by (seed, tensor tag, index), so
one expert's weights can be regenerated without drawing the others.  bf16
tensors are rounded on the host (round-to-nearest-even) and carried as uint16
bit patterns: identical bytes go to the CPU oracle and to the GPU.

Nothing here computes any part of the MoE layer.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, List, Tuple

import numpy as np

_TAG_X, _TAG_LOGITS, _TAG_ROUTER, _TAG_BIAS, _TAG_GATE, _TAG_UP, _TAG_DOWN = range(1, 8)


@dataclass(frozen=True)
class LayerConfig:
    name: str
    T: int          # tokens in the batch
    d: int          # hidden size (paper: h)
    f: int          # expert intermediate size (paper: h')
    E: int          # experts
    k: int          # experts per token (paper: K / top-k)
    dtype: str      # "f32" or "bf16": storage type of x, weights, xp, h, y, out
    router: str     # "weights": logits = x @ W_r^T ; "logits": logits drawn directly
    zipf_s: float = 0.0
    micro_batches: int = 1

    @property
    def A(self) -> int:
        return self.T * self.k

    def with_T(self, T: int) -> "LayerConfig":
        return replace(self, T=T, name=f"{self.name.split('_T')[0]}_T{T}")


CONFIGS: Dict[str, LayerConfig] = {
    # small layer the CPU oracle finishes in well under a second
    "tiny_fp32": LayerConfig("tiny_fp32", T=64, d=256, f=512, E=8, k=2, dtype="f32", router="weights"),
    # Mixtral-8x22B-shaped decode micro-batch: the configuration the headline metric is quoted on
    "mixtral_T256": LayerConfig("mixtral_T256", T=256, d=6144, f=16384, E=8, k=2, dtype="bf16", router="logits"),
    # DBRX-shaped layer with Zipf(1.0) expert popularity
    "dbrx_zipf_T1024": LayerConfig("dbrx_zipf_T1024", T=1024, d=6144, f=10752, E=16, k=4, dtype="bf16",
                                   router="logits", zipf_s=1.0),
    # fine-grained many-expert layer, 3 micro-batches
    "finegrained_T8192": LayerConfig("finegrained_T8192", T=8192, d=4096, f=1408, E=64, k=6, dtype="bf16",
                                     router="logits", micro_batches=3),
    # the paper's third evaluation model (Section 7, model table: Scaled-MoE), as a decode micro-batch with
    # 256 tokens per expert on average; an extra benchmark row, near-uniform load
    "scaled_moe_T2048": LayerConfig("scaled_moe_T2048", T=2048, d=8192, f=8192, E=32, k=4, dtype="bf16",
                                    router="logits"),
}

MIXTRAL_SWEEP_T: Tuple[int, ...] = (32, 64, 128, 256, 512, 1024, 2048, 4096)


def mixtral_sweep_config(T: int) -> LayerConfig:
    """The Mixtral-shaped layer at another token count (one weight set serves the whole sweep)."""
    return CONFIGS["mixtral_T256"].with_T(T)


def _rng(seed: int, tag: int, index: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([int(seed), int(tag), int(index)])))


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns the uint16 bit patterns.

    Inputs are finite by construction (normal draws), so no NaN handling is needed.
    """
    a = np.ascontiguousarray(a, dtype=np.float32)
    out = np.empty(a.shape, dtype=np.uint16)
    flat_in = a.reshape(-1)
    flat_out = out.reshape(-1)
    step = 1 << 24
    for s in range(0, flat_in.size, step):
        u = flat_in[s:s + step].view(np.uint32)
        r = (u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))) >> np.uint32(16)
        flat_out[s:s + step] = r.astype(np.uint16)
    return out


def _store(a: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "f32":
        return np.ascontiguousarray(a, dtype=np.float32)
    if dtype == "bf16":
        return f32_to_bf16_bits(a)
    raise ValueError(f"unknown dtype {dtype!r}")


def _normal(rng: np.random.Generator, shape, std: float) -> np.ndarray:
    a = rng.standard_normal(shape, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    return a


def make_activations(cfg: LayerConfig, seed: int = 0) -> np.ndarray:
    """x[T, d] ~ N(0,1) at the layer's storage type (float32, or uint16 bf16 bits)."""
    return _store(_normal(_rng(seed, _TAG_X, cfg.T), (cfg.T, cfg.d), 1.0), cfg.dtype)


def make_router_weight(cfg: LayerConfig, seed: int = 0) -> np.ndarray:
    """W_r[E, d] ~ N(0, 1/d), float32 (only the tiny fp32 layer routes through a gating matrix)."""
    return _normal(_rng(seed, _TAG_ROUTER), (cfg.E, cfg.d), 1.0 / np.sqrt(cfg.d))


def zipf_bias(cfg: LayerConfig, seed: int = 0) -> np.ndarray:
    """Per-expert logit bias -s*ln(rank_e); rank is a seeded permutation of 1..E."""
    if cfg.zipf_s == 0.0:
        return np.zeros(cfg.E, dtype=np.float32)
    rank = _rng(seed, _TAG_BIAS).permutation(cfg.E) + 1
    return (-cfg.zipf_s * np.log(rank.astype(np.float64))).astype(np.float32)


def expected_load_skew(cfg: LayerConfig) -> float:
    """How many times the mean load this workload's router is expected to give its most popular expert
    (what a serving engine that tracks expert popularity would know): 1 for the near-uniform routers; under
    the Zipf(s) bias, the head's share of first picks times E, capped at E / k because a token picks an
    expert at most once."""
    if cfg.zipf_s == 0.0:
        return 1.0
    p = np.arange(1, cfg.E + 1, dtype=np.float64) ** -cfg.zipf_s
    return float(min(cfg.E * p[0] / p.sum(), cfg.E / cfg.k))


def make_logits(cfg: LayerConfig, seed: int = 0) -> np.ndarray:
    """Router logits[T, E] float32 ~ N(0,1) (+ Zipf bias), for layers whose router input is the logits."""
    lg = _normal(_rng(seed, _TAG_LOGITS, cfg.T), (cfg.T, cfg.E), 1.0)
    if cfg.zipf_s != 0.0:
        lg = lg + zipf_bias(cfg, seed)[None, :]
    return np.ascontiguousarray(lg, dtype=np.float32)


def make_expert_weights(cfg: LayerConfig, seed: int, e: int):
    """One expert's (W_gate[f,d], W_up[f,d], W_down[d,f]) ~ N(0, 1/fan_in) at the storage type."""
    wg = _store(_normal(_rng(seed, _TAG_GATE, e), (cfg.f, cfg.d), 1.0 / np.sqrt(cfg.d)), cfg.dtype)
    wu = _store(_normal(_rng(seed, _TAG_UP, e), (cfg.f, cfg.d), 1.0 / np.sqrt(cfg.d)), cfg.dtype)
    wd = _store(_normal(_rng(seed, _TAG_DOWN, e), (cfg.d, cfg.f), 1.0 / np.sqrt(cfg.f)), cfg.dtype)
    return wg, wu, wd


def microbatch_ranges(T: int, m: int) -> List[Tuple[int, int]]:
    """Split T tokens into m contiguous micro-batches whose sizes differ by at most one (larger first)."""
    base, extra = divmod(T, m)
    out, start = [], 0
    for i in range(m):
        n = base + (1 if i < extra else 0)
        out.append((start, start + n))
        start += n
    return out


def make_all_expert_weights(cfg: LayerConfig, seed: int = 0, workers: int = 8):
    """All experts' weights stacked: (W_gate[E,f,d], W_up[E,f,d], W_down[E,d,f]).

    Same values as make_expert_weights(cfg, seed, e) for every e; experts are drawn in
    parallel threads (each has its own stream, so the result does not depend on `workers`).
    """
    from concurrent.futures import ThreadPoolExecutor

    np_dtype = np.float32 if cfg.dtype == "f32" else np.uint16
    wg = np.empty((cfg.E, cfg.f, cfg.d), dtype=np_dtype)
    wu = np.empty((cfg.E, cfg.f, cfg.d), dtype=np_dtype)
    wd = np.empty((cfg.E, cfg.d, cfg.f), dtype=np_dtype)

    def one(e: int):
        wg[e], wu[e], wd[e] = make_expert_weights(cfg, seed, e)

    with ThreadPoolExecutor(max_workers=max(1, workers)) as pool:
        list(pool.map(one, range(cfg.E)))
    return wg, wu, wd
