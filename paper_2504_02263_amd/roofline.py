"""Flop and byte accounting for the MoE layer, and the paper's roofline model.

Host-side arithmetic only (no GPU, no numerics of the layer itself).

The model is the one in the paper's Section 2.3: a (b x h)·(h x n) GEMM costs 2·b·h·n flops
and reads h·n parameters (2·h·n bytes in bf16); it is compute-bound once b >= F/B, with F the
peak flop rate and B the memory bandwidth; for an MoE layer each expert sees only
b·topk/#experts tokens, so util = min(topk/#experts · B/F · b, 1).
"""
from __future__ import annotations

from dataclasses import dataclass

# MI355X published peaks used as roofline denominators.
MI355X_HBM_BYTES_PER_S = 8.0e12          # HBM3E, 8 TB/s
MI355X_BF16_DENSE_FLOPS = 2.5e15         # dense bf16 MFMA, 2.5 PFLOP/s
MI355X_FP32_VECTOR_FLOPS = 157.3e12      # fp32 vector ALU


def gemm_flops(b: int, h: int, n: int) -> int:
    """Flops of a (b x h)·(h x n) GEMM (Section 2.3)."""
    return 2 * b * h * n


def gemm_param_bytes(h: int, n: int, elem_bytes: int = 2) -> int:
    """Parameter bytes such a GEMM must read (Section 2.3: 2·h·n for bfloat16)."""
    return elem_bytes * h * n


def ridge_batch(peak_flops: float, mem_bytes_per_s: float, elem_bytes: int = 2) -> float:
    """Smallest batch b at which the GEMM is compute-bound: 2bhn/F >= s·hn/B  =>  b >= (s/2)·F/B.
    For bf16 (s = 2) this is the paper's b >= F/B."""
    return (elem_bytes / 2.0) * peak_flops / mem_bytes_per_s


def tokens_per_expert(batch: float, topk: int, num_experts: int) -> float:
    """Average tokens each expert sees out of a batch (Section 2.3)."""
    return batch * topk / num_experts


def moe_ffn_util(batch: float, topk: int, num_experts: int, peak_flops: float, mem_bytes_per_s: float) -> float:
    """Theoretical FFN utilisation of an MoE layer at a given batch (Section 2.3)."""
    return min(topk / num_experts * mem_bytes_per_s / peak_flops * batch, 1.0)


def dispatch_message_bytes(tokens: int, topk: int, num_experts: int, hidden: int, elem_bytes: int, tp: int = 1) -> float:
    """Average bytes one source sends to one expert (Section 7.3):
    tokens·topk/#experts·hidden·sizeof(dtype)/TP."""
    return tokens * topk / num_experts * hidden * elem_bytes / tp


@dataclass(frozen=True)
class LayerCost:
    """Algorithmic cost of one layer call, per step of the path (bytes the method itself must move)."""
    flops: int              # 6·A·d·f: three 2·c_e·d·f GEMMs summed over experts
    ffn_in_flops: int       # gate+up GEMMs, 4·A·d·f
    ffn_out_flops: int      # down GEMM, 2·A·d·f
    weight_bytes: int       # 3·d·f·s per expert that has at least one token
    route_bytes: int
    dispatch_bytes: int
    ffn_in_bytes: int       # gate+up weights + xp read + h write
    ffn_out_bytes: int      # down weights + h read + y write
    combine_bytes: int
    layer_min_bytes: int    # compulsory for the whole layer: weights + x + out + logits

    @property
    def ffn_bytes(self) -> int:
        return self.ffn_in_bytes + self.ffn_out_bytes

    @property
    def staged_bytes(self) -> int:
        return self.route_bytes + self.dispatch_bytes + self.ffn_bytes + self.combine_bytes


def layer_cost(T: int, d: int, f: int, E: int, k: int, elem_bytes: int, active_experts: int | None = None) -> LayerCost:
    """Cost of one call of the four-step path on T tokens.

    active_experts = number of experts with at least one token (defaults to min(E, T·k)).
    """
    A = T * k
    s = elem_bytes
    act = min(E, A) if active_experts is None else active_experts
    w_in = 2 * d * f * s * act
    w_out = d * f * s * act
    return LayerCost(
        flops=6 * A * d * f,
        ffn_in_flops=4 * A * d * f,
        ffn_out_flops=2 * A * d * f,
        weight_bytes=w_in + w_out,
        route_bytes=T * E * 4 + 8 * A + 4 * (2 * E + 1),
        dispatch_bytes=T * d * s + A * d * s + 12 * A,
        ffn_in_bytes=w_in + A * d * s + A * f * s,
        ffn_out_bytes=w_out + A * f * s + A * d * s,
        combine_bytes=A * d * s + T * d * s + 8 * A,
        layer_min_bytes=w_in + w_out + 2 * T * d * s + T * E * 4,
    )


def fit_linear(b, t):
    """Least-squares line t = k3*b + k4 through points (b_i, t_i); returns (k3, k4, max relative residual).

    This is the paper's expert-time model T_e = k3*b_e + k4 (Section 4.2, "Performance simulation"),
    whose constants it obtains by profiling."""
    n = len(b)
    if n < 2 or n != len(t):
        raise ValueError("need at least two (b, t) points")
    mb, mt = sum(b) / n, sum(t) / n
    sxx = sum((x - mb) ** 2 for x in b)
    if sxx == 0:
        raise ValueError("all b equal")
    k3 = sum((x - mb) * (y - mt) for x, y in zip(b, t)) / sxx
    k4 = mt - k3 * mb
    resid = max(abs(k3 * x + k4 - y) / y for x, y in zip(b, t))
    return k3, k4, resid


def fit_expert_time(b, t, split: float):
    """Fit T_e(b_e) as the paper's single line and as two regimes (b <= split: weight-streaming,
    b > split: compute) and return both, with the batch at which the two regime lines cross (the
    measured ridge, to be compared with the roofline's F/B)."""
    lo = [(x, y) for x, y in zip(b, t) if x <= split]
    hi = [(x, y) for x, y in zip(b, t) if x > split]
    out = {"single": dict(zip(("k3", "k4", "max_rel_resid"), fit_linear(b, t)))}
    if len(lo) >= 2 and len(hi) >= 2:
        a1, c1, r1 = fit_linear(*zip(*lo))
        a2, c2, r2 = fit_linear(*zip(*hi))
        out["streaming"] = {"k3": a1, "k4": c1, "max_rel_resid": r1}
        out["compute"] = {"k3": a2, "k4": c2, "max_rel_resid": r2}
        out["crossover_b"] = (c1 - c2) / (a2 - a1) if a2 != a1 else None
    return out
