"""The benchmark's flop/byte accounting against the values the paper prints (tests/golden)."""
import os

from paper_2504_02263_amd import roofline as R

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_roofline_example.txt")


def _golden():
    out = {}
    with open(GOLDEN) as fh:
        for line in fh:
            line = line.split("#")[0].strip()
            if line:
                key, val = (s.strip() for s in line.split("="))
                out[key] = float(val)
    return out


def test_paper_worked_example():
    g = _golden()
    F, B = g["peak_tflops"] * 1e12, g["mem_tb_per_s"] * 1e12
    b = R.ridge_batch(F, B)
    assert b == g["ridge_batch_tokens"]
    assert R.tokens_per_expert(b, int(g["topk"]), int(g["num_experts"])) == g["tokens_per_expert_at_ridge"]
    assert R.moe_ffn_util(b, int(g["topk"]), int(g["num_experts"]), F, B) == g["ffn_mfu_at_ridge"]
    # dense model at the ridge batch is fully utilised; MoE needs E/topk times the batch
    assert R.moe_ffn_util(b, 1, 1, F, B) == 1.0
    assert R.moe_ffn_util(4 * b, 2, 8, F, B) == 1.0
    assert R.moe_ffn_util(8 * b, 2, 8, F, B) == 1.0            # clipped at 1


def test_paper_message_size():
    g = _golden()
    assert R.dispatch_message_bytes(128, 2, 8, 6144, 2, tp=2) == g["m2n_message_bytes"]


def test_gemm_counts_and_ridge_consistency():
    b, h, n = 39, 6144, 16384
    assert R.gemm_flops(b, h, n) == 2 * b * h * n
    assert R.gemm_param_bytes(h, n) == 2 * h * n
    # at the ridge batch the flop time equals the parameter-read time
    F, B = 312e12, 2e12
    rb = R.ridge_batch(F, B)
    assert abs(R.gemm_flops(rb, h, n) / F - R.gemm_param_bytes(h, n) / B) < 1e-12
    assert R.ridge_batch(R.MI355X_BF16_DENSE_FLOPS, R.MI355X_HBM_BYTES_PER_S) == 312.5


def test_layer_cost_mixtral_decode():
    c = R.layer_cost(T=256, d=6144, f=16384, E=8, k=2, elem_bytes=2)
    assert c.flops == 6 * 512 * 6144 * 16384
    assert c.weight_bytes == 3 * 6144 * 16384 * 2 * 8            # 4.83 GB
    assert c.ffn_in_flops + c.ffn_out_flops == c.flops
    # three GEMMs per expert, each 2*c_e*d*f flops
    assert c.flops == 3 * R.gemm_flops(512, 6144, 16384)
    assert c.layer_min_bytes == c.weight_bytes + 2 * 256 * 6144 * 2 + 256 * 8 * 4
    assert c.staged_bytes > c.layer_min_bytes
    # fewer active experts -> fewer weight bytes
    assert R.layer_cost(2, 6144, 16384, 8, 2, 2).weight_bytes == 3 * 6144 * 16384 * 2 * 4


def test_expert_time_fit_recovers_a_known_line_and_crossover():
    b = [8, 16, 32, 64, 128, 512, 1024, 2048]
    t = [0.75 + 1e-4 * x for x in b[:5]] + [0.2 + 1.3e-3 * x for x in b[5:]]
    k3, k4, resid = R.fit_linear(b[5:], t[5:])
    assert abs(k3 - 1.3e-3) < 1e-12 and abs(k4 - 0.2) < 1e-9 and resid < 1e-9
    fit = R.fit_expert_time(b, t, split=128)
    assert abs(fit["streaming"]["k3"] - 1e-4) < 1e-12 and abs(fit["streaming"]["k4"] - 0.75) < 1e-9
    assert abs(fit["crossover_b"] - (0.75 - 0.2) / (1.3e-3 - 1e-4)) < 1e-6
    assert fit["single"]["max_rel_resid"] > 0.01          # one line does not describe both regimes
