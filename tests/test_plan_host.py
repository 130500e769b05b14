"""The library's host planner (moe_plan_experts) against the plan oracle: same integers, same
node costs bit for bit, on seeded instances shaped like the benchmark's (Zipf loads, a cold-expert
floor, one or two spare slots per node) and on edge cases. Host code only: no GPU needed."""
import random

import numpy as np
import pytest

from oracle import plan_oracle as P
from paper_2504_02263_amd import binding as B


def _same(a, K, N, S):
    ref = P.plan_experts(a, K, N, S)
    replicas, slots, cost = B.moe_plan_experts(a, K, N, S)
    assert replicas == ref["replicas"]
    assert slots == ref["slots"]
    assert cost == ref["node_cost"]                 # same doubles, not just close
    return ref


def test_hand_worked_instance_through_the_c_abi():
    replicas, slots, cost = B.moe_plan_experts([10, 4, 3, 1], 2, 2, 3)
    assert replicas == [2, 1, 1, 1]
    assert slots == [[(0, 0), (1, 0)], [(0, 1), (2, 0), (3, 0)]]
    assert cost == [9.0, 10.0]


def test_random_instances_match_the_oracle_exactly():
    rnd = random.Random(7)
    for _ in range(400):
        M = rnd.randint(1, 40)
        N = rnd.randint(1, 12)
        S = (M + N - 1) // N + rnd.randint(0, 2)
        kind = rnd.randint(0, 2)
        if kind == 0:
            a = [rnd.random() * 100 for _ in range(M)]
        elif kind == 1:                                  # many equal costs: every tie-break is exercised
            a = [float(rnd.choice([1, 2, 2, 3, 8])) for _ in range(M)]
        else:                                            # Zipf popularity in a random order
            a = [1000.0 / r for r in range(1, M + 1)]
            rnd.shuffle(a)
        _same(a, rnd.choice([0.0, 2.0, 50.0]), N, S)


@pytest.mark.parametrize("E,k,T,N,S", [(16, 4, 1024, 4, 5), (16, 4, 1024, 8, 3), (64, 6, 8192, 8, 9), (8, 2, 256, 8, 2)])
def test_benchmark_shaped_loads(E, k, T, N, S):
    rng = np.random.default_rng(E * 1000 + N)
    bias = -np.log(rng.permutation(E) + 1.0)
    logits = rng.standard_normal((T, E)) + bias
    counts = np.bincount(np.argsort(-logits, axis=1)[:, :k].ravel(), minlength=E)
    ref = _same([float(c) for c in counts], float(T * k / E / 4), N, S)
    assert max(ref["node_cost"]) >= sum(max(float(c), T * k / E / 4) for c in counts) / N - 1e-9


def test_argument_errors():
    lib = B.load_library()
    import ctypes
    a = (ctypes.c_double * 3)(1.0, 2.0, 3.0)
    r = (ctypes.c_int32 * 3)()
    se, sc = (ctypes.c_int32 * 4)(), (ctypes.c_int32 * 4)()
    c = (ctypes.c_double * 2)()
    assert lib.moe_plan_experts(3, 2, 2, a, 0.0, r, se, sc, c) == B.MOE_OK
    assert lib.moe_plan_experts(3, 1, 2, a, 0.0, r, se, sc, c) == B.MOE_ERR_INVALID_ARG      # 2 slots < 3 experts
    assert lib.moe_plan_experts(0, 2, 2, a, 0.0, r, se, sc, c) == B.MOE_ERR_INVALID_ARG
    assert lib.moe_plan_experts(3, 2, 2, None, 0.0, r, se, sc, c) == B.MOE_ERR_INVALID_ARG
    nan = (ctypes.c_double * 3)(1.0, float("nan"), 3.0)
    assert lib.moe_plan_experts(3, 2, 2, nan, 0.0, r, se, sc, c) == B.MOE_ERR_INVALID_ARG
    with pytest.raises(B.MoeError):
        B.moe_plan_experts([1.0, 2.0, 3.0], 0.0, 1, 2)
