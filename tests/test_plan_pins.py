"""Pins for the expert-plan oracle (hot-expert redundancy, paper Section 6 "Load balance").

The paper states the optimisation problem and says only that a greedy approximation solves it,
so these tests pin the oracle to what the problem itself fixes: its constraints, its lower
bounds, closed forms, a hand-worked instance, and the true optimum found by brute force over
every replica vector and placement of tiny instances.
"""
import itertools
import random

import numpy as np
import pytest

from oracle import moe_oracle as O
from oracle import plan_oracle as P


def _check_constraints(a, K, N, S, plan):
    M = len(a)
    R, slots = plan["replicas"], plan["slots"]
    assert len(slots) == N and all(len(s) <= S for s in slots)
    x = np.zeros((M, N))
    for j, node in enumerate(slots):
        experts = [e for e, _ in node]
        assert len(set(experts)) == len(experts)           # at most one copy of an expert per node
        for e, r in node:
            assert 0 <= r < R[e]
            x[e, j] += 1.0 / R[e]
    np.testing.assert_allclose(x.sum(axis=1), 1.0, atol=1e-12)   # fractions of every expert sum to one
    copies = sorted((e, r) for node in slots for e, r in node)
    assert copies == [(e, r) for e in range(M) for r in range(R[e])]   # every copy placed exactly once
    w = np.maximum(np.asarray(a, float), K)
    np.testing.assert_allclose(plan["node_cost"], x.T @ w, rtol=1e-12)  # C_j = sum_i x_ij max(a_i, K)
    np.testing.assert_allclose(P.node_costs(a, K, R, slots), plan["node_cost"], rtol=1e-12)
    return w


def test_hand_worked_instance():
    # M=4, N=2, S=3, a=[10,4,3,1], K=2: w=[10,4,3,2], sum 19, mean node cost 9.5, two spare slots.
    # Largest share 10 > 9.5: expert 0 gets a second copy (share 5 <= 9.5: stop).
    # Copies by share: (0,0)=5, (0,1)=5, (1,0)=4, (2,0)=3, (3,0)=2.
    # 5 -> node 0; 5 -> node 1 (node 0 already hosts expert 0); 4 -> node 0 (5 = 5, lower index): 9;
    # 3 -> node 1: 8; 2 -> node 1: 10.
    plan = P.plan_experts([10, 4, 3, 1], 2, 2, 3)
    assert plan["replicas"] == [2, 1, 1, 1]
    assert plan["slots"] == [[(0, 0), (1, 0)], [(0, 1), (2, 0), (3, 0)]]
    assert plan["node_cost"] == [9.0, 10.0]


def test_cold_floor_K_lifts_cheap_experts():
    # every expert cheaper than K costs K: four experts on two nodes cost 2K each
    plan = P.plan_experts([0.1, 0.0, 0.3, 0.2], 5.0, 2, 2)
    assert plan["node_cost"] == [10.0, 10.0] and plan["replicas"] == [1, 1, 1, 1]


@pytest.mark.parametrize("M,N,S", [(8, 4, 2), (16, 4, 5), (12, 3, 4), (6, 6, 2)])
def test_equal_costs_balance_exactly_without_copies(M, N, S):
    plan = P.plan_experts([3.0] * M, 1.0, N, S)
    assert plan["replicas"] == [1] * M                     # share 3 never exceeds the mean 3*M/N >= 3
    assert max(plan["node_cost"]) - min(plan["node_cost"]) <= (3.0 if M % N else 0.0)
    if M % N == 0:
        assert plan["node_cost"] == [3.0 * M / N] * N


def test_single_hot_expert_is_copied_until_its_share_reaches_the_mean():
    # w = [90, 1 x 9]: sum 99, N = 3, mean 33. Shares 90 -> 45 -> 30 <= 33: three copies, one per node.
    plan = P.plan_experts([90] + [1] * 9, 0.5, 3, 6)
    assert plan["replicas"] == [3] + [1] * 9
    assert [sum(1 for e, _ in node if e == 0) for node in plan["slots"]] == [1, 1, 1]
    assert max(plan["node_cost"]) == 33.0                  # 30 + three cold experts each: the optimum
    # without spare slots the hot expert cannot be copied and one node carries all of it
    tight = P.plan_experts([90] + [1] * 8, 0.5, 3, 3)
    assert tight["replicas"] == [1] * 9 and max(tight["node_cost"]) == 92.0


def _brute_optimum(w, N, S):
    """Best max-node-cost over every choice of hosting node set per expert (equal split), S slots per node."""
    subsets = [s for r in range(1, N + 1) for s in itertools.combinations(range(N), r)]
    best = None
    for choice in itertools.product(subsets, repeat=len(w)):
        cnt, cost = [0] * N, [0.0] * N
        for i, sub in enumerate(choice):
            for j in sub:
                cnt[j] += 1
                cost[j] += w[i] / len(sub)
        if max(cnt) <= S:
            best = max(cost) if best is None else min(best, max(cost))
    return best


def test_against_brute_force_optimum_and_lower_bounds():
    rnd = random.Random(1)
    worst = 0.0
    done = 0
    while done < 250:
        M, N = rnd.randint(1, 4), rnd.randint(1, 3)
        S = rnd.randint((M + N - 1) // N, max(3, (M + N - 1) // N))
        a = [rnd.choice([1, 2, 3, 5, 8, 13, 40]) * rnd.random() for _ in range(M)]
        K = rnd.choice([0, 1, 3])
        plan = P.plan_experts(a, K, N, S)
        w = _check_constraints(a, K, N, S, plan)
        got = max(plan["node_cost"])
        opt = _brute_optimum(list(w), N, S)
        assert got >= opt - 1e-12                          # nothing beats the optimum
        assert opt >= w.sum() / N - 1e-12 and opt >= w.max() / N - 1e-12   # the problem's lower bounds
        assert got <= 2.0 * opt + 1e-12                    # list-scheduling quality: mean + largest share
        worst = max(worst, got / opt)
        done += 1
    print(f"worst greedy / optimum over {done} tiny instances: {worst:.3f}")


def test_zipf_load_needs_and_gets_copies():
    # Zipf(1) popularity over 16 experts, 8 nodes with 3 slots each: the hottest expert alone
    # exceeds the mean node cost, so it must be split; the plan's maximum then sits near the mean.
    a = [1000.0 / r for r in range(1, 17)]
    K = 40.0
    base = P.plan_experts(a, K, 8, 2)                      # 16 slots for 16 experts: no copies possible
    plan = P.plan_experts(a, K, 8, 3)
    w = _check_constraints(a, K, 8, 3, plan)
    mean = w.sum() / 8
    assert max(base["node_cost"]) >= 1000.0 > mean
    assert plan["replicas"][0] >= 2
    assert max(plan["node_cost"]) < 0.6 * max(base["node_cost"])
    assert max(plan["node_cost"]) <= 1.35 * mean


def test_rejects_too_few_slots():
    with pytest.raises(ValueError):
        P.plan_experts([1, 2, 3], 0, 1, 2)


# --------------------------------------------------------------------------- running a plan

def test_slot_segments_partition_every_expert():
    rng = np.random.default_rng(5)
    counts = rng.integers(0, 40, size=12)
    counts[3] = 0
    offsets = np.concatenate([[0], np.cumsum(counts)])
    plan = P.plan_experts(list(counts.astype(float)), 4.0, 4, 5)
    covered = np.zeros(offsets[-1], dtype=int)
    sizes = {}
    for node in plan["slots"]:
        b, e, ex = P.slot_segments(offsets, plan["replicas"], node)
        for lo, hi, i in zip(b, e, ex):
            assert offsets[i] <= lo <= hi <= offsets[i + 1]
            covered[lo:hi] += 1
            sizes.setdefault(i, []).append(hi - lo)
    assert (covered == 1).all()                            # every row belongs to exactly one copy
    for i, s in sizes.items():
        assert len(s) == plan["replicas"][i] and sum(s) == counts[i] and max(s) - min(s) <= 1


def test_running_all_nodes_of_a_plan_equals_the_unreplicated_layer():
    rng = np.random.default_rng(11)
    E, d, f = 6, 8, 12
    counts = np.array([9, 0, 3, 17, 1, 5])
    offsets = np.concatenate([[0], np.cumsum(counts)])
    xp = rng.standard_normal((offsets[-1], d))
    W = [(rng.standard_normal((f, d)), rng.standard_normal((f, d)), rng.standard_normal((d, f))) for _ in range(E)]
    plan = P.plan_experts(list(counts.astype(float)), 2.0, 3, 4)
    assert max(plan["replicas"]) > 1
    y = None
    for node in plan["slots"]:
        y = O.expert_ffn_segments(xp, *P.slot_segments(offsets, plan["replicas"], node), W, y=y)
    np.testing.assert_allclose(y, O.expert_ffn(xp, offsets, W), rtol=1e-12, atol=1e-12)
    # and against the definition row by row (no segments at all)
    for r in range(offsets[-1]):
        e = int(np.searchsorted(offsets, r, side="right") - 1)
        g, u = W[e][0] @ xp[r], W[e][1] @ xp[r]
        np.testing.assert_allclose(y[r], W[e][2] @ (g / (1 + np.exp(-g)) * u), rtol=1e-11, atol=1e-11)
