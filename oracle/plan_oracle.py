"""CPU oracle for the expert plan (hot-expert redundancy). TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this
module. The GPU library never does, and the two share no code.

What the paper states (Section 6, "Load balance"): M experts are spread over N
expert nodes with on-device redundancy for popular experts. With x[i][j] the
fraction of expert i served by node j (each expert's fractions sum to one), a_i
the cost of computing expert i's active tokens and K the lowest cost a cold
expert can have, the plan should minimise the largest node cost
    C_j = sum_i x[i][j] * max(a_i, K).
The paper solves this greedily and gives no further detail,
so the steps below are a reading, taken in this order:

  0. w_i = max(a_i, K).
  1. Replica counts. Every expert starts with one copy; free = N*S - M spare
     slots (S = expert slots a node has room for). While free > 0, take the
     expert with the largest per-copy share w_i / R_i (ties: lower index) among
     those with fewer than N copies; stop if that share is already no larger
     than the mean node cost sum(w) / N (no plan can beat the mean, and every
     extra copy costs memory); otherwise give it one more copy.
  2. Fractions. An expert's copies share its tokens equally: x = 1 / R_i on
     each node that hosts a copy.
  3. Placement, longest-processing-time first. All copies, ordered by share
     descending (ties: lower expert, then lower copy number), go one by one to
     the node with the smallest cost so far among nodes that have a free slot
     and do not yet host that expert (ties: lower node index).

Token split between copies (needed to run a plan): expert i's rows in the
expert-contiguous layout, [lo, lo + c), are cut into R_i consecutive parts,
copy r taking [lo + floor(r*c/R_i), lo + floor((r+1)*c/R_i)).

All arithmetic is IEEE double in the order written, so that an independent
implementation following the same steps reproduces the integers exactly.

Parity pins (tests/test_plan_pins.py): a hand-worked instance, the constraints
of the optimisation problem, its lower bounds, closed forms (equal costs; one
hot expert), and brute force over every replica vector and placement of tiny
instances.
"""
from __future__ import annotations


def plan_experts(a, K: float, N: int, S: int):
    """Greedy expert plan. a: per-expert costs (length M). Returns a dict with
    replicas[M], slots[N] (lists of (expert, copy) in placement order) and node_cost[N]."""
    M = len(a)
    if M < 1 or N < 1 or S < 1 or N * S < M:
        raise ValueError("need M >= 1 experts and N*S >= M slots")
    w = [max(float(x), float(K)) for x in a]
    total = 0.0
    for x in w:
        total += x
    mean = total / N
    R = [1] * M
    free = N * S - M
    while free > 0:
        best = -1
        for i in range(M):
            if R[i] < N and (best < 0 or w[i] / R[i] > w[best] / R[best]):
                best = i
        if best < 0 or w[best] / R[best] <= mean:
            break
        R[best] += 1
        free -= 1
    items = [(i, r) for i in range(M) for r in range(R[i])]
    items.sort(key=lambda ir: (-(w[ir[0]] / R[ir[0]]), ir[0], ir[1]))
    slots = [[] for _ in range(N)]
    cost = [0.0] * N
    for i, r in items:
        node = -1
        for j in range(N):
            if len(slots[j]) < S and all(e != i for e, _ in slots[j]) and (node < 0 or cost[j] < cost[node]):
                node = j
        if node < 0:
            raise ValueError("placement stuck: no node with a free slot that lacks this expert")
        slots[node].append((i, r))
        cost[node] += w[i] / R[i]
    return {"replicas": R, "slots": slots, "node_cost": cost}


def node_costs(a, K: float, replicas, slots):
    """The paper's C_j for a plan whose copies split their expert equally."""
    return [sum(max(float(a[i]), float(K)) / replicas[i] for i, _ in node) for node in slots]


def slot_segments(offsets, replicas, node_slots):
    """Row ranges of one node's slots: copy r of expert i gets the r-th of R_i consecutive parts
    of [offsets[i], offsets[i+1]). Returns (begin, end, expert) lists, one entry per slot."""
    begin, end, expert = [], [], []
    for i, r in node_slots:
        lo, c, Ri = int(offsets[i]), int(offsets[i + 1]) - int(offsets[i]), int(replicas[i])
        begin.append(lo + (r * c) // Ri)
        end.append(lo + ((r + 1) * c) // Ri)
        expert.append(i)
    return begin, end, expert
