"""Property pins for the CPU oracle, searched with hypothesis (CPU only).

Each property restates a piece of the layer's definition (paper Section 2.2; Section 6 "Fused kernels") in a
different form from the oracle's own code: selection by repeated arg-max with a strict comparison instead of a
sort, the counting sort as a filter per expert instead of a cursor loop, the layer as a per-token sum over
experts with no dispatch at all. Small integer-valued logits make ties the common case."""
import math

import numpy as np
from hypothesis import given, settings, strategies as st

from oracle import moe_oracle as O

SETTINGS = dict(max_examples=120, deadline=None)


@st.composite
def logits_and_k(draw):
    T = draw(st.integers(1, 12))
    E = draw(st.integers(1, 9))
    k = draw(st.integers(1, E))
    vals = draw(st.lists(st.sampled_from([-2.0, -1.0, -0.0, 0.0, 0.5, 1.0, 3.0]), min_size=T * E, max_size=T * E))
    return np.array(vals, dtype=np.float32).reshape(T, E), k


def _argmax_picks(row, k):
    """k rounds of arg-max over the remaining experts; a later expert replaces the best only if strictly larger."""
    cand = list(range(len(row)))
    picks = []
    for _ in range(k):
        best = cand[0]
        for e in cand[1:]:
            if row[e] > row[best]:
                best = e
        picks.append(best)
        cand.remove(best)
    return picks


@settings(**SETTINGS)
@given(logits_and_k())
def test_route_is_repeated_argmax_with_ties_to_the_lower_index(lk):
    logits, k = lk
    idx, w, counts, offsets = O.route(logits, k)
    T, E = logits.shape
    for t in range(T):
        assert idx[t].tolist() == _argmax_picks(logits[t], k)
        sel = [float(logits[t, e]) for e in idx[t]]
        den = math.fsum(math.exp(v - sel[0]) for v in sel)
        for j in range(k):
            assert abs(float(w[t, j]) - math.exp(sel[j] - sel[0]) / den) <= 1e-6
        assert abs(float(np.sum(w[t].astype(np.float64))) - 1.0) <= 1e-6
        assert all(w[t, j] >= w[t, j + 1] for j in range(k - 1))      # weights follow the pick order
    assert counts.sum() == T * k and offsets[0] == 0 and offsets[-1] == T * k
    assert [int(c) for c in counts] == [int((idx == e).sum()) for e in range(E)]
    assert (np.diff(offsets) == counts).all()


@settings(**SETTINGS)
@given(logits_and_k(), st.integers(1, 3))
def test_dispatch_is_the_stable_grouping_by_expert(lk, d):
    logits, k = lk
    T, E = logits.shape
    idx, _, _, offsets = O.route(logits, k)
    x = np.arange(T * d, dtype=np.float32).reshape(T, d) + 0.25
    xp, pos, src = O.dispatch(x, idx, offsets)
    flat = idx.ravel()
    expected_src = [i for e in range(E) for i in range(T * k) if flat[i] == e]   # filter per expert, order kept
    assert src.tolist() == expected_src
    assert [int(pos.ravel()[i]) for i in expected_src] == list(range(T * k))     # pos is the inverse permutation
    for r, i in enumerate(expected_src):
        assert offsets[flat[i]] <= r < offsets[flat[i] + 1]
        assert (xp[r] == x[i // k]).all()


@settings(max_examples=40, deadline=None)
@given(logits_and_k(), st.integers(0, 2 ** 31 - 1))
def test_layer_is_the_weighted_sum_over_each_tokens_experts(lk, seed):
    logits, k = lk
    T, E = logits.shape
    d, f = 3, 4
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((T, d))
    W = [(rng.standard_normal((f, d)), rng.standard_normal((f, d)), rng.standard_normal((d, f))) for _ in range(E)]
    ref = O.moe_layer(x, logits, k, lambda e: W[e])
    for t in range(T):
        picks = _argmax_picks(logits[t], k)
        sel = [float(logits[t, e]) for e in picks]
        den = math.fsum(math.exp(v - sel[0]) for v in sel)
        out = np.zeros(d)
        for j, e in enumerate(picks):
            g, u = W[e][0] @ x[t], W[e][1] @ x[t]
            out += (math.exp(sel[j] - sel[0]) / den) * (W[e][2] @ (g / (1.0 + np.exp(-g)) * u))
        np.testing.assert_allclose(ref["out"][t], out, rtol=1e-5, atol=1e-6)  # weights are float32 in the oracle
