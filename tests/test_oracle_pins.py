"""Pins for the CPU oracle: brute force, closed forms, library routines and invariants.

None of these re-types the oracle's own formula: each checks it against something fixed by
the mathematics (or by a hand-derived example), so that a dropped term, a wrong sign or
index, or a transposed operand in the oracle fails at least one test.
"""
import itertools
import math

import numpy as np
import pytest

from oracle import moe_oracle as O
from workloads import synth


def _rng(seed):
    return np.random.default_rng(seed)


# --------------------------------------------------------------------------- route: top-k

def _brute_topk(row, k):
    """All C(E,k) subsets: the best one maximises the descending-sorted logit tuple; among
    equally good subsets the lexicographically smallest index set wins. Listing order:
    descending logit, equal logits by ascending index."""
    E = len(row)
    best_key, best = None, None
    for sub in itertools.combinations(range(E), k):
        key = (tuple(sorted((float(row[e]) for e in sub), reverse=True)), tuple(-e for e in sub))
        if best_key is None or key > best_key:
            best_key, best = key, sub
    return sorted(best, key=lambda e: (-float(row[e]), e))


@pytest.mark.parametrize("E,k", [(4, 1), (4, 2), (5, 3), (8, 2), (8, 4), (8, 8), (6, 5)])
def test_topk_matches_subset_brute_force(E, k):
    rng = _rng(100 + 10 * E + k)
    # few distinct values => many ties
    logits = rng.integers(-2, 3, size=(60, E)).astype(np.float32)
    logits[::3] = rng.standard_normal((len(logits[::3]), E)).astype(np.float32)
    idx, _, _, _ = O.route(logits, k)
    for t in range(logits.shape[0]):
        assert list(idx[t]) == _brute_topk(logits[t], k), (t, logits[t])


def test_topk_adversarial_ties():
    E, k = 8, 3
    same = np.full((3, E), 0.25, np.float32)
    idx, w, _, _ = O.route(same, k)
    assert (idx == np.arange(k)).all()
    np.testing.assert_allclose(w, 1.0 / k, rtol=0, atol=1e-15)
    dec = np.arange(E, 0, -1, dtype=np.float32)[None]
    assert list(O.route(dec, k)[0][0]) == [0, 1, 2]
    inc = np.arange(E, dtype=np.float32)[None]
    assert list(O.route(inc, k)[0][0]) == [7, 6, 5]
    dup = np.array([[0, 5, 1, 5, 5, 2, 0, 1]], np.float32)
    assert list(O.route(dup, 2)[0][0]) == [1, 3]
    assert list(O.route(dup, 4)[0][0]) == [1, 3, 4, 5]
    zeros = np.array([[0.0, -0.0, 0.0, -0.0]], np.float32)      # -0.0 == 0.0: index order decides
    assert list(O.route(zeros, 3)[0][0]) == [0, 1, 2]
    neg_inf = np.array([[-np.inf, 1.0, -np.inf, -np.inf]], np.float32)
    assert list(O.route(neg_inf, 3)[0][0]) == [1, 0, 2]


def test_hand_worked_routing_example():
    """T=2, E=4, k=2, worked by hand.
    token 0: logits 1,3,3,0 -> experts 1 and 2 tie at 3 -> [1,2], weights .5/.5
    token 1: all zero      -> [0,1], weights .5/.5
    flat assignments i=0..3 go to experts 1,2,0,1 -> counts [1,2,1,0], offsets [0,1,3,4,4]
    expert 0 rows: i=2 -> row 0; expert 1 rows: i=0,3 -> rows 1,2; expert 2: i=1 -> row 3."""
    logits = np.array([[1, 3, 3, 0], [0, 0, 0, 0]], np.float32)
    idx, w, counts, offsets = O.route(logits, 2)
    assert idx.tolist() == [[1, 2], [0, 1]]
    assert w.tolist() == [[0.5, 0.5], [0.5, 0.5]]
    assert counts.tolist() == [1, 2, 1, 0]
    assert offsets.tolist() == [0, 1, 3, 4, 4]
    x = np.array([[10.0, 11.0], [20.0, 21.0]], np.float32)
    xp, pos, src = O.dispatch(x, idx, offsets)
    assert src.tolist() == [2, 0, 3, 1]
    assert pos.tolist() == [[1, 3], [0, 2]]
    assert xp.tolist() == [[20.0, 21.0], [10.0, 11.0], [20.0, 21.0], [10.0, 11.0]]


# --------------------------------------------------------------------------- route: weights

def test_weights_closed_forms():
    rng = _rng(7)
    logits = rng.standard_normal((200, 8)).astype(np.float32)
    # k = 1: the single weight is 1
    assert (O.route(logits, 1)[1] == 1.0).all()
    # k = 2: logistic of the logit gap
    idx, w, _, _ = O.route(logits, 2)
    l = np.take_along_axis(logits.astype(np.float64), idx.astype(np.int64), 1)
    for t in range(200):
        gap = l[t, 0] - l[t, 1]
        assert gap >= 0
        assert math.isclose(w[t, 0], 1.0 / (1.0 + math.exp(-gap)), rel_tol=1e-14)
        assert math.isclose(w[t, 1], 1.0 / (1.0 + math.exp(gap)), rel_tol=1e-13)
    # k = E: plain softmax over all logits (scipy), in pick order
    from scipy.special import softmax
    idx, w, _, _ = O.route(logits, 8)
    full = softmax(logits.astype(np.float64), axis=1)
    np.testing.assert_allclose(w, np.take_along_axis(full, idx.astype(np.int64), 1), rtol=1e-13)


@pytest.mark.parametrize("k", [2, 4, 6])
def test_weights_equal_full_softmax_renormalised(k):
    from scipy.special import softmax
    rng = _rng(8 + k)
    logits = (3 * rng.standard_normal((128, 16))).astype(np.float32)
    idx, w, _, _ = O.route(logits, k)
    full = softmax(logits.astype(np.float64), axis=1)
    picked = np.take_along_axis(full, idx.astype(np.int64), 1)
    np.testing.assert_allclose(w, picked / picked.sum(1, keepdims=True), rtol=1e-12)
    np.testing.assert_allclose(w.sum(1), 1.0, rtol=0, atol=1e-15)
    assert (np.diff(w, axis=1) <= 0).all()          # non-increasing in pick order
    assert (w > 0).all()


# --------------------------------------------------------------------------- counts / offsets

@pytest.mark.parametrize("T,E,k", [(1, 4, 2), (64, 8, 2), (333, 16, 4), (500, 64, 6), (0, 8, 2)])
def test_counts_offsets(T, E, k):
    logits = _rng(T + E).standard_normal((T, E)).astype(np.float32)
    idx, _, counts, offsets = O.route(logits, k)
    assert counts.dtype == np.int32 and offsets.dtype == np.int32 and idx.dtype == np.int32
    assert counts.sum() == T * k                                   # token conservation (Section 4.2: b_e*E/K = B)
    assert (counts == np.bincount(idx.ravel(), minlength=E)).all()
    assert (offsets == np.concatenate([[0], np.cumsum(counts)])).all()
    assert offsets[E] == T * k
    if T:
        # a token never picks one expert twice
        assert all(len(set(r)) == k for r in idx.tolist())


def test_mean_tokens_per_expert_matches_paper_example():
    # Section 2.3: batch 156, top-2 of 8 experts -> 39 tokens per expert on average
    logits = _rng(1).standard_normal((156, 8)).astype(np.float32)
    _, _, counts, _ = O.route(logits, 2)
    assert counts.mean() == 39.0


# --------------------------------------------------------------------------- dispatch

@pytest.mark.parametrize("T,E,k,d", [(64, 8, 2, 16), (257, 16, 4, 8), (100, 64, 6, 4), (5, 4, 1, 3)])
def test_dispatch_is_stable_counting_sort(T, E, k, d):
    rng = _rng(T * 7 + E)
    logits = rng.standard_normal((T, E)).astype(np.float32)
    x = rng.standard_normal((T, d)).astype(np.float32)
    idx, _, counts, offsets = O.route(logits, k)
    xp, pos, src = O.dispatch(x, idx, offsets)
    A = T * k
    assert (src == np.argsort(idx.ravel(), kind="stable")).all()      # library routine
    assert (pos.ravel()[src] == np.arange(A)).all()                   # permutation ...
    assert (src[pos.ravel()] == np.arange(A)).all()                   # ... and its inverse
    assert (xp == x[src // k]).all() and xp.dtype == x.dtype          # pure copy
    row_expert = idx.ravel()[src]
    assert (np.diff(row_expert) >= 0).all()
    for e in range(E):
        assert (row_expert[offsets[e]:offsets[e + 1]] == e).all()
        seg = src[offsets[e]:offsets[e + 1]]
        assert (np.diff(seg) > 0).all()                               # ascending flat index inside a segment


def test_dispatch_copies_bf16_bits_unchanged():
    rng = _rng(3)
    x = rng.integers(0, 65536, size=(10, 8)).astype(np.uint16)
    idx, _, _, offsets = O.route(rng.standard_normal((10, 4)).astype(np.float32), 2)
    xp, _, src = O.dispatch(x, idx, offsets)
    assert xp.dtype == np.uint16 and (xp == x[src // 2]).all()


def test_dispatch_empty():
    idx, _, _, offsets = O.route(np.zeros((0, 4), np.float32), 2)
    xp, pos, src = O.dispatch(np.zeros((0, 8), np.float32), idx, offsets)
    assert xp.shape == (0, 8) and pos.shape == (0, 2) and src.shape == (0,)


# --------------------------------------------------------------------------- widen (bf16)

def test_widen_bf16_exact():
    # hand-known bit patterns: 1.0 = 0x3F80, -2.0 = 0xC000, 0.5 = 0x3F00, 3.140625 = 0x4049
    bits = np.array([0x3F80, 0xC000, 0x3F00, 0x4049, 0x0000, 0x8000], np.uint16)
    assert O.widen(bits).tolist() == [1.0, -2.0, 0.5, 3.140625, 0.0, -0.0]
    # the generator's rounding is nearest-even onto values with an 8-bit significand
    vals = np.array([1.0, 1.00390625, 1.01171875, 1.0 + 2 ** -9, -(1.0 + 3 * 2 ** -9)], np.float32)
    back = O.widen(synth.f32_to_bf16_bits(vals))
    #   1+2^-8 is a tie between 1 and 1+2^-7 -> even (1.0); 1+3*2^-8 is a tie -> even (1+2^-6)
    assert back.tolist() == [1.0, 1.0, 1.015625, 1.0, -1.0078125]
    x = _rng(5).standard_normal(4096).astype(np.float32)
    b = O.widen(synth.f32_to_bf16_bits(x))
    assert np.max(np.abs(b - x) / np.abs(x)) <= 2.0 ** -8              # half an ulp of an 8-bit significand
    import torch
    tb = torch.from_numpy(x).to(torch.bfloat16).to(torch.float64).numpy()
    assert (tb == b).all()                                            # independent RNE implementation


# --------------------------------------------------------------------------- expert FFN

def _loop_ffn_row(xrow, wg, wu, wd):
    """One row, scalar Python loops (no matmul, no vector ops)."""
    f, d = len(wg), len(xrow)
    h = []
    for n in range(f):
        g = math.fsum(xrow[c] * wg[n][c] for c in range(d))
        u = math.fsum(xrow[c] * wu[n][c] for c in range(d))
        h.append(g / (1.0 + math.exp(-g)) * u)
    return [math.fsum(h[n] * wd[c][n] for n in range(f)) for c in range(d)]


def test_ffn_tiny_integer_case_by_hand():
    # one expert, one row, d=2, f=2; numbers small enough to check on paper:
    # g = [1*1+2*0, 1*0+2*1] = [1, 2]; u = [1*2+2*1, 1*(-1)+2*1] = [4, 1]
    # h = [silu(1)*4, silu(2)*1]; y = [h0*1 + h1*2, h0*(-1) + h1*0.5]
    xp = np.array([[1.0, 2.0]])
    wg = np.array([[1.0, 0.0], [0.0, 1.0]])
    wu = np.array([[2.0, 1.0], [-1.0, 1.0]])
    wd = np.array([[1.0, 2.0], [-1.0, 0.5]])
    y, h = O.expert_ffn(xp, np.array([0, 1]), [(wg, wu, wd)], return_h=True)
    s1, s2 = 1 / (1 + math.exp(-1)), 2 / (1 + math.exp(-2))
    np.testing.assert_allclose(h[0], [4 * s1, s2], rtol=1e-15)
    np.testing.assert_allclose(y[0], [4 * s1 + 2 * s2, -4 * s1 + 0.5 * s2], rtol=1e-15)


def test_ffn_matches_scalar_loops_and_respects_segments():
    rng = _rng(11)
    T, d, f, E, k = 7, 5, 3, 3, 2          # non-square on purpose: a transposed operand cannot pass
    x = rng.standard_normal((T, d))
    W = [(rng.standard_normal((f, d)), rng.standard_normal((f, d)), rng.standard_normal((d, f))) for _ in range(E)]
    idx, w, counts, offsets = O.route(rng.standard_normal((T, E)).astype(np.float32), k)
    xp, pos, src = O.dispatch(x, idx, offsets)
    y = O.expert_ffn(xp, offsets, W)
    row_expert = idx.ravel()[src]
    for r in range(T * k):
        wg, wu, wd = W[row_expert[r]]
        ref = _loop_ffn_row(xp[r].tolist(), wg.tolist(), wu.tolist(), wd.tolist())
        np.testing.assert_allclose(y[r], ref, rtol=1e-12, atol=1e-13)


def test_ffn_special_cases():
    rng = _rng(12)
    d, f = 6, 10
    xp = rng.standard_normal((9, d))
    wg, wu, wd = rng.standard_normal((f, d)), rng.standard_normal((f, d)), rng.standard_normal((d, f))
    offs = np.array([0, 9])
    y = O.expert_ffn(xp, offs, [(wg, wu, wd)])
    # zero gate => silu(0) = 0 => y == 0 exactly
    assert (O.expert_ffn(xp, offs, [(np.zeros_like(wg), wu, wd)]) == 0).all()
    # zero up => 0
    assert (O.expert_ffn(xp, offs, [(wg, np.zeros_like(wu), wd)]) == 0).all()
    # doubling W_down doubles y exactly (power of two); y is linear in W_up too
    assert (O.expert_ffn(xp, offs, [(wg, wu, 2 * wd)]) == 2 * y).all()
    assert (O.expert_ffn(xp, offs, [(wg, 2 * wu, wd)]) == 2 * y).all()
    # large positive gate pre-activation: silu(g) -> g, so y -> ((x Wg^T) * (x Wu^T)) Wd^T
    xpos = np.abs(xp) + 1.0
    wbig = np.abs(wg) * 50 + 50
    ybig = O.expert_ffn(xpos, offs, [(wbig, wu, wd)])
    np.testing.assert_allclose(ybig, ((xpos @ wbig.T) * (xpos @ wu.T)) @ wd.T, rtol=1e-12)
    # large negative gate: silu -> 0
    assert np.abs(O.expert_ffn(xpos, offs, [(-wbig, wu, wd)])).max() < 1e-15
    # silu is not symmetric: flipping the sign of the gate changes the result (catches silu(-g))
    assert not np.allclose(O.expert_ffn(xp, offs, [(-wg, wu, wd)]), y)
    # swapping the roles of gate and up changes the result (catches silu applied to the wrong branch)
    assert not np.allclose(O.expert_ffn(xp, offs, [(wu, wg, wd)]), y)
    # empty experts are skipped and never asked for weights
    def get(e):
        assert e == 1
        return wg, wu, wd
    y2 = O.expert_ffn(xp, np.array([0, 0, 9, 9]), get)
    assert (y2 == y).all()


def test_ffn_bf16_inputs_are_widened_not_rounded():
    rng = _rng(13)
    cfg = synth.LayerConfig("t", T=4, d=8, f=4, E=1, k=1, dtype="bf16", router="logits")
    wg, wu, wd = synth.make_expert_weights(cfg, 0, 0)
    xp = synth.f32_to_bf16_bits(rng.standard_normal((4, 8)).astype(np.float32))
    y_bits = O.expert_ffn(xp, np.array([0, 4]), [(wg, wu, wd)])
    y_f64 = O.expert_ffn(O.widen(xp), np.array([0, 4]), [(O.widen(wg), O.widen(wu), O.widen(wd))])
    assert (y_bits == y_f64).all()


# --------------------------------------------------------------------------- combine

def test_combine_identity_experts_returns_input():
    """With 'identity experts' (y := xp) the combine returns x, because the weights sum to 1."""
    rng = _rng(21)
    T, E, k, d = 50, 8, 3, 12
    x = rng.standard_normal((T, d))
    idx, w, _, offsets = O.route(rng.standard_normal((T, E)).astype(np.float32), k)
    xp, pos, _ = O.dispatch(x, idx, offsets)
    np.testing.assert_allclose(O.combine(xp, pos, w), x, rtol=1e-14, atol=1e-15)


def test_combine_k1_is_a_gather_and_weights_matter():
    rng = _rng(22)
    T, E, d = 20, 4, 6
    y = rng.standard_normal((T, d))
    idx, w, _, offsets = O.route(rng.standard_normal((T, E)).astype(np.float32), 1)
    _, pos, _ = O.dispatch(y, idx, offsets)
    assert (O.combine(y, pos, w) == y[pos[:, 0]]).all()
    # explicit tiny case: out = 0.25*row2 + 0.75*row0
    y3 = np.array([[1.0, 2.0], [100.0, 100.0], [10.0, 20.0]])
    out = O.combine(y3, np.array([[2, 0]], np.int32), np.array([[0.25, 0.75]]))
    assert out.tolist() == [[0.25 * 10 + 0.75 * 1, 0.25 * 20 + 0.75 * 2]]


# --------------------------------------------------------------------------- whole layer

def _dense_layer_token(xt, logit_row, k, W):
    """out[t] = sum over the token's top-k experts of w_e * FFN_e(x_t): no dispatch, no
    packing, scalar loops only. Top-k by brute force, weights by direct softmax."""
    picks = _brute_topk(logit_row, k)
    z = [math.exp(float(logit_row[e]) - float(logit_row[picks[0]])) for e in picks]
    s = math.fsum(z)
    out = [0.0] * len(xt)
    for e, ze in zip(picks, z):
        wg, wu, wd = W[e]
        ye = _loop_ffn_row(list(xt), wg.tolist(), wu.tolist(), wd.tolist())
        out = [o + (ze / s) * v for o, v in zip(out, ye)]
    return out


def test_whole_layer_matches_dense_per_token_brute_force():
    rng = _rng(31)
    T, d, f, E, k = 9, 4, 3, 5, 2
    x = rng.standard_normal((T, d))
    logits = rng.integers(-1, 2, size=(T, E)).astype(np.float32)         # ties included
    logits[::2] = rng.standard_normal((len(logits[::2]), E)).astype(np.float32)
    W = [(rng.standard_normal((f, d)), rng.standard_normal((f, d)), rng.standard_normal((d, f))) for _ in range(E)]
    res = O.moe_layer(x, logits, k, W)
    for t in range(T):
        np.testing.assert_allclose(res["out"][t], _dense_layer_token(x[t], logits[t], k, W), rtol=1e-12, atol=1e-13)
    # the per-token sampler used at full size agrees too
    sample = [8, 0, 3]
    got = O.token_outputs(x, res["topk_idx"], res["topk_w"], sample, W)
    for n, t in enumerate(sample):
        np.testing.assert_allclose(got[n], _dense_layer_token(x[t], logits[t], k, W), rtol=1e-12, atol=1e-13)


def test_whole_layer_token_permutation_equivariance():
    rng = _rng(32)
    cfg = synth.LayerConfig("t", T=24, d=16, f=8, E=6, k=3, dtype="f32", router="logits")
    x = synth.make_activations(cfg, 1)
    logits = synth.make_logits(cfg, 1)
    W = [synth.make_expert_weights(cfg, 1, e) for e in range(cfg.E)]
    perm = rng.permutation(cfg.T)
    a = O.moe_layer(x, logits, cfg.k, W)["out"]
    b = O.moe_layer(x[perm], logits[perm], cfg.k, W)["out"]
    np.testing.assert_allclose(b, a[perm], rtol=1e-13, atol=1e-14)


def test_single_expert_layer_is_a_dense_swiglu_mlp():
    rng = _rng(33)
    T, d, f = 10, 6, 4
    x = rng.standard_normal((T, d))
    wg, wu, wd = rng.standard_normal((f, d)), rng.standard_normal((f, d)), rng.standard_normal((d, f))
    out = O.moe_layer(x, np.zeros((T, 1), np.float32), 1, [(wg, wu, wd)])["out"]
    import torch
    xt, g, u, dn = (torch.from_numpy(a) for a in (x, wg, wu, wd))
    ref = torch.nn.functional.linear(torch.nn.functional.silu(torch.nn.functional.linear(xt, g))
                                     * torch.nn.functional.linear(xt, u), dn)
    np.testing.assert_allclose(out, ref.numpy(), rtol=1e-12, atol=1e-13)


def test_gate_logits_against_loops():
    rng = _rng(41)
    x = rng.standard_normal((5, 7)).astype(np.float32)
    wr = rng.standard_normal((3, 7)).astype(np.float32)
    lg = O.gate_logits(x, wr)
    assert lg.dtype == np.float32 and lg.shape == (5, 3)
    for t in range(5):
        for e in range(3):
            assert lg[t, e] == np.float32(math.fsum(float(x[t, c]) * float(wr[e, c]) for c in range(7)))


def test_tiny_config_end_to_end_invariants():
    cfg = synth.CONFIGS["tiny_fp32"]
    x = synth.make_activations(cfg)
    logits = O.gate_logits(x, synth.make_router_weight(cfg))
    W = [synth.make_expert_weights(cfg, 0, e) for e in range(cfg.E)]
    res = O.moe_layer(x, logits, cfg.k, W)
    assert res["counts"].sum() == cfg.T * cfg.k
    assert res["out"].shape == (cfg.T, cfg.d) and np.isfinite(res["out"]).all()
    # x ~ N(0,1), weights N(0,1/fan_in): outputs are O(1), not degenerate
    assert 0.01 < np.abs(res["out"]).mean() < 10


def test_bf16_store_diagnostic_rounds_like_the_input_generator_and_stays_close():
    """round_to_bf16 against the generators' own float32 -> bfloat16 conversion (written separately), and the
    store_bf16 diagnostic against the definition: it may move y by bf16 rounding only."""
    rng = _rng(77)
    a = rng.standard_normal(5000) * np.exp(rng.uniform(-20, 20, 5000))
    a[:4] = [0.0, -0.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8]           # two exact ties: to even
    via_bits = O.widen(synth.f32_to_bf16_bits(a.astype(np.float32)))
    np.testing.assert_array_equal(O.round_to_bf16(a), via_bits)
    assert O.round_to_bf16(np.array([1.0 + 2.0 ** -8]))[0] == 1.0 and O.round_to_bf16(np.array([1.0 + 3 * 2.0 ** -8]))[0] == 1.0 + 2.0 ** -6
    E, d, f = 3, 16, 24
    offsets = np.array([0, 5, 5, 12])
    xp = rng.standard_normal((12, d))
    W = [(rng.standard_normal((f, d)) / 4, rng.standard_normal((f, d)) / 4, rng.standard_normal((d, f)) / 5) for _ in range(E)]
    y = O.expert_ffn(xp, offsets, W)
    yb = O.expert_ffn(xp, offsets, W, store_bf16=True)
    err = np.linalg.norm(yb - y) / np.linalg.norm(y)
    assert 1e-4 < err < 2 ** -7                                          # two bf16 roundings, nothing more
