"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded
inputs. Integer outputs (indices, counts, offsets, permutations, copied rows) must be bit-exact;
token weights within a few float32 roundings (w_tol below); floating-point tensors within relative Frobenius error 1e-5 (fp32) or
1e-2 (bf16)."""
import numpy as np
import pytest
import torch

from oracle import moe_oracle as O
from paper_2504_02263_amd import binding as B
from workloads import synth

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 1e-2}


def w_tol(k: int) -> float:
    """Bound on |w_gpu - w_oracle| for the softmax over k picks, float32 on the GPU against float64.
    With u = 2^-24 (rounding to nearest) and weights <= 1: expf is within 1 ulp = 2u, in the numerator and
    (as a weighted mean) in the denominator: 4u; the subtraction l_j - l_0 is rounded, which moves exp by
    u*|x|e^-|x| <= 0.37u, twice: 0.74u; the k-term sum rounds k - 1 times: (k - 1)u; the division: u.
    Together (4.74 + k)u, rounded up to (5 + k)u: 4.2e-7 at k = 2, 6.6e-7 at k = 6; never looser than 1e-6."""
    return min(1e-6, (5 + k) * 2.0 ** -24)


def dev(a: np.ndarray) -> torch.Tensor:
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t: torch.Tensor) -> np.ndarray:
    """Device tensor -> numpy at storage precision (bf16 comes back as uint16 bits)."""
    if t.dtype == torch.bfloat16:
        return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def rel_fro(gpu: np.ndarray, ref: np.ndarray) -> float:
    g = O.widen(gpu)
    den = np.linalg.norm(ref)
    return float(np.linalg.norm(g - ref) / den) if den > 0 else float(np.linalg.norm(g))


def small_cfg(T, d, f, E, k, dtype):
    return synth.LayerConfig(f"t{T}_{d}_{f}_{E}_{k}_{dtype}", T=T, d=d, f=f, E=E, k=k, dtype=dtype, router="logits")


def run_layer(cfg, x, logits, W, T_max=None):
    """Full path on the GPU; returns the MoEPath (buffers hold every intermediate)."""
    path = B.MoEPath(T_max or max(cfg.T, 1), cfg.d, cfg.f, cfg.E, cfg.k, cfg.dtype)
    path.pack_weights(dev(W[0]), dev(W[1]), dev(W[2]))
    path.forward(dev(x), dev(logits))
    torch.cuda.synchronize()
    return path


def check_integers(path, ref, T, k):
    A = T * k
    assert (host(path.topk_idx)[:T] == ref["topk_idx"]).all()
    assert (host(path.counts) == ref["counts"]).all()
    assert (host(path.offsets) == ref["offsets"]).all()
    assert (host(path.pos)[:T] == ref["pos"]).all()
    assert (host(path.src)[:A] == ref["src"]).all()
    assert (host(path.xp)[:A] == ref["xp"]).all()                 # rows are copied bit for bit
    np.testing.assert_allclose(host(path.topk_w)[:T], ref["topk_w"], rtol=0, atol=w_tol(k))


# ------------------------------------------------------------------------------- route

@pytest.mark.parametrize("T,E,k", [(1, 8, 2), (64, 8, 2), (257, 8, 1), (1000, 16, 4), (513, 32, 4), (700, 64, 6),
                                   (300, 5, 5), (129, 100, 7), (64, 256, 8), (33, 3, 2), (4096, 8, 2), (0, 8, 2)])
def test_route_bit_exact(T, E, k):
    rng = np.random.default_rng(T * 1000 + E * 10 + k)
    logits = rng.standard_normal((T, E)).astype(np.float32)
    if T > 8:
        logits[::5] = rng.integers(-1, 2, size=logits[::5].shape).astype(np.float32)   # heavy ties
        logits[1] = 0.0
        logits[2] = np.arange(E, dtype=np.float32)
        logits[3] = -np.arange(E, dtype=np.float32)
        logits[4, : E // 2] = -0.0
        logits[4, E // 2:] = 0.0
    idx, w, counts, offsets = O.route(logits, k)
    ctx = B.moe_create(max(T, 1), 128, 128, E, k, "f32")
    g_idx = torch.full((max(T, 1), k), -7, dtype=torch.int32, device="cuda")
    g_w = torch.zeros((max(T, 1), k), dtype=torch.float32, device="cuda")
    g_counts = torch.full((E,), -7, dtype=torch.int32, device="cuda")
    g_offsets = torch.full((E + 1,), -7, dtype=torch.int32, device="cuda")
    B.moe_route(ctx, T, dev(logits) if T else torch.zeros(4, device="cuda"), g_idx, g_w, g_counts, g_offsets)
    torch.cuda.synchronize()
    B.moe_destroy(ctx)
    assert (host(g_idx)[:T] == idx).all()
    assert (host(g_counts) == counts).all()
    assert (host(g_offsets) == offsets).all()
    np.testing.assert_allclose(host(g_w)[:T], w, rtol=0, atol=w_tol(k))
    if T:
        np.testing.assert_allclose(host(g_w)[:T].sum(1), 1.0, rtol=0, atol=4e-7)


# ------------------------------------------------------------------------------- dispatch / combine

@pytest.mark.parametrize("T,E,k,d,dtype", [(64, 8, 2, 256, "f32"), (1000, 16, 4, 128, "bf16"), (777, 64, 6, 384, "bf16"),
                                           (5000, 8, 2, 128, "f32"), (3, 4, 1, 128, "bf16"), (2731, 64, 6, 256, "bf16")])
def test_dispatch_and_combine(T, E, k, d, dtype):
    cfg = small_cfg(T, d, 128, E, k, dtype)
    x = synth.make_activations(cfg, 3)
    logits = synth.make_logits(cfg, 3)
    logits[:, E - 1] = -50.0 if E > k else logits[:, E - 1]        # one empty expert where possible
    idx, w, counts, offsets = O.route(logits, k)
    xp, pos, src = O.dispatch(x, idx, offsets)
    path = B.MoEPath(T, d, 128, E, k, dtype)
    path.route(dev(logits))
    path.dispatch(dev(x))
    torch.cuda.synchronize()
    A = T * k
    assert (host(path.pos) == pos).all()
    assert (host(path.src)[:A] == src).all()
    assert (host(path.xp)[:A] == xp).all()
    first = (path.pos.clone(), path.src.clone(), path.xp.clone())
    xd = dev(x)
    same = torch.ones((), dtype=torch.bool, device="cuda")
    for _ in range(100):                                          # same answer every time (no atomics-order effects)
        path.pos.fill_(-1)
        path.dispatch(xd)
        same &= torch.equal(path.pos, first[0]) & torch.equal(path.src, first[1]) & torch.equal(path.xp, first[2])
    torch.cuda.synchronize()
    assert bool(same)
    # identity experts: y := xp, so combine must return x (weights sum to 1)
    path.y.copy_(path.xp)
    path.combine(T)
    torch.cuda.synchronize()
    ref = O.combine(xp, pos, w)
    assert rel_fro(host(path.out), ref) <= (1e-6 if dtype == "f32" else 4e-3)
    assert rel_fro(host(path.out), O.widen(x)) <= (1e-6 if dtype == "f32" else 4e-3)
    # a real weighted sum of unrelated rows
    yy = synth.make_activations(small_cfg(A, d, 128, E, k, dtype), 9)
    path.y.copy_(dev(yy))
    path.combine(T)
    torch.cuda.synchronize()
    assert rel_fro(host(path.out), O.combine(yy, pos, host(path.topk_w))) <= (1e-6 if dtype == "f32" else 4e-3)
    path.close()


# ------------------------------------------------------------------------------- expert FFN

FFN_CASES = [
    # T, d, f, E, k, dtype : spans every m-tile height (mean rows/expert 10..350), both ring depths
    (40, 256, 512, 8, 2, "bf16"), (160, 256, 512, 8, 2, "bf16"), (320, 256, 512, 8, 2, "bf16"),
    (800, 256, 512, 8, 2, "bf16"), (700, 384, 640, 4, 2, "bf16"), (100, 384, 128, 16, 4, "bf16"),
    (333, 128, 384, 64, 6, "bf16"), (64, 256, 512, 8, 2, "f32"), (300, 128, 384, 5, 3, "f32"),
    # large-batch kernel: shortest possible K loop (2 chunks), ragged multi-tile segments, one 32-row group
    (600, 128, 128, 2, 1, "bf16"), (1100, 256, 384, 3, 2, "bf16"), (150, 128, 256, 1, 1, "bf16"),
    # large-batch kernel with many segments in a short launch (tiles ranked by height across 64 and 200 experts)
    (2000, 128, 128, 64, 8, "bf16"), (3000, 128, 128, 200, 16, "bf16"),
]


@pytest.mark.parametrize("T,d,f,E,k,dtype", FFN_CASES)
def test_layer_small(T, d, f, E, k, dtype):
    cfg = small_cfg(T, d, f, E, k, dtype)
    x = synth.make_activations(cfg, 1)
    logits = synth.make_logits(cfg, 1)
    if E > k + 1:
        logits[:, 1] = -60.0                                       # expert 1 gets no tokens
    W = synth.make_all_expert_weights(cfg, 1, workers=4)
    ref = O.moe_layer(x, logits, k, lambda e: (W[0][e], W[1][e], W[2][e]))
    y_ref, h_ref = O.expert_ffn(ref["xp"], ref["offsets"], lambda e: (W[0][e], W[1][e], W[2][e]), return_h=True)
    path = run_layer(cfg, x, logits, W)
    A = T * k
    check_integers(path, ref, T, k)
    tol = TOL[dtype]
    eh, ey, eo = rel_fro(host(path.h)[:A], h_ref), rel_fro(host(path.y)[:A], y_ref), rel_fro(host(path.out)[:T], ref["out"])
    print(f"{cfg.name}: rel-Frobenius h {eh:.2e}  y {ey:.2e}  out {eo:.2e}")
    assert eh <= tol and ey <= tol and eo <= tol
    path.close()


def test_ffn_arbitrary_offsets_and_smaller_T_than_T_max():
    """moe_expert_ffn is a function of (xp, offsets) alone: very uneven hand-made segments."""
    d, f, E, k = 256, 384, 6, 1
    sizes = [0, 5, 0, 600, 1, 33]
    A = sum(sizes)
    offsets = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    cfg = small_cfg(A, d, f, E, k, "bf16")
    xp = synth.make_activations(cfg, 5)
    W = synth.make_all_expert_weights(cfg, 5, workers=4)
    y_ref, h_ref = O.expert_ffn(xp, offsets, lambda e: (W[0][e], W[1][e], W[2][e]), return_h=True)
    path = B.MoEPath(A + 100, d, f, E, k, "bf16")
    path.pack_weights(dev(W[0]), dev(W[1]), dev(W[2]))
    path.xp[:A].copy_(dev(xp))
    path.offsets.copy_(dev(offsets))
    path.y.fill_(7.0)
    path.expert_ffn(A)
    torch.cuda.synchronize()
    assert rel_fro(host(path.h)[:A], h_ref) <= 1e-2
    assert rel_fro(host(path.y)[:A], y_ref) <= 1e-2
    assert (path.y[A:] == 7.0).all()                               # nothing written past the last row
    path.close()


def test_tiny_fp32_config():
    """The tiny fp32 layer: logits from the gating matrix (computed once, on the host, and routed by both sides)."""
    cfg = synth.CONFIGS["tiny_fp32"]
    x = synth.make_activations(cfg)
    logits = O.gate_logits(x, synth.make_router_weight(cfg))
    W = synth.make_all_expert_weights(cfg, 0, workers=4)
    ref = O.moe_layer(x, logits, cfg.k, lambda e: (W[0][e], W[1][e], W[2][e]))
    path = run_layer(cfg, x, logits, W)
    check_integers(path, ref, cfg.T, cfg.k)
    err = rel_fro(host(path.out), ref["out"])
    print(f"tiny_fp32: rel-Frobenius out {err:.2e}")
    assert err <= 1e-5
    path.close()


def test_empty_batch():
    path = B.MoEPath(16, 128, 128, 8, 2, "bf16")
    path.packed = torch.zeros(B.moe_packed_weight_bytes(16, 128, 128, 8, 2, "bf16"), dtype=torch.uint8, device="cuda")
    path.counts.fill_(-1)
    path.offsets.fill_(-1)
    x = torch.zeros((0, 128), dtype=torch.bfloat16, device="cuda")
    path.route(torch.zeros(4, device="cuda"), T=0)
    path.dispatch(path.xp, T=0)
    path.expert_ffn(0)
    path.combine(0)
    torch.cuda.synchronize()
    assert (path.counts == 0).all() and (path.offsets == 0).all()
    path.close()


def test_calls_run_on_the_given_stream():
    cfg = small_cfg(200, 256, 256, 8, 2, "bf16")
    x, logits = synth.make_activations(cfg, 2), synth.make_logits(cfg, 2)
    W = synth.make_all_expert_weights(cfg, 2, workers=4)
    ref = O.moe_layer(x, logits, cfg.k, lambda e: (W[0][e], W[1][e], W[2][e]))
    path = B.MoEPath(cfg.T, cfg.d, cfg.f, cfg.E, cfg.k, cfg.dtype)
    path.pack_weights(dev(W[0]), dev(W[1]), dev(W[2]))
    xd, ld = dev(x), dev(logits)
    torch.cuda.synchronize()
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        path.forward(xd, ld)           # binding picks up torch's current stream
    path.forward(xd, ld, stream=s)     # and an explicit one
    s.synchronize()
    assert rel_fro(host(path.out), ref["out"]) <= 1e-2
    path.close()


@pytest.mark.parametrize("T,d,f,E,k", [(200, 256, 512, 8, 2), (700, 256, 256, 16, 4)])
def test_layer_replays_from_a_hip_graph(T, d, f, E, k):
    """The hot calls allocate nothing, never synchronise and record no memset, so a caller may capture
    the whole layer into a HIP graph. Every replay (new inputs in the same buffers, eager work and
    synchronisations in between) must reproduce the eager result bit for bit."""
    cfg = small_cfg(T, d, f, E, k, "bf16")
    W = synth.make_all_expert_weights(cfg, 4, workers=4)
    path = B.MoEPath(cfg.T, cfg.d, cfg.f, cfg.E, cfg.k, cfg.dtype)
    path.pack_weights(dev(W[0]), dev(W[1]), dev(W[2]))
    inputs = [(dev(synth.make_activations(cfg, s)), dev(synth.make_logits(cfg, s))) for s in (10, 11, 12, 13)]
    eager = []
    for xd, ld in inputs:
        path.forward(xd, ld)
        torch.cuda.synchronize()
        eager.append([host(t).copy() for t in (path.topk_idx, path.offsets, path.pos, path.src, path.xp, path.y, path.out)])
    xs, ls = torch.empty_like(inputs[0][0]), torch.empty_like(inputs[0][1])
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                      # warm-up on the capture stream's side, as torch asks
        xs.copy_(inputs[0][0]); ls.copy_(inputs[0][1])
        path.forward(xs, ls)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        path.forward(xs, ls)
    for rep in (1, 2, 3, 1, 0):
        xs.copy_(inputs[rep][0]); ls.copy_(inputs[rep][1])
        path.out.zero_(); path.y.zero_(); path.xp.zero_()          # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = [host(t) for t in (path.topk_idx, path.offsets, path.pos, path.src, path.xp, path.y, path.out)]
        for a, b in zip(got, eager[rep]):
            assert (a == b).all(), f"replay of input {rep} differs from the eager run"
    del graph
    path.close()


# ------------------------------------------------------------------------------- fused gate GEMM + routing

@pytest.mark.parametrize("T,d,E,k,dtype", [(64, 256, 8, 2, "f32"), (257, 384, 16, 4, "bf16"), (1000, 512, 64, 6, "bf16"),
                                           (70, 128, 100, 7, "bf16"), (33, 256, 256, 8, "f32"), (5, 128, 5, 3, "bf16"),
                                           (256, 6144, 8, 2, "bf16"), (45, 256, 32, 4, "bf16"), (40, 128, 256, 8, "bf16"),
                                           (333, 1024, 17, 5, "bf16"), (100, 384, 128, 64, "bf16")])
def test_gate_route(T, d, E, k, dtype):
    """moe_gate_route: the gate scores against the oracle's float64 product, and the routing
    bit-exact against the oracle routed on the very logits the GPU produced."""
    cfg = small_cfg(T, d, 128, E, k, dtype)
    x = synth.make_activations(cfg, 4)
    w_r = synth.make_router_weight(cfg, 4)
    path = B.MoEPath(T, d, 128, E, k, dtype)
    logits = torch.full((T, E), 7.0, dtype=torch.float32, device="cuda")
    path.gate_route(dev(x), dev(w_r), logits)
    torch.cuda.synchronize()
    g_logits = host(logits)
    ref_logits = O.gate_logits(x, w_r)
    err = float(np.linalg.norm(g_logits - ref_logits.astype(np.float64)) / np.linalg.norm(ref_logits))
    assert err <= 1e-5, err
    idx, w, counts, offsets = O.route(g_logits, k)
    assert (host(path.topk_idx)[:T] == idx).all()
    assert (host(path.counts) == counts).all() and (host(path.offsets) == offsets).all()
    np.testing.assert_allclose(host(path.topk_w)[:T], w, rtol=0, atol=w_tol(k))
    # without the logits output the routing is the same
    first = host(path.topk_idx).copy()
    path.gate_route(dev(x), dev(w_r), None)
    torch.cuda.synchronize()
    assert (host(path.topk_idx) == first).all() and (host(path.counts) == counts).all()
    path.close()


# ------------------------------------------------------------------------------- more edge cases

def test_route_largest_supported_k_and_E():
    """E = 256 experts with k = 64 picks: four experts per lane, one lane per pick."""
    T, E, k = 37, 256, 64
    rng = np.random.default_rng(5)
    logits = rng.standard_normal((T, E)).astype(np.float32)
    logits[::4] = rng.integers(-2, 3, size=logits[::4].shape).astype(np.float32)
    idx, w, counts, offsets = O.route(logits, k)
    path = B.MoEPath(T, 128, 128, E, k, "f32")
    path.route(dev(logits))
    torch.cuda.synchronize()
    assert (host(path.topk_idx) == idx).all() and (host(path.counts) == counts).all()
    assert (host(path.offsets) == offsets).all()
    np.testing.assert_allclose(host(path.topk_w), w, rtol=0, atol=w_tol(k))
    path.close()


def test_route_nan_and_inf_logits_follow_the_documented_rule():
    """NaN ranks as -inf; -inf is an ordinary (smallest) value; ties still go to the lower index."""
    logits = np.array([[np.nan, 1.0, 2.0, np.nan], [-np.inf, -np.inf, 0.5, -np.inf], [np.inf, 1.0, np.inf, 0.0]],
                      np.float32)
    canon = np.where(np.isnan(logits), -np.inf, logits).astype(np.float32)
    idx, _, counts, offsets = O.route(canon, 3)
    path = B.MoEPath(3, 128, 128, 4, 3, "f32")
    path.route(dev(logits))
    torch.cuda.synchronize()
    assert (host(path.topk_idx) == idx).all()
    assert idx.tolist() == [[2, 1, 0], [2, 0, 1], [0, 2, 1]]
    assert (host(path.counts) == counts).all() and (host(path.offsets) == offsets).all()
    path.close()


def test_expert_ffn_equals_its_two_stages_and_is_deterministic():
    cfg = small_cfg(500, 256, 384, 6, 2, "bf16")
    x, logits = synth.make_activations(cfg, 6), synth.make_logits(cfg, 6)
    W = synth.make_all_expert_weights(cfg, 6, workers=4)
    path = run_layer(cfg, x, logits, W)
    A = cfg.T * cfg.k
    h1, y1 = host(path.h)[:A].copy(), host(path.y)[:A].copy()
    path.h.zero_()
    path.y.zero_()
    path.ffn_input(cfg.T)
    path.ffn_output(cfg.T)
    torch.cuda.synchronize()
    assert (host(path.h)[:A] == h1).all() and (host(path.y)[:A] == y1).all()      # bitwise
    for _ in range(3):
        path.expert_ffn(cfg.T)
    torch.cuda.synchronize()
    assert (host(path.h)[:A] == h1).all() and (host(path.y)[:A] == y1).all()
    path.close()


@pytest.mark.parametrize("T,d,f,E,k", [(1500, 256, 384, 4, 2), (3000, 512, 256, 6, 3), (900, 384, 1024, 3, 1)])
def test_both_gemm_kernels_give_the_same_bits(T, d, f, E, k):
    """Which GEMM kernel a launch runs is picked on the host from the expected rows per segment. Both
    accumulate K in the same order with the same matrix-core instruction, so the pick must never show in a
    result: the same rows through the streaming kernel (small rows hint) and the large-batch kernel (true hint)."""
    cfg = small_cfg(T, d, f, E, k, "bf16")
    x, logits = synth.make_activations(cfg, 3), synth.make_logits(cfg, 3)
    W = synth.make_all_expert_weights(cfg, 3, workers=4)
    path = run_layer(cfg, x, logits, W)
    A = T * k
    seg_e = torch.arange(E, dtype=torch.int32, device="cuda")
    beg, end = path.offsets[:E].clone(), path.offsets[1:E + 1].clone()
    got = []
    for hint in (8 * E, A):
        path.h.zero_()
        path.y.zero_()
        B.moe_expert_ffn_segments(path.ctx, T, E, hint, path.xp, beg, end, seg_e, path.packed, path.h, path.y)
        torch.cuda.synchronize()
        got.append((host(path.h)[:A].copy(), host(path.y)[:A].copy()))
    assert (got[0][0] == got[1][0]).all() and (got[0][1] == got[1][1]).all()
    path.close()


def test_all_tokens_to_one_expert():
    """Degenerate routing: every token picks the same experts (k = 2 of 4), so two segments hold
    all rows and two are empty."""
    cfg = small_cfg(300, 128, 256, 4, 2, "bf16")
    x = synth.make_activations(cfg, 8)
    logits = np.tile(np.array([[5.0, -5.0, 4.0, -6.0]], np.float32), (cfg.T, 1))
    W = synth.make_all_expert_weights(cfg, 8, workers=4)
    ref = O.moe_layer(x, logits, cfg.k, lambda e: (W[0][e], W[1][e], W[2][e]))
    assert ref["counts"].tolist() == [300, 0, 300, 0]
    path = run_layer(cfg, x, logits, W)
    check_integers(path, ref, cfg.T, cfg.k)
    assert rel_fro(host(path.out), ref["out"]) <= 1e-2
    path.close()


@pytest.mark.parametrize("T,E,k,d,dtype", [(1, 8, 2, 256, "bf16"), (256, 8, 2, 512, "bf16"), (512, 8, 4, 128, "bf16"),
                                           (513, 8, 2, 128, "bf16"), (300, 64, 6, 256, "bf16"), (32, 256, 64, 128, "f32"),
                                           (341, 16, 4, 384, "f32"), (2000, 8, 2, 128, "bf16")])
def test_route_dispatch_one_call_equals_the_two_calls(T, E, k, d, dtype):
    """moe_route_dispatch (a single launch up to T = 512, T*k = 2048; the four kernels beyond) against the
    oracle and against moe_route + moe_dispatch: integers and copied rows bit for bit, weights identical."""
    cfg = small_cfg(T, d, 128, E, k, dtype)
    x = synth.make_activations(cfg, 21)
    logits = synth.make_logits(cfg, 21)
    logits[::5, : min(E, 3)] = 0.5                                   # ties inside the top-k
    idx, w, counts, offsets = O.route(logits, k)
    xp, pos, src = O.dispatch(x, idx, offsets)
    ref = dict(topk_idx=idx, topk_w=w, counts=counts, offsets=offsets, xp=xp, pos=pos, src=src)
    a = B.MoEPath(T, d, 128, E, k, dtype)
    b = B.MoEPath(T, d, 128, E, k, dtype)
    xd, ld = dev(x), dev(logits)
    for p in (a, b):
        for t in (p.topk_idx, p.pos, p.src, p.counts, p.offsets):
            t.fill_(-7)
        p.xp.zero_()
    a.route_dispatch(xd, ld)
    b.route(ld)
    b.dispatch(xd)
    torch.cuda.synchronize()
    check_integers(a, ref, T, k)
    for name in ("topk_idx", "topk_w", "counts", "offsets", "xp", "pos", "src"):
        assert torch.equal(getattr(a, name), getattr(b, name)), name
    a.close()
    b.close()


def test_roofline_probes_run_and_report_their_work():
    """The two measuring kernels: argument handling and reported work (their rates are bench.py's business)."""
    path = B.MoEPath(8, 128, 128, 2, 1, "bf16")
    buf = torch.randint(0, 255, (8 * 1024 * 1024 + 100,), dtype=torch.uint8, device="cuda")
    sink = torch.zeros(16, dtype=torch.float32, device="cuda")
    got = B.moe_probe_stream_read(path.ctx, buf, buf.numel(), sink)
    assert 0 < got <= buf.numel() and got % (4096 * 1024) == 0       # whole 1 KiB loads for each of 4096 wavefronts
    assert B.moe_probe_stream_read(path.ctx, buf, 1000, sink) == 0     # too small for one load per wavefront: nothing runs
    flops = B.moe_probe_mfma(path.ctx, buf, 10, 8, sink)
    assert flops == 8 * 4 * 10 * 16 * 2 * 32 * 32 * 16
    torch.cuda.synchronize()
    assert float(sink.abs().sum()) == 0.0                              # the sink is only a place the kernels may write
    with pytest.raises(B.MoeError):
        B.moe_probe_mfma(path.ctx, buf, -1, 8, sink)
    path.close()


@pytest.mark.parametrize("T,d,f,E,k", [(160, 256, 512, 8, 2), (1100, 256, 384, 3, 2), (333, 128, 384, 64, 6)])
def test_ffn_against_the_bf16_store_diagnostic(T, d, f, E, k):
    """A sharper look at the GEMMs than the 1e-2 bound allows: against the oracle that rounds h and y to bf16
    where the GPU stores them, what is left is float32 accumulation order and the few roundings it flips
    (a flip is one bf16 ulp, 2^-8 relative, on roughly one value in a thousand): a few 1e-4 at most."""
    cfg = small_cfg(T, d, f, E, k, "bf16")
    x = synth.make_activations(cfg, 6)
    logits = synth.make_logits(cfg, 6)
    W = synth.make_all_expert_weights(cfg, 6, workers=4)
    get = lambda e: (W[0][e], W[1][e], W[2][e])
    idx, w, counts, offsets = O.route(logits, k)
    xp, pos, src = O.dispatch(x, idx, offsets)
    y_ref, h_ref = O.expert_ffn(xp, offsets, get, return_h=True, store_bf16=True)
    path = run_layer(cfg, x, logits, W)
    A = T * k
    eh, ey = rel_fro(host(path.h)[:A], h_ref), rel_fro(host(path.y)[:A], y_ref)
    print(f"{cfg.name}: against the bf16-store diagnostic: h {eh:.2e}  y {ey:.2e}")
    assert eh <= 3e-4 and ey <= 3e-4
    path.close()


@pytest.mark.parametrize("T,d,f,E,k,dtype", [(1, 128, 128, 1, 1, "bf16"), (1, 128, 128, 2, 2, "f32"), (2, 128, 256, 256, 64, "bf16"),
                                             (700, 128, 128, 1, 1, "bf16"), (257, 128, 128, 2, 2, "bf16")])
def test_smallest_shapes_and_single_tokens(T, d, f, E, k, dtype):
    """The smallest legal hidden sizes (two K chunks), one expert, one token, and 256 experts with 64 picks."""
    cfg = small_cfg(T, d, f, E, k, dtype)
    x = synth.make_activations(cfg, 8)
    logits = synth.make_logits(cfg, 8)
    W = synth.make_all_expert_weights(cfg, 8, workers=4)
    ref = O.moe_layer(x, logits, k, lambda e: (W[0][e], W[1][e], W[2][e]))
    path = run_layer(cfg, x, logits, W)
    check_integers(path, ref, T, k)
    err = rel_fro(host(path.out)[:T], ref["out"])
    print(f"{cfg.name}: rel-Frobenius out {err:.2e}")
    assert err <= TOL[dtype]
    path.close()


def _random_cases(n, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for _ in range(n):
        E = int(rng.choice([1, 2, 3, 5, 8, 12, 16, 24, 40, 64, 100]))
        k = int(rng.integers(1, min(E, 8) + 1))
        d = 128 * int(rng.integers(1, 4))
        f = 128 * int(rng.integers(1, 5))
        T = int(rng.choice([1, 7, 33, 64, 129, 300, 640, 1500]))
        skew = float(rng.choice([0.0, 1.0, 3.0]))
        cases.append((T, d, f, E, k, "bf16" if rng.random() < 0.8 else "f32", skew))
    return cases


@pytest.mark.parametrize("T,d,f,E,k,dtype,skew", _random_cases(24, 2024))
def test_seeded_random_layers(T, d, f, E, k, dtype, skew):
    """A seeded sweep over shapes nobody picked by hand: odd expert counts, every k, skewed loads (so tiles of
    every height and both GEMM kernels occur), each checked like the hand-picked cases."""
    cfg = small_cfg(T, d, f, E, k, dtype)
    x = synth.make_activations(cfg, 31)
    logits = synth.make_logits(cfg, 31)
    if skew:
        logits = (logits - skew * np.log(np.arange(1, E + 1, dtype=np.float32))).astype(np.float32)
    W = synth.make_all_expert_weights(cfg, 31, workers=4)
    ref = O.moe_layer(x, logits, k, lambda e: (W[0][e], W[1][e], W[2][e]))
    path = run_layer(cfg, x, logits, W)
    check_integers(path, ref, T, k)
    err = rel_fro(host(path.out)[:T], ref["out"])
    assert err <= TOL[dtype], (cfg.name, err)
    path.close()


def _random_large_batch_cases(n, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for _ in range(n):
        E = int(rng.choice([1, 2, 3, 4, 6, 8, 16]))
        k = int(rng.integers(1, min(E, 4) + 1))
        cases.append((int(rng.choice([900, 1500, 2222, 3000, 4097])), 128 * int(rng.integers(2, 7)),
                      128 * int(rng.integers(2, 9)), E, k, float(rng.choice([0.0, 0.5, 1.0, 2.0]))))
    return cases


@pytest.mark.parametrize("T,d,f,E,k,skew", _random_large_batch_cases(16, 77))
def test_seeded_random_large_batch_layers(T, d, f, E, k, skew):
    """The same sweep at hundreds to thousands of rows per expert: every tile height of the large-batch kernel,
    experts split over several tiles, both orders of the tile queue, K from 256 to 1024."""
    cfg = small_cfg(T, d, f, E, k, "bf16")
    x = synth.make_activations(cfg, 32)
    logits = synth.make_logits(cfg, 32)
    if skew:
        logits = (logits - skew * np.log(np.arange(1, E + 1, dtype=np.float32))).astype(np.float32)
    W = synth.make_all_expert_weights(cfg, 32, workers=4)
    ref = O.moe_layer(x, logits, k, lambda e: (W[0][e], W[1][e], W[2][e]))
    path = run_layer(cfg, x, logits, W)
    check_integers(path, ref, T, k)
    err = rel_fro(host(path.out)[:T], ref["out"])
    assert err <= TOL["bf16"], (cfg.name, err)
    path.close()


def test_millions_of_assignments():
    """Near the largest batch a context accepts (T*k <= 2^22): 2.24 M assignments. The ranking kernel gives each
    workgroup several 256-assignment chunks, the float32 GEMM's grid has more than 65 535 m-tiles, counting is
    one workgroup; every integer is still exact and the layer output still matches the oracle."""
    T, d, f, E, k = 280_000, 128, 128, 16, 8
    cfg = small_cfg(T, d, f, E, k, "f32")
    x = synth.make_activations(cfg, 12)
    logits = synth.make_logits(cfg, 12)
    W = synth.make_all_expert_weights(cfg, 12, workers=4)
    ref = O.moe_layer(x, logits, k, lambda e: (W[0][e], W[1][e], W[2][e]))
    path = run_layer(cfg, x, logits, W)
    check_integers(path, ref, T, k)
    err = rel_fro(host(path.out)[:T], ref["out"])
    print(f"{cfg.name}: rel-Frobenius out {err:.2e}")
    assert err <= TOL["f32"]
    path.close()
    with pytest.raises(B.MoeError):
        B.moe_create((1 << 22) // k + 1, d, f, E, k, "f32")          # one token more than the limit


@pytest.mark.parametrize("T,d,E,k,dtype", [(64, 256, 8, 2, "f32"), (256, 6144, 8, 2, "bf16"), (257, 384, 16, 4, "bf16"),
                                           (341, 512, 64, 6, "bf16"), (512, 128, 8, 4, "bf16"), (1000, 512, 64, 6, "bf16"),
                                           (33, 256, 256, 8, "f32"), (1, 128, 5, 3, "bf16"), (2731, 256, 64, 6, "bf16")])
def test_gate_route_dispatch_one_call(T, d, E, k, dtype):
    """moe_gate_route_dispatch: from the token embeddings to the packed rows in one call (two launches at decode
    sizes). The gate scores against the oracle's float64 product; everything after them bit-exact against the
    oracle run on the very logits the GPU produced (two float32 sums in different order may flip a near-tie, so
    exact routing is only defined on identical logits); and identical to moe_gate_route + moe_dispatch."""
    cfg = small_cfg(T, d, 128, E, k, dtype)
    x = synth.make_activations(cfg, 4)
    w_r = synth.make_router_weight(cfg, 4)
    a = B.MoEPath(T, d, 128, E, k, dtype)
    b = B.MoEPath(T, d, 128, E, k, dtype)
    xd, wd = dev(x), dev(w_r)
    for p in (a, b):
        for t in (p.topk_idx, p.pos, p.src, p.counts, p.offsets):
            t.fill_(-7)
        p.xp.zero_()
    logits = torch.full((T, E), 7.0, dtype=torch.float32, device="cuda")
    a.gate_route_dispatch(xd, wd, logits)
    b.gate_route(xd, wd, None)
    b.dispatch(xd)
    torch.cuda.synchronize()
    g_logits = host(logits)
    ref_logits = O.gate_logits(x, w_r)
    assert float(np.linalg.norm(g_logits - ref_logits.astype(np.float64)) / np.linalg.norm(ref_logits)) <= 1e-5
    idx, w, counts, offsets = O.route(g_logits, k)
    xp, pos, src = O.dispatch(x, idx, offsets)
    check_integers(a, dict(topk_idx=idx, topk_w=w, counts=counts, offsets=offsets, xp=xp, pos=pos, src=src), T, k)
    for name in ("topk_idx", "topk_w", "counts", "offsets", "xp", "pos", "src"):
        assert torch.equal(getattr(a, name), getattr(b, name)), name
    a.gate_route_dispatch(xd, wd, None)                    # without the logits output: same picks, same rows
    torch.cuda.synchronize()
    assert torch.equal(a.topk_idx, b.topk_idx) and torch.equal(a.src, b.src) and torch.equal(a.xp, b.xp)
    a.close()
    b.close()
