"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times.

Integer outputs (routing, counts, permutation, copied rows) are checked in full, bit for bit. The
layer output is checked against the oracle on all tokens when the oracle can afford it (T <= 256,
and the Mixtral shape at T = 1024) and on a stratified sample of tokens beyond that: each token's
output depends only on its own row and its own k experts, so the oracle computes sampled outputs
one by one. The sample takes one row out of EVERY 32-row group of every expert's segment (first
row, last row or a random row of the group, in turn), so whatever way a kernel cuts a segment into
m-tiles, every tile and every 32-row group of it, the first and the last included, is compared.
For one whole expert segment per workload the intermediate h and the FFN output y are compared
with the oracle too."""
import numpy as np
import pytest
import torch

from oracle import moe_oracle as O
from oracle import plan_oracle as P
from paper_2504_02263_amd import binding as B
from workloads import synth

from test_gpu_parity import dev, host, rel_fro, w_tol

pytestmark = pytest.mark.gpu


def stratified_tokens(offsets, src, k, seed, at_least=64):
    """Tokens owning one row of every 32-row group of every expert segment, topped up with random tokens
    to `at_least` (or all tokens, if the batch has fewer)."""
    rng = np.random.default_rng(seed)
    T = len(src) // k
    tokens = set()
    for e in range(len(offsets) - 1):
        lo, hi = int(offsets[e]), int(offsets[e + 1])
        for n, g0 in enumerate(range(lo, hi, 32)):
            g1 = min(g0 + 32, hi)
            r = g0 if n % 3 == 0 else g1 - 1 if n % 3 == 1 else int(rng.integers(g0, g1))
            tokens.add(int(src[r]) // k)
    rest = [t for t in rng.permutation(T).tolist() if t not in tokens]
    tokens.update(rest[:max(0, min(at_least, T) - len(tokens))])
    return sorted(tokens)


def compare_outputs(name, got_out, x, idx, w, tokens, weights, counts):
    ref = O.token_outputs(x, idx, w, tokens, weights)
    got = got_out[tokens]
    err = rel_fro(got, ref)
    # per-token worst case too: no single sampled token may be far off
    worst = max(rel_fro(got[i:i + 1], ref[i:i + 1]) for i in range(len(tokens)))
    print(f"{name}: counts min/mean/max {counts.min()}/{counts.mean():.0f}/{counts.max()}  "
          f"rel-Frobenius out {err:.2e} over {len(tokens)} tokens (worst token {worst:.2e})")
    assert err <= 1e-2 and worst <= 2e-2


class Layer:
    """One weight set on the GPU (packed once) plus the host copy the oracle reads."""

    def __init__(self, cfg, T_max, seed=0, paths=1, load_skew=0.0):
        self.cfg, self.seed = cfg, seed
        self.W = synth.make_all_expert_weights(cfg, seed, workers=16)
        self.paths = [B.MoEPath(T_max, cfg.d, cfg.f, cfg.E, cfg.k, cfg.dtype, load_skew=load_skew) for _ in range(paths)]
        self.path = self.paths[0]
        wg, wu, wd = (dev(w) for w in self.W)
        self.path.pack_weights(wg, wu, wd)
        for p in self.paths[1:]:
            p.packed = self.path.packed                 # one packed weight set serves every stream
        torch.cuda.synchronize()
        del wg, wu, wd
        torch.cuda.empty_cache()

    def weights(self, e):
        return self.W[0][e], self.W[1][e], self.W[2][e]

    def check(self, cfg, sample="stratified", x=None, logits=None, segment=True):
        """Run the path on cfg's inputs; compare integers in full, `out` on all tokens (sample=None) or on the
        stratified sample, and h and y on one whole expert segment (the expert with the median row count)."""
        T, k = cfg.T, cfg.k
        x = synth.make_activations(cfg, self.seed) if x is None else x
        logits = synth.make_logits(cfg, self.seed) if logits is None else logits
        idx, w, counts, offsets = O.route(logits, k)
        xp, pos, src = O.dispatch(x, idx, offsets)
        p = self.path
        p.out.zero_()
        p.forward(dev(x), dev(logits))
        torch.cuda.synchronize()
        A = T * k
        assert (host(p.topk_idx)[:T] == idx).all()
        assert (host(p.counts) == counts).all() and (host(p.offsets) == offsets).all()
        assert (host(p.pos)[:T] == pos).all() and (host(p.src)[:A] == src).all()
        assert (host(p.xp)[:A] == xp).all()
        np.testing.assert_allclose(host(p.topk_w)[:T], w, rtol=0, atol=w_tol(k))
        tokens = list(range(T)) if sample is None else stratified_tokens(offsets, src, k, 1234 + T)
        assert len(tokens) >= min(T, 64)
        compare_outputs(cfg.name, host(p.out), x, idx, w, tokens, self.weights, counts)
        assert np.isfinite(O.widen(host(p.out)[:T])).all()
        if segment:
            e = int(np.argsort(counts, kind="stable")[len(counts) // 2])
            lo, hi = int(offsets[e]), int(offsets[e + 1])
            if hi > lo:
                y_ref, h_ref = O.expert_ffn(xp[lo:hi], np.array([0, hi - lo]), lambda _: self.weights(e), return_h=True)
                eh, ey = rel_fro(host(p.h[lo:hi]), h_ref), rel_fro(host(p.y[lo:hi]), y_ref)
                print(f"{cfg.name}: expert {e} ({hi - lo} rows) rel-Frobenius h {eh:.2e}  y {ey:.2e}")
                assert eh <= 1e-2 and ey <= 1e-2
        return counts

    def close(self):
        for p in self.paths:
            p.packed = None
            p.close()
        del self.W


@pytest.fixture(scope="module")
def mixtral():
    layer = Layer(synth.CONFIGS["mixtral_T256"], T_max=4096)
    yield layer
    layer.close()


def test_mixtral_T256_all_tokens(mixtral):
    """The configuration the headline number is quoted on: every output token against the oracle."""
    mixtral.check(synth.CONFIGS["mixtral_T256"], sample=None)


@pytest.mark.parametrize("T", [32, 64, 128])
def test_mixtral_sweep_small_all_tokens(mixtral, T):
    mixtral.check(synth.mixtral_sweep_config(T), sample=None)


def test_mixtral_T1024_all_tokens(mixtral):
    """The ridge of the roofline (256 rows per expert), every token."""
    mixtral.check(synth.mixtral_sweep_config(1024), sample=None)


@pytest.mark.parametrize("T", [512, 2048, 4096])
def test_mixtral_sweep_stratified(mixtral, T):
    mixtral.check(synth.mixtral_sweep_config(T))


def test_dbrx_zipf_stratified():
    cfg = synth.CONFIGS["dbrx_zipf_T1024"]
    layer = Layer(cfg, T_max=cfg.T)
    counts = layer.check(cfg)
    assert counts.max() >= 2 * counts.mean()            # the Zipf bias really skews the load
    # The same layer run node by node under the expert plan bench.py times (8 nodes, 3 slots each):
    # the hot experts get copies, and no bit of any row changes (check() above tied those rows to the oracle).
    p, A = layer.path, cfg.T * cfg.k
    y_plain, h_plain = p.y[:A].clone(), p.h[:A].clone()
    a = [float(c) for c in counts]
    ref = P.plan_experts(a, float(counts.mean()) / 4, 8, 3)
    replicas, slots, _ = B.moe_plan_experts(a, float(counts.mean()) / 4, 8, 3)
    assert replicas == ref["replicas"] and slots == ref["slots"] and max(replicas) > 1
    p.y.zero_()
    p.h.zero_()
    for node in slots:
        share = p.node_share(node, replicas)
        p.expert_ffn_node(cfg.T, share, rows_hint=A // 8)
        b, e, _ = P.slot_segments(host(p.offsets), replicas, node)
        assert host(share.seg_begin)[:len(node)].tolist() == b and host(share.seg_end)[:len(node)].tolist() == e
    torch.cuda.synchronize()
    assert torch.equal(p.y[:A], y_plain) and torch.equal(p.h[:A], h_plain)
    layer.close()


@pytest.mark.parametrize("T,hint", [(256, False), (256, True), (512, True)])
def test_dbrx_zipf_mixed_tile_classes(T, hint):
    """Under the Zipf router at these batch sizes some experts hold a handful of rows and others hundreds:
    one launch mixes decode-sized and large segments. Without the load_skew hint the mean (64 rows at
    T = 256) sends the launch to the streaming kernel, whose popular experts become two tiles; with the
    hint bench.py gives (the workload's own skew) the large-batch kernel runs every segment."""
    cfg = synth.CONFIGS["dbrx_zipf_T1024"].with_T(T)
    layer = Layer(cfg, T_max=cfg.T, load_skew=synth.expected_load_skew(cfg) if hint else 0.0)
    counts = layer.check(cfg)
    assert counts.min() < 64 < 128 < counts.max()
    layer.close()


def test_scaled_moe_stratified():
    cfg = synth.CONFIGS["scaled_moe_T2048"]
    layer = Layer(cfg, T_max=cfg.T)
    layer.check(cfg)
    layer.close()


@pytest.mark.parametrize("m", [3, 8])
def test_finegrained_microbatches_on_two_streams(m):
    """The many-expert layer exactly as bench.py times it: m micro-batches (m = 3: 2731/2731/2730 tokens, 256 rows
    per expert; m = 8: 1024 tokens, 96 rows per expert, the decode-sized tile class) issued on two alternating
    streams, each stream with its own buffer set, both sharing one packed weight buffer, no synchronisation
    between micro-batches. Every micro-batch's results are copied out on its own stream before its buffers are
    used again, then compared with the oracle: integers in full, the output on the stratified sample."""
    cfg = synth.CONFIGS["finegrained_T8192"]
    x = synth.make_activations(cfg, 0)
    logits = synth.make_logits(cfg, 0)
    ranges = synth.microbatch_ranges(cfg.T, m)
    if m == 3:
        assert [b - a for a, b in ranges] == [2731, 2731, 2730]
    layer = Layer(cfg, T_max=max(b - a for a, b in ranges), paths=2)
    x_d, l_d = dev(x), dev(logits)
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    names = ("topk_idx", "topk_w", "counts", "offsets", "pos", "src", "xp", "out")
    snaps = []
    for i, (a, b) in enumerate(ranges):                    # streams A, B, A, ... as bench.py's step()
        path, stream = layer.paths[i % 2], streams[i % 2]
        T = b - a
        path.route_dispatch(x_d[a:b], l_d[a:b], T, stream)
        path.ffn_input(T, stream)
        path.ffn_output(T, stream)
        path.combine(T, stream)
        with torch.cuda.stream(stream):
            snaps.append({n: getattr(path, n).clone() for n in names})
    torch.cuda.synchronize()
    k = cfg.k
    for i, (a, b) in enumerate(ranges):
        T, A, s = b - a, (b - a) * k, snaps[i]
        idx, w, counts, offsets = O.route(logits[a:b], k)
        xp, pos, src = O.dispatch(x[a:b], idx, offsets)
        assert (host(s["topk_idx"])[:T] == idx).all()
        assert (host(s["counts"]) == counts).all() and (host(s["offsets"]) == offsets).all()
        assert (host(s["pos"])[:T] == pos).all() and (host(s["src"])[:A] == src).all()
        assert (host(s["xp"])[:A] == xp).all()
        np.testing.assert_allclose(host(s["topk_w"])[:T], w, rtol=0, atol=w_tol(k))
        tokens = stratified_tokens(offsets, src, k, 99 + i)
        if m > 3 and i not in (0, 1, m - 1):
            tokens = tokens[::8]                           # the oracle's time is spent on the first and last micro-batches
        compare_outputs(f"{cfg.name} m={m} micro-batch {i}", host(s["out"]), x[a:b], idx, w, tokens, layer.weights, counts)
    layer.close()
