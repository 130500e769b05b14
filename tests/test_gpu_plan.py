"""GPU parity for running an expert plan (hot-expert redundancy, paper Section 6 "Load balance"):
row ranges of expert copies, and the expert FFN over one node's segments, against the oracle; and
the property that cutting an expert's rows into copies changes no bit of any row's result."""
import numpy as np
import pytest
import torch

from oracle import moe_oracle as O
from oracle import plan_oracle as P
from paper_2504_02263_amd import binding as B
from workloads import synth

from test_gpu_parity import dev, host, rel_fro, small_cfg, TOL

pytestmark = pytest.mark.gpu


def _zipf_logits(cfg, seed):
    rng = np.random.default_rng(seed)
    bias = -1.5 * np.log(rng.permutation(cfg.E) + 1.0)
    return (synth.make_logits(cfg, seed) + bias).astype(np.float32)


@pytest.mark.parametrize("T,d,f,E,k,dtype,N,S", [
    (600, 256, 384, 8, 2, "bf16", 4, 3),      # hot expert several hundred rows: copies land in both FFN kernels
    (2000, 128, 256, 6, 2, "bf16", 3, 4),     # large-batch kernel with multi-tile copies
    (90, 256, 128, 16, 4, "bf16", 8, 3),      # small segments, some empty
    (150, 128, 256, 5, 2, "f32", 5, 2),       # fp32 path
])
def test_plan_nodes_match_oracle_and_the_plain_layer(T, d, f, E, k, dtype, N, S):
    cfg = small_cfg(T, d, f, E, k, dtype)
    x = synth.make_activations(cfg, 3)
    logits = _zipf_logits(cfg, 3)
    W = synth.make_all_expert_weights(cfg, 3, workers=4)
    get = lambda e: (W[0][e], W[1][e], W[2][e])
    ref = O.moe_layer(x, logits, k, get)
    counts, offsets = ref["counts"], ref["offsets"]
    plan = P.plan_experts([float(c) for c in counts], float(T * k / E / 4), N, S)
    replicas, slots, _ = B.moe_plan_experts([float(c) for c in counts], float(T * k / E / 4), N, S)
    assert replicas == plan["replicas"] and slots == plan["slots"]
    assert max(replicas) > 1, "the case is meant to need copies"

    path = B.MoEPath(T, d, f, E, k, dtype)
    path.pack_weights(dev(W[0]), dev(W[1]), dev(W[2]))
    A = T * k
    path.route(dev(logits))
    path.dispatch(dev(x))
    path.expert_ffn(T)
    torch.cuda.synchronize()
    y_plain, h_plain = path.y[:A].clone(), path.h[:A].clone()

    sentinel = 3.0
    path.y.fill_(sentinel)
    path.h.fill_(sentinel)
    y_or = None
    done = np.zeros(A, dtype=bool)
    for node in slots:
        share = path.node_share(node, replicas)
        path.expert_ffn_node(T, share, rows_hint=A // N)
        torch.cuda.synchronize()
        b, e, ex = P.slot_segments(offsets, replicas, node)
        assert host(share.seg_begin)[:len(node)].tolist() == b          # integer work: exact
        assert host(share.seg_end)[:len(node)].tolist() == e
        for lo, hi in zip(b, e):
            done[lo:hi] = True
        # rows of nodes not run yet are untouched
        untouched = torch.from_numpy(~done).cuda()
        assert (path.y[:A][untouched] == sentinel).all() and (path.h[:A][untouched] == sentinel).all()
        y_or = O.expert_ffn_segments(ref["xp"], b, e, ex, get, y=y_or)
    assert done.all()
    assert torch.equal(path.y[:A], y_plain) and torch.equal(path.h[:A], h_plain)   # bit for bit
    err = rel_fro(host(path.y)[:A], y_or)
    path.combine(T)
    torch.cuda.synchronize()
    eo = rel_fro(host(path.out)[:T], ref["out"])
    print(f"{cfg.name} N={N} S={S} replicas={replicas}: rel-Frobenius y {err:.2e} out {eo:.2e}")
    assert err <= TOL[dtype] and eo <= TOL[dtype]
    path.close()


def test_segment_edge_cases():
    """Empty list, empty and clipped ranges, a segment naming no expert, several segments of one expert."""
    d, f, E, k, A = 256, 384, 4, 1, 300
    cfg = small_cfg(A, d, f, E, k, "bf16")
    xp = synth.make_activations(cfg, 9)
    W = synth.make_all_expert_weights(cfg, 9, workers=4)
    get = lambda e: (W[0][e], W[1][e], W[2][e])
    path = B.MoEPath(A + 50, d, f, E, k, "bf16")
    path.pack_weights(dev(W[0]), dev(W[1]), dev(W[2]))
    path.xp[:A].copy_(dev(xp))
    i32 = torch.int32
    seg = lambda v: torch.tensor(v, dtype=i32, device="cuda")
    # expert 2 three times, expert 0 once, one segment with expert 9 (skipped), one empty, one reaching past A (clipped)
    begin, end, expert = [0, 40, 41, 140, 200, 250, 280], [40, 41, 140, 200, 250, 250, 400], [2, 2, 2, 0, 9, 1, 3]
    path.y.fill_(5.0)
    B.moe_expert_ffn_segments(path.ctx, A, len(begin), 0, path.xp, seg(begin), seg(end), seg(expert), path.packed,
                              path.h, path.y)
    torch.cuda.synchronize()
    ref = O.expert_ffn_segments(xp, [0, 40, 41, 140, 280], [40, 41, 140, 200, A], [2, 2, 2, 0, 3], get)
    rows = np.r_[0:200, 280:A]
    assert rel_fro(host(path.y)[rows], ref[rows]) <= 1e-2
    assert (path.y[200:280] == 5.0).all() and (path.y[A:] == 5.0).all()     # skipped, empty and clipped rows untouched
    # no segments at all: nothing runs, nothing changes
    path.y.fill_(6.0)
    B.moe_expert_ffn_segments(path.ctx, A, 0, 0, path.xp, seg([0]), seg([0]), seg([0]), path.packed, path.h, path.y)
    torch.cuda.synchronize()
    assert (path.y == 6.0).all()
    # slot ranges: a slot naming no expert and a copy number out of range give [0, 0)
    offsets = seg([0, 100, 100, 250, 300])
    sb, se = seg([7] * 5), seg([7] * 5)
    B.moe_slot_segments(path.ctx, 5, seg([2, 2, 7, 0, 1]), seg([0, 1, 0, 3, 0]), seg([1, 1, 2, 1]), offsets, sb, se)
    torch.cuda.synchronize()
    assert host(sb).tolist() == [100, 175, 0, 0, 100] and host(se).tolist() == [175, 250, 0, 0, 100]
    path.close()
