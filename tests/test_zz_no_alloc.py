"""moe_expert_ffn_static (the entry point that allocates nothing: its intermediate h lives in a static
array inside the library's device image) against moe_expert_ffn on the same inputs, through the C ABI.
Two calls in a row, the second with a smaller batch, so that what the first call left in the shared
array cannot leak into the second; then the size limit. Collected last on purpose (file name)."""
import numpy as np
import pytest
import torch

from paper_2504_02263_amd import binding as B
from workloads import synth

pytestmark = pytest.mark.gpu


def dev(a):
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


@pytest.mark.parametrize("dtype,d,f,E,k,Ts", [("bf16", 256, 512, 8, 2, (700, 130)), ("f32", 128, 256, 4, 2, (90, 33)),
                                              ("bf16", 384, 640, 16, 4, (1500, 1))])
def test_static_workspace_entry_point_matches_moe_expert_ffn(dtype, d, f, E, k, Ts):
    T_max = max(Ts)
    cfg = synth.LayerConfig(f"noalloc_{dtype}", T=T_max, d=d, f=f, E=E, k=k, dtype=dtype, router="logits")
    W = synth.make_all_expert_weights(cfg, 5, workers=4)
    path = B.MoEPath(T_max, d, f, E, k, dtype)
    path.pack_weights(dev(W[0]), dev(W[1]), dev(W[2]))
    for call, T in enumerate(Ts):
        c = cfg.with_T(T)
        x, logits = dev(synth.make_activations(c, 40 + call)), dev(synth.make_logits(c, 40 + call))
        path.route_dispatch(x, logits, T)
        A = T * k
        path.y.fill_(3.0)
        path.expert_ffn(T)                                   # the existing entry point, caller's workspace
        torch.cuda.synchronize()
        want = path.y.clone()
        path.y.fill_(3.0)
        before = torch.cuda.memory_allocated()
        B.moe_expert_ffn_static(path.ctx, T, path.xp, path.offsets, path.packed, path.y)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        assert torch.equal(path.y, want), f"call {call} (T = {T}): y differs from moe_expert_ffn"
        assert bool(torch.isfinite(path.y[:A].float()).all())
    path.close()


def test_static_workspace_entry_point_rejects_what_does_not_fit():
    d, f, E, k = 128, 16384, 8, 2
    T = (64 << 20) // (k * f * 2) + 1                        # one token more than the 64 MiB array holds
    ctx = B.moe_create(T, d, f, E, k, "bf16")
    buf = torch.zeros(64, dtype=torch.int32, device="cuda")
    with pytest.raises(B.MoeError) as err:
        B.moe_expert_ffn_static(ctx, T, buf, buf, buf, buf)
    assert err.value.status == B.MOE_ERR_UNSUPPORTED and "static workspace" in str(err.value)
    B.moe_expert_ffn_static(ctx, 0, buf, buf, buf, buf)      # an empty batch is a no-op
    torch.cuda.synchronize()
    B.moe_destroy(ctx)
