"""The C-ABI library builds/loads, exports every symbol the header declares, and rejects bad
arguments on the host before anything is launched (no GPU needed for any of this)."""
import ctypes
import os
import re

import pytest

from paper_2504_02263_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "moe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(moe_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = B.load_library()
    names = _declared()
    assert set(names) == set(B.EXPORTS)
    for name in names:
        assert getattr(lib, name) is not None


def test_status_strings():
    lib = B.load_library()
    assert lib.moe_status_string(0) == b"MOE_OK"
    assert lib.moe_status_string(1) == b"MOE_ERR_INVALID_ARG"
    assert lib.moe_status_string(2) == b"MOE_ERR_UNSUPPORTED"
    assert lib.moe_status_string(3) == b"MOE_ERR_HIP"


def test_create_validates_config():
    ok = B.moe_create(64, 256, 512, 8, 2, "f32")
    assert ok
    B.moe_destroy(ok)
    for bad, status in [((64, 256, 512, 8, 9, "f32"), B.MOE_ERR_INVALID_ARG),      # k > E
                        ((64, 256, 512, 0, 1, "f32"), B.MOE_ERR_INVALID_ARG),
                        ((-1, 256, 512, 8, 2, "f32"), B.MOE_ERR_INVALID_ARG),
                        ((64, 250, 512, 8, 2, "bf16"), B.MOE_ERR_UNSUPPORTED),     # d not a multiple of 128
                        ((64, 256, 512, 512, 2, "bf16"), B.MOE_ERR_UNSUPPORTED),   # E > 256
                        ((64, 256, 512, 128, 65, "bf16"), B.MOE_ERR_UNSUPPORTED)]:  # k > 64
        with pytest.raises(B.MoeError) as ei:
            B.moe_create(*bad)
        assert ei.value.status == status, bad
    for skew in (0.5, -1.0, float("nan"), float("inf")):          # the load hint is 0 (unknown) or >= 1
        with pytest.raises(B.MoeError) as ei:
            B.moe_create(64, 256, 512, 8, 2, "bf16", load_skew=skew)
        assert ei.value.status == B.MOE_ERR_INVALID_ARG, skew
    B.moe_destroy(B.moe_create(64, 256, 512, 8, 2, "bf16", load_skew=3.5))
    lib = B.load_library()
    assert lib.moe_create(None, None) == B.MOE_ERR_INVALID_ARG


def test_packed_weight_bytes():
    assert B.moe_packed_weight_bytes(64, 256, 512, 8, 2, "f32") == 3 * 8 * 256 * 512 * 4
    assert B.moe_packed_weight_bytes(256, 6144, 16384, 8, 2, "bf16") == 3 * 8 * 6144 * 16384 * 2
    assert B.moe_packed_weight_bytes(64, 250, 512, 8, 2, "f32") == 0


def test_hot_calls_reject_bad_arguments_before_launch():
    lib = B.load_library()
    ctx = B.moe_create(64, 256, 512, 8, 2, "bf16")
    good = 0x1000   # any 16-byte-aligned non-null address: the checks fail before it is used
    try:
        # null pointer
        assert lib.moe_route(ctx, 4, None, good, good, good, good, None) == B.MOE_ERR_INVALID_ARG
        assert b"null" in lib.moe_last_error(ctx)
        # T out of range
        assert lib.moe_route(ctx, 65, good, good, good, good, good, None) == B.MOE_ERR_INVALID_ARG
        assert b"T_max" in lib.moe_last_error(ctx)
        assert lib.moe_dispatch(ctx, -1, good, good, good, good, good, good, None) == B.MOE_ERR_INVALID_ARG
        # misaligned pointer
        assert lib.moe_combine(ctx, 4, good + 4, good, good, good, None) == B.MOE_ERR_INVALID_ARG
        assert b"aligned" in lib.moe_last_error(ctx)
        assert lib.moe_expert_ffn(ctx, 4, good, good, None, good, good, None) == B.MOE_ERR_INVALID_ARG
        assert lib.moe_pack_weights(ctx, good, good, good, None, None) == B.MOE_ERR_INVALID_ARG
        # segment calls: slot / segment count outside [0, 256], null list, T out of range
        assert lib.moe_slot_segments(ctx, 257, good, good, good, good, good, good, None) == B.MOE_ERR_INVALID_ARG
        assert b"n_slots" in lib.moe_last_error(ctx)
        assert lib.moe_slot_segments(ctx, 4, good, None, good, good, good, good, None) == B.MOE_ERR_INVALID_ARG
        assert lib.moe_expert_ffn_segments(ctx, 4, -1, 0, good, good, good, good, good, good, good, None) == B.MOE_ERR_INVALID_ARG
        assert b"n_segs" in lib.moe_last_error(ctx)
        assert lib.moe_expert_ffn_segments(ctx, 65, 2, 0, good, good, good, good, good, good, good, None) == B.MOE_ERR_INVALID_ARG
        assert lib.moe_expert_ffn_segments(ctx, 4, 2, 0, good, good, good, None, good, good, good, None) == B.MOE_ERR_INVALID_ARG
        assert lib.moe_route_dispatch(ctx, 4, good, None, good, good, good, good, good, good, good, None) == B.MOE_ERR_INVALID_ARG
        assert lib.moe_route_dispatch(ctx, 65, good, good, good, good, good, good, good, good, good, None) == B.MOE_ERR_INVALID_ARG
        assert lib.moe_gate_route_dispatch(ctx, 4, good, None, None, good, good, good, good, good, good, good, None) == B.MOE_ERR_INVALID_ARG
        assert lib.moe_gate_route_dispatch(ctx, 4, good, good, good + 8, good, good, good, good, good, good, good, None) == B.MOE_ERR_INVALID_ARG
        # null context
        assert lib.moe_route(None, 4, good, good, good, good, good, None) == B.MOE_ERR_INVALID_ARG
    finally:
        B.moe_destroy(ctx)


def test_binding_has_no_cpu_fallback():
    import torch
    if torch.cuda.is_available():
        pytest.skip("GPU present")
    with pytest.raises(RuntimeError):
        B.MoEPath(64, 256, 512, 8, 2, "f32")


def test_product_never_mentions_the_oracle():
    pkg = os.path.join(ROOT, "paper_2504_02263_amd")
    for dirpath, _, files in os.walk(pkg):
        for name in files:
            if name.endswith((".py", ".hip", ".h", ".cpp")):
                assert "oracle" not in open(os.path.join(dirpath, name)).read().lower(), name
