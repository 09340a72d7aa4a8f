"""Host-only checks of the C ABI: the library loads, exports every declared symbol and rejects bad arguments
before touching a device."""
import ctypes as C
import os
import re

import pytest

from paper_2605_05607_amd import binding as B
from paper_2605_05607_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "moe355.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"MOE355_API\s+[\w\s\*]+?\b(moe_\w+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_symbols()
    assert {"moe_route_topk", "moe_build_dispatch", "moe_fused_forward", "moe_pack_weights"} <= set(names)
    assert len(names) >= 12
    lib = B.lib()
    for n in names:
        assert hasattr(lib, n), n


def test_status_strings():
    assert B.status_string(0) == "ok"
    for code in (-1, -2, -3, -4, -99):
        assert B.status_string(code)


def good_shape(**kw):
    base = dict(T=64, d=64, f=128, E=8, k=2, R=4, local_rank_begin=0, local_rank_end=4, dtype=B.MOE_BF16)
    base.update(kw)
    return B.make_shape(**base)


@pytest.mark.parametrize("kw", [dict(E=10, R=4), dict(k=9), dict(k=0), dict(k=33, E=64), dict(T=-1), dict(d=60),
                                dict(f=100), dict(local_rank_begin=2, local_rank_end=2), dict(local_rank_end=5),
                                dict(local_rank_begin=-1), dict(R=0)])
def test_invalid_shapes_are_rejected_everywhere(kw):
    s = good_shape(**kw)
    lib = B.lib()
    fake = 4096  # never dereferenced: validation fails first
    assert lib.moe_route_topk(C.byref(s), fake, fake, fake, None) == B.MOE_ERR_INVALID_ARG
    assert B.moe_dispatch_workspace_bytes(s) == 0 and B.moe_forward_workspace_bytes(s) == 0
    assert B.moe_packed_weight_bytes(s, 0) == 0
    assert lib.moe_pack_weights(C.byref(s), fake, fake, fake, fake, fake, None) == B.MOE_ERR_INVALID_ARG


def test_unsupported_dtype_and_extent():
    lib = B.lib()
    assert lib.moe_route_topk(C.byref(good_shape(dtype=7)), 4096, 4096, 4096, None) == B.MOE_ERR_UNSUPPORTED
    assert lib.moe_route_topk(C.byref(good_shape(E=8192, R=1, local_rank_end=1)), 4096, 4096, 4096, None) \
        == B.MOE_ERR_UNSUPPORTED


def test_forward_rejects_misaligned_rows():
    lib = B.lib()
    s = good_shape()
    tb = B.moe_dispatch(*([4096] * 9))
    need = B.moe_forward_workspace_bytes(s)
    ok = [4096, 4096, 4096, C.byref(tb), 4096, 4096, 4096]     # x, topk_idx, topk_w, tables, gate_up, down, y
    for pos in (0, 4, 5, 6):
        args = list(ok)
        args[pos] = 4096 + 8
        assert lib.moe_fused_forward(C.byref(s), *args, 4096, need, None) == B.MOE_ERR_INVALID_ARG


def test_gemm_launch_rule_follows_rows_per_expert():
    lib = B.lib()
    assert lib.moe_forward_gemm_launches(C.byref(good_shape(T=4096, E=256, k=8, R=8))) == 1   # 128 rows per expert
    assert lib.moe_forward_gemm_launches(C.byref(good_shape(T=8192, E=256, k=8, R=8))) == 2   # 256
    assert lib.moe_forward_gemm_launches(C.byref(good_shape(T=8, E=8, k=2, R=1, local_rank_end=1, dtype=B.MOE_F32))) == 2
    assert lib.moe_forward_gemm_launches(C.byref(good_shape(E=6, R=4))) == 0                 # invalid shape


def test_forward_rejects_extents_beyond_32bit_row_offsets():
    lib = B.lib()
    s = good_shape(T=1 << 20, d=8192, f=8192, k=2)
    tb = B.moe_dispatch(*([4096] * 9))
    need = B.moe_forward_workspace_bytes(s)
    assert need > 0
    assert lib.moe_fused_forward(C.byref(s), 4096, 4096, 4096, C.byref(tb), 4096, 4096, 4096, 4096, need, None) \
        == B.MOE_ERR_UNSUPPORTED


def test_null_pointers_and_small_workspace():
    lib = B.lib()
    s = good_shape()
    fake = 4096
    assert lib.moe_route_topk(None, fake, fake, fake, None) == B.MOE_ERR_INVALID_ARG
    assert lib.moe_route_topk(C.byref(s), None, fake, fake, None) == B.MOE_ERR_INVALID_ARG
    tb = B.moe_dispatch(*([fake] * 9))
    assert lib.moe_build_dispatch(C.byref(s), None, C.byref(tb), fake, 1 << 20, None) == B.MOE_ERR_INVALID_ARG
    assert lib.moe_build_dispatch(C.byref(s), fake, C.byref(tb), fake, 16, None) == B.MOE_ERR_WORKSPACE
    assert lib.moe_build_dispatch(C.byref(s), fake, C.byref(tb), None, 1 << 20, None) == B.MOE_ERR_WORKSPACE
    holes = B.moe_dispatch(*([fake] * 8 + [None]))
    assert lib.moe_build_dispatch(C.byref(s), fake, C.byref(holes), fake, 1 << 20, None) == B.MOE_ERR_INVALID_ARG
    need = B.moe_forward_workspace_bytes(s)
    args = (C.byref(s), fake, fake, fake, C.byref(tb), fake, fake, fake)
    assert lib.moe_fused_forward(*args, 4096, need - 1, None) == B.MOE_ERR_WORKSPACE
    assert lib.moe_fused_forward(*args, 4096 + 8, need, None) == B.MOE_ERR_INVALID_ARG  # misaligned workspace
    assert lib.moe_fused_forward(C.byref(s), None, fake, fake, C.byref(tb), fake, fake, fake, 4096, need, None) \
        == B.MOE_ERR_INVALID_ARG
    assert lib.moe_unfused_forward(*args, 4096, need, None) == B.MOE_ERR_WORKSPACE  # needs the larger workspace
    assert lib.moe_dispatch_gather(C.byref(s), fake, C.byref(tb), None, None) == B.MOE_ERR_INVALID_ARG
    assert lib.moe_combine_reduce(C.byref(s), None, fake, C.byref(tb), fake, None) == B.MOE_ERR_INVALID_ARG


def test_sizes_for_the_named_configs():
    for name, cfg in wl.CONFIGS.items():
        s = B.shape_of(cfg)
        assert B.moe_dispatch_workspace_bytes(s) >= 64 * (cfg.E + cfg.R) * 4
        elt = 2 if cfg.dtype == wl.BF16 else 4
        raw = cfg.E_loc * cfg.d * cfg.f * elt
        assert B.moe_packed_weight_bytes(s, 0) >= 2 * raw and B.moe_packed_weight_bytes(s, 1) >= raw
        assert B.moe_packed_weight_bytes(s, 0) < 2.2 * raw + (1 << 20)
        rows = cfg.T * min(cfg.k, cfg.E_loc)
        assert B.moe_forward_workspace_bytes(s) >= rows * (cfg.f * elt + cfg.d * 4)
        assert B.moe_unfused_workspace_bytes(s) > B.moe_forward_workspace_bytes(s)


def test_t_zero_is_a_noop_on_the_host():
    s = good_shape(T=0)
    lib = B.lib()
    assert lib.moe_route_topk(C.byref(s), 4096, 4096, 4096, None) == B.MOE_OK


def test_router_logits_arguments():
    lib = B.lib()
    s = good_shape()
    need = B.moe_router_workspace_bytes(s)
    assert need >= 256 and need % 256 == 0
    assert B.moe_router_workspace_bytes(good_shape(E=0)) == 0
    fake = 4096
    assert lib.moe_router_logits(C.byref(s), None, fake, fake, fake, need, None) == B.MOE_ERR_INVALID_ARG
    assert lib.moe_router_logits(C.byref(s), fake, fake, None, fake, need, None) == B.MOE_ERR_INVALID_ARG
    assert lib.moe_router_logits(C.byref(s), fake + 2, fake, fake, fake, need, None) == B.MOE_ERR_INVALID_ARG
    assert lib.moe_router_logits(C.byref(s), fake, fake, fake, fake, need - 1, None) == B.MOE_ERR_WORKSPACE
    assert lib.moe_router_logits(C.byref(s), fake, fake, fake, None, need, None) == B.MOE_ERR_WORKSPACE
    assert lib.moe_router_logits(C.byref(good_shape(T=0)), fake, fake, fake, fake, 1 << 20, None) == B.MOE_OK
    # the partial sums of the parts of the reduction range fit: parts <= 8
    for cfg in wl.CONFIGS.values():
        sh = B.shape_of(cfg)
        assert B.moe_router_workspace_bytes(sh) <= 8 * cfg.T * cfg.E * 4 + 512


def test_fp8_entry_points_arguments():
    lib = B.lib()
    s = good_shape()
    fake = 4096
    tb = B.moe_dispatch(*([fake] * 9))
    need = B.moe_fp8_forward_workspace_bytes(s)
    assert need > B.moe_forward_workspace_bytes(s) + s.T * s.d  # room for x as codes and its scales
    for which in (0, 1):
        raw = (s.local_rank_end - s.local_rank_begin) * (s.E // s.R) * s.d * s.f * (2 if which == 0 else 1)
        assert raw <= B.moe_fp8_packed_weight_bytes(s, which) < 2.2 * raw + (1 << 20)  # one byte per weight + padding
    assert B.moe_fp8_packed_weight_bytes(s, 2) == 0
    args = (C.byref(s), fake, fake, fake, C.byref(tb), fake, fake)
    assert lib.moe_fp8_fused_forward(*args, None, fake, fake, need, None, None) == B.MOE_ERR_INVALID_ARG  # no h_scale
    assert lib.moe_fp8_fused_forward(*args, fake, fake, fake, need - 1, None, None) == B.MOE_ERR_WORKSPACE
    assert lib.moe_fp8_fused_forward(*args, fake, None, fake, need, None, None) == B.MOE_ERR_INVALID_ARG
    odd = good_shape(d=72)  # rows are not whole 16-code chunks
    big = 1 << 30
    assert lib.moe_fp8_fused_forward(C.byref(odd), fake, fake, fake, C.byref(tb), fake, fake, fake, fake, fake, big,
                                     None, None) == B.MOE_ERR_UNSUPPORTED
    assert lib.moe_fp8_pack_weights(C.byref(odd), fake, fake, fake, fake, fake, None) == B.MOE_ERR_UNSUPPORTED
    f32 = good_shape(dtype=B.MOE_F32)
    assert lib.moe_fp8_pack_weights(C.byref(f32), fake, fake, fake, fake, fake, None) == B.MOE_ERR_UNSUPPORTED
    assert lib.moe_fp8_pack_weights(C.byref(s), fake, None, fake, fake, fake, None) == B.MOE_ERR_INVALID_ARG
    assert lib.moe_fp8_quantize_rows(4, 12, fake, fake, fake, None) == B.MOE_ERR_INVALID_ARG   # cols % 8
    assert lib.moe_fp8_quantize_rows(4, 16, fake + 4, fake, fake, None) == B.MOE_ERR_INVALID_ARG  # misaligned
    assert lib.moe_fp8_quantize_rows(-1, 16, fake, fake, fake, None) == B.MOE_ERR_INVALID_ARG
    assert lib.moe_fp8_quantize_rows(0, 16, fake, fake, fake, None) == B.MOE_OK
    assert lib.moe_fp8_fused_forward(C.byref(good_shape(T=0)), fake, fake, fake, C.byref(tb), fake, fake, fake, fake,
                                     fake, big, None, None) == B.MOE_OK


def test_route_gate_arguments():
    lib = B.lib()
    s = good_shape()
    fake = 4096
    assert lib.moe_route_topk_gate(C.byref(s), fake, None, 2, fake, fake, None) == B.MOE_ERR_INVALID_ARG  # gate
    assert lib.moe_route_topk_gate(C.byref(s), None, None, 1, fake, fake, None) == B.MOE_ERR_INVALID_ARG
    assert lib.moe_route_topk_gate(C.byref(good_shape(k=9)), fake, None, 1, fake, fake, None) == B.MOE_ERR_INVALID_ARG
    assert lib.moe_route_topk_gate(C.byref(good_shape(T=0)), fake, None, 1, fake, fake, None) == B.MOE_OK


def test_training_entry_points_arguments():
    lib = B.lib()
    s = good_shape()
    fake = 4096
    tb = B.moe_dispatch(*([fake] * 9))
    kept = B.moe_train_kept_bytes(s)
    ws = B.moe_backward_workspace_bytes(s)
    El = (s.local_rank_end - s.local_rank_begin) * (s.E // s.R)
    rows = s.T * min(s.k, El)
    assert kept >= rows * (2 * s.f * 2 + s.d * 4)           # g, u in bf16 and the weighted rows in fp32
    assert ws >= rows * (3 * s.f * 2 + s.d * 4) + (2 * s.d + 3 * s.f) * rows * 2  # intermediates + transposed operands
    assert B.moe_backward_packed_weight_bytes(s, 0) >= El * s.d * s.f * 2
    assert B.moe_backward_packed_weight_bytes(s, 1) >= 2 * El * s.d * s.f * 2
    assert B.moe_backward_packed_weight_bytes(s, 2) == 0
    fwd_ws = B.moe_forward_workspace_bytes(s)
    f_args = (C.byref(s), fake, fake, fake, C.byref(tb), fake, fake, fake)
    assert lib.moe_fused_forward_train(*f_args, fake, kept - 1, fake, fwd_ws, None) == B.MOE_ERR_WORKSPACE
    assert lib.moe_fused_forward_train(*f_args, None, kept, fake, fwd_ws, None) == B.MOE_ERR_WORKSPACE
    assert lib.moe_fused_forward_train(*f_args, fake, kept, fake, fwd_ws - 1, None) == B.MOE_ERR_WORKSPACE
    assert lib.moe_fused_forward_train(C.byref(good_shape(dtype=B.MOE_F32)), fake, fake, fake, C.byref(tb), fake, fake,
                                       fake, fake, 1 << 30, fake, 1 << 30, None) == B.MOE_ERR_UNSUPPORTED
    b_args = (C.byref(s), fake, fake, fake, fake, C.byref(tb), fake, fake, fake, kept, fake, fake)
    assert lib.moe_fused_backward(*b_args, None, None, None, fake, ws - 1, None) == B.MOE_ERR_WORKSPACE
    assert lib.moe_fused_backward(*b_args, fake, None, None, fake, ws, None) == B.MOE_ERR_INVALID_ARG  # all three or none
    assert lib.moe_fused_backward(C.byref(s), fake, None, fake, fake, C.byref(tb), fake, fake, fake, kept, fake, fake,
                                  None, None, None, fake, ws, None) == B.MOE_ERR_INVALID_ARG           # no dy
    # weight gradients leave in 16-byte stores: a pointer that is only 8-byte aligned is rejected
    assert lib.moe_fused_backward(*b_args, fake, fake + 8, fake, fake, ws, None) == B.MOE_ERR_INVALID_ARG
    odd = good_shape(f=72)  # the backward needs whole 64-index reduction tiles over f
    assert lib.moe_fused_backward(C.byref(odd), fake, fake, fake, fake, C.byref(tb), fake, fake, fake, 1 << 30, fake,
                                  fake, None, None, None, fake, 1 << 30, None) == B.MOE_ERR_UNSUPPORTED
    assert lib.moe_pack_weights_backward(C.byref(odd), fake, fake, fake, fake, fake, None) == B.MOE_ERR_UNSUPPORTED
    assert lib.moe_pack_weights_backward(C.byref(s), fake, fake, None, fake, fake, None) == B.MOE_ERR_INVALID_ARG
    # (T = 0 launches a fill for the weight gradients, or nothing without them: exercised on the GPU)


def test_route_backward_arguments():
    lib = B.lib()
    s = good_shape()
    fake = 4096
    assert lib.moe_route_backward(C.byref(s), fake, fake, None, fake, None) == B.MOE_ERR_INVALID_ARG
    assert lib.moe_route_backward(C.byref(s), fake, fake, fake, None, None) == B.MOE_ERR_INVALID_ARG
    assert lib.moe_route_backward(None, fake, fake, fake, fake, None) == B.MOE_ERR_INVALID_ARG
    assert lib.moe_route_backward(C.byref(good_shape(T=0)), fake, fake, fake, fake, None) == B.MOE_OK


def test_mfma_rate_probe_arguments():
    lib = B.lib()
    fl = C.c_double(0.0)
    assert lib.moe_probe_mfma_rate(0, 10, 4096, 1 << 20, C.byref(fl), None) == B.MOE_ERR_INVALID_ARG
    assert lib.moe_probe_mfma_rate(4, 0, 4096, 1 << 20, C.byref(fl), None) == B.MOE_ERR_INVALID_ARG
    assert lib.moe_probe_mfma_rate(4, 10, None, 1 << 20, C.byref(fl), None) == B.MOE_ERR_INVALID_ARG
    assert lib.moe_probe_mfma_rate(4, 10, 4096, 4 * 512 - 1, C.byref(fl), None) == B.MOE_ERR_WORKSPACE


def test_noalloc_dispatch_rejects_bad_arguments_before_any_device_call():
    lib = B.lib()
    s = good_shape()
    tb = B.moe_dispatch(*([4096] * 9))
    assert lib.moe_build_dispatch_noalloc(None, 4096, C.byref(tb), None) == B.MOE_ERR_INVALID_ARG
    assert lib.moe_build_dispatch_noalloc(C.byref(s), None, C.byref(tb), None) == B.MOE_ERR_INVALID_ARG
    assert lib.moe_build_dispatch_noalloc(C.byref(s), 4096, None, None) == B.MOE_ERR_INVALID_ARG
    holes = B.moe_dispatch(*([4096] * 8 + [None]))
    assert lib.moe_build_dispatch_noalloc(C.byref(s), 4096, C.byref(holes), None) == B.MOE_ERR_INVALID_ARG
    assert lib.moe_build_dispatch_noalloc(C.byref(good_shape(E=10, R=4)), 4096, C.byref(tb), None) \
        == B.MOE_ERR_INVALID_ARG
    # beyond the static scratch (E + R counters per chunk): a clear error, nothing launched
    big = good_shape(E=1024, R=1, k=2, local_rank_begin=0, local_rank_end=1)
    assert lib.moe_build_dispatch_noalloc(C.byref(big), 4096, C.byref(tb), None) == B.MOE_ERR_UNSUPPORTED
    big = good_shape(E=2048, R=2, k=2, local_rank_begin=0, local_rank_end=1)
    assert lib.moe_build_dispatch_noalloc(C.byref(big), 4096, C.byref(tb), None) == B.MOE_ERR_UNSUPPORTED


def test_one_workspace_query_covers_both_calls():
    for kw in (dict(), dict(T=4096, d=7168, f=2048, E=256, k=8, R=8, local_rank_begin=4, local_rank_end=5),
               dict(T=0), dict(dtype=B.MOE_F32)):
        s = good_shape(**kw)
        assert B.moe_workspace_bytes(s) == max(B.moe_dispatch_workspace_bytes(s), B.moe_forward_workspace_bytes(s))
        assert B.moe_workspace_bytes(s) > 0
    assert B.moe_workspace_bytes(good_shape(k=0)) == 0


def test_forward_status_and_bounded_forward_reject_bad_arguments():
    lib = B.lib()
    flag = C.c_int32(7)
    assert lib.moe_forward_status(None, C.byref(flag), None) == B.MOE_ERR_INVALID_ARG
    assert lib.moe_forward_status(4096, None, None) == B.MOE_ERR_INVALID_ARG
    s = good_shape()
    tb = B.moe_dispatch(*([4096] * 9))
    args = (C.byref(s), 4096, 4096, 4096, C.byref(tb), 4096, 4096, 4096, 4096, 1 << 30, None)
    assert lib.moe_fused_forward_bounded(*args, 0, 0) == B.MOE_ERR_INVALID_ARG       # bound below 1
    assert lib.moe_fused_forward_bounded(*args, 10, -1) == B.MOE_ERR_INVALID_ARG     # negative extra count
    ev = (C.c_void_p * 5)()
    assert lib.moe_fused_forward_resident(*args, ev, -1, 0) == B.MOE_ERR_INVALID_ARG   # negative bound
    assert lib.moe_fused_forward_resident(*args, ev, 0, -1) == B.MOE_ERR_INVALID_ARG   # negative extra count
    assert lib.moe_fused_forward_resident(C.byref(s), None, *args[2:], None, 0, 0) == B.MOE_ERR_INVALID_ARG
    small_ws = args[:9] + (16, None)
    assert lib.moe_fused_forward_resident(*small_ws, None, 0, 0) == B.MOE_ERR_WORKSPACE
    f32 = good_shape(dtype=B.MOE_F32)
    assert lib.moe_fused_forward_resident(C.byref(f32), *args[1:], None, 0, 0) == B.MOE_ERR_UNSUPPORTED  # bf16 only
    args32 = (C.byref(f32),) + args[1:]
    assert lib.moe_fused_forward_bounded(*args32, 10, 0) == B.MOE_ERR_UNSUPPORTED    # resident kernel: bf16 only


def test_route_from_x_rejects_bad_arguments():
    lib = B.lib()
    s = good_shape()
    need = B.moe_route_from_x_workspace_bytes(s)
    assert need >= s.T * s.E * 4 and B.moe_route_from_x_workspace_bytes(good_shape(k=0)) == 0
    ok = (4096, 4096, None, 4096, 4096, 4096, need, None)
    assert lib.moe_route_from_x(C.byref(good_shape(E=10, R=4)), *ok) == B.MOE_ERR_INVALID_ARG
    assert lib.moe_route_from_x(C.byref(s), None, *ok[1:]) == B.MOE_ERR_INVALID_ARG
    assert lib.moe_route_from_x(C.byref(s), 4096, None, *ok[2:]) == B.MOE_ERR_INVALID_ARG
    assert lib.moe_route_from_x(C.byref(s), 4096, 4096, None, None, 4096, 4096, need, None) == B.MOE_ERR_INVALID_ARG
    assert lib.moe_route_from_x(C.byref(s), 4104, *ok[1:]) == B.MOE_ERR_INVALID_ARG            # x not 16-byte aligned
    assert lib.moe_route_from_x(C.byref(s), 4096, 4096, None, 4096, 4096, None, need, None) == B.MOE_ERR_WORKSPACE
    assert lib.moe_route_from_x(C.byref(s), 4096, 4096, None, 4096, 4096, 4096, need - 1, None) == B.MOE_ERR_WORKSPACE
    assert lib.moe_route_from_x(C.byref(good_shape(T=0)), *ok) == B.MOE_OK                      # empty layer: a no-op
