"""Thin ctypes binding of ``libmoe355.so``: argument marshalling only.

Every function has the name and argument order of its C entry point in ``include/moe355.h``; tensors are
``torch`` device tensors used as plain device memory, the stream is torch's current HIP stream.  There is no
CPU fallback: if the library is missing, loading fails.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("MOE355_LIB", os.path.join(_PKG, "libmoe355.so"))
_lib: Optional[C.CDLL] = None

MOE_F32 = 0
MOE_BF16 = 1
MOE_OK = 0
MOE_ERR_INVALID_ARG = -1
MOE_ERR_UNSUPPORTED = -2
MOE_ERR_WORKSPACE = -3
MOE_ERR_HIP = -4


class moe_shape(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("T", "d", "f", "E", "k", "R", "local_rank_begin", "local_rank_end", "dtype")]


class moe_dispatch(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("counts", "offsets", "perm", "inv_perm", "rank_counts", "rank_offsets",
                                          "dedup_tok", "dedup_mask", "pair_to_dedup")]


class MoeError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} ({status})")


def lib() -> C.CDLL:
    """Load the HIP library; raises if it has not been built (there is no fallback path)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'`")
        # torch ships its own HIP runtime (same SONAME as the system one).  Import it first so that this library
        # binds to the runtime that owns torch's streams and allocations instead of loading a second copy.
        import torch  # noqa: F401
        L = C.CDLL(LIB_PATH)
        vp, sz, i32 = C.c_void_p, C.c_size_t, C.c_int
        sp, dp = C.POINTER(moe_shape), C.POINTER(moe_dispatch)
        L.moe_dispatch_workspace_bytes.restype = sz
        L.moe_dispatch_workspace_bytes.argtypes = [sp]
        L.moe_forward_workspace_bytes.restype = sz
        L.moe_forward_workspace_bytes.argtypes = [sp]
        L.moe_unfused_workspace_bytes.restype = sz
        L.moe_unfused_workspace_bytes.argtypes = [sp]
        L.moe_forward_gemm_launches.restype = i32
        L.moe_forward_gemm_launches.argtypes = [sp]
        L.moe_packed_weight_bytes.restype = sz
        L.moe_packed_weight_bytes.argtypes = [sp, i32]
        L.moe_router_workspace_bytes.restype = sz
        L.moe_router_workspace_bytes.argtypes = [sp]
        L.moe_router_logits.restype = i32
        L.moe_router_logits.argtypes = [sp, vp, vp, vp, vp, sz, vp]
        L.moe_route_topk.restype = i32
        L.moe_route_topk.argtypes = [sp, vp, vp, vp, vp]
        L.moe_route_from_x_workspace_bytes.restype = sz
        L.moe_route_from_x_workspace_bytes.argtypes = [sp]
        L.moe_route_from_x.restype = i32
        L.moe_route_from_x.argtypes = [sp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.moe_build_dispatch.restype = i32
        L.moe_build_dispatch.argtypes = [sp, vp, dp, vp, sz, vp]
        L.moe_build_dispatch_noalloc.restype = i32
        L.moe_build_dispatch_noalloc.argtypes = [sp, vp, dp, vp]
        L.moe_workspace_bytes.restype = sz
        L.moe_workspace_bytes.argtypes = [sp]
        L.moe_forward_status.restype = i32
        L.moe_forward_status.argtypes = [vp, C.POINTER(C.c_int32), vp]
        L.moe_fused_forward_bounded.restype = i32
        L.moe_fused_forward_bounded.argtypes = [sp, vp, vp, vp, dp, vp, vp, vp, vp, sz, vp, i32, i32]
        L.moe_pack_weights.restype = i32
        L.moe_pack_weights.argtypes = [sp, vp, vp, vp, vp, vp, vp]
        for name in ("moe_fused_forward", "moe_unfused_forward"):
            fn = getattr(L, name)
            fn.restype = i32
            fn.argtypes = [sp, vp, vp, vp, dp, vp, vp, vp, vp, sz, vp]
        for name in ("moe_fused_forward_timed", "moe_fused_forward_two_launch", "moe_fused_forward_one_launch"):
            fn = getattr(L, name)
            fn.restype = i32
            fn.argtypes = [sp, vp, vp, vp, dp, vp, vp, vp, vp, sz, vp, C.POINTER(vp)]
        L.moe_fused_forward_resident.restype = i32
        L.moe_fused_forward_resident.argtypes = [sp, vp, vp, vp, dp, vp, vp, vp, vp, sz, vp, C.POINTER(vp), i32, i32]
        L.moe_route_topk_gate.restype = i32
        L.moe_route_topk_gate.argtypes = [sp, vp, vp, i32, vp, vp, vp]
        L.moe_probe_mfma_rate.restype = i32
        L.moe_probe_mfma_rate.argtypes = [i32, i32, vp, sz, C.POINTER(C.c_double), vp]
        L.moe_route_backward.restype = i32
        L.moe_route_backward.argtypes = [sp, vp, vp, vp, vp, vp]
        L.moe_fp8_packed_weight_bytes.restype = sz
        L.moe_fp8_packed_weight_bytes.argtypes = [sp, i32]
        L.moe_fp8_forward_workspace_bytes.restype = sz
        L.moe_fp8_forward_workspace_bytes.argtypes = [sp]
        L.moe_fp8_pack_weights.restype = i32
        L.moe_fp8_pack_weights.argtypes = [sp, vp, vp, vp, vp, vp, vp]
        L.moe_fp8_quantize_rows.restype = i32
        L.moe_fp8_quantize_rows.argtypes = [C.c_int64, i32, vp, vp, vp, vp]
        L.moe_fp8_fused_forward.restype = i32
        L.moe_fp8_fused_forward.argtypes = [sp, vp, vp, vp, dp, vp, vp, vp, vp, vp, sz, vp, C.POINTER(vp)]
        for name in ("moe_train_kept_bytes", "moe_backward_workspace_bytes"):
            getattr(L, name).restype = sz
            getattr(L, name).argtypes = [sp]
        L.moe_backward_packed_weight_bytes.restype = sz
        L.moe_backward_packed_weight_bytes.argtypes = [sp, i32]
        L.moe_pack_weights_backward.restype = i32
        L.moe_pack_weights_backward.argtypes = [sp, vp, vp, vp, vp, vp, vp]
        L.moe_fused_forward_train.restype = i32
        L.moe_fused_forward_train.argtypes = [sp, vp, vp, vp, dp, vp, vp, vp, vp, sz, vp, sz, vp]
        L.moe_fused_backward.restype = i32
        L.moe_fused_backward.argtypes = [sp, vp, vp, vp, vp, dp, vp, vp, vp, sz, vp, vp, vp, vp, vp, vp, sz, vp]
        L.moe_dispatch_gather.restype = i32
        L.moe_dispatch_gather.argtypes = [sp, vp, dp, vp, vp]
        L.moe_combine_reduce.restype = i32
        L.moe_combine_reduce.argtypes = [sp, vp, vp, dp, vp, vp]
        L.moe_status_string.restype = C.c_char_p
        L.moe_status_string.argtypes = [i32]
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().moe_status_string(int(status)).decode()


def make_shape(T, d, f, E, k, R, local_rank_begin, local_rank_end, dtype) -> moe_shape:
    return moe_shape(T, d, f, E, k, R, local_rank_begin, local_rank_end, dtype)


def shape_of(cfg) -> moe_shape:
    """moe_shape of a workloads.MoEConfig-like object."""
    return moe_shape(cfg.T, cfg.d, cfg.f, cfg.E, cfg.k, cfg.R, cfg.local_rank_begin, cfg.local_rank_end, cfg.dtype)


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is not None:
        return int(stream)
    import torch
    return int(torch.cuda.current_stream().cuda_stream)


def _check(rc: int, where: str) -> None:
    if rc != MOE_OK:
        raise MoeError(rc, where)


class DispatchTables:
    """Caller-owned device arrays of a moe_dispatch plus the struct that points at them."""

    def __init__(self, shape: moe_shape, device="cuda"):
        import torch
        T, E, k, R = shape.T, shape.E, shape.k, shape.R
        i32 = dict(dtype=torch.int32, device=device)
        n = max(1, T * k)
        cap = max(1, T * min(k, R))
        self.counts = torch.empty(E, **i32)
        self.offsets = torch.empty(E + 1, **i32)
        self.perm = torch.empty(n, **i32)
        self.inv_perm = torch.empty(n, **i32)
        self.rank_counts = torch.empty(R, **i32)
        self.rank_offsets = torch.empty(R + 1, **i32)
        self.dedup_tok = torch.empty(cap, **i32)
        self.dedup_mask = torch.empty(cap, **i32)  # bit patterns of uint32
        self.pair_to_dedup = torch.empty(n, **i32)
        self.struct = moe_dispatch(*(getattr(self, n_).data_ptr() for n_, _ in moe_dispatch._fields_))


def moe_dispatch_workspace_bytes(shape: moe_shape) -> int:
    return int(lib().moe_dispatch_workspace_bytes(C.byref(shape)))


def moe_forward_workspace_bytes(shape: moe_shape) -> int:
    return int(lib().moe_forward_workspace_bytes(C.byref(shape)))


def moe_unfused_workspace_bytes(shape: moe_shape) -> int:
    return int(lib().moe_unfused_workspace_bytes(C.byref(shape)))


def moe_packed_weight_bytes(shape: moe_shape, which: int) -> int:
    return int(lib().moe_packed_weight_bytes(C.byref(shape), which))


def moe_router_workspace_bytes(shape: moe_shape) -> int:
    return int(lib().moe_router_workspace_bytes(C.byref(shape)))


def moe_router_logits(shape, x, W_r, logits, workspace, workspace_bytes=None, stream=None) -> None:
    nbytes = workspace.numel() * workspace.element_size() if workspace_bytes is None else workspace_bytes
    _check(lib().moe_router_logits(C.byref(shape), _ptr(x), _ptr(W_r), _ptr(logits), _ptr(workspace), nbytes,
                                   _stream(stream)), "moe_router_logits")


def moe_route_from_x_workspace_bytes(shape: moe_shape) -> int:
    return int(lib().moe_route_from_x_workspace_bytes(C.byref(shape)))


def moe_route_from_x(shape, x, W_r, logits, topk_idx, topk_w, workspace, workspace_bytes=None, stream=None) -> None:
    """`logits` may be None: the logits then never reach memory."""
    nbytes = workspace.numel() * workspace.element_size() if workspace_bytes is None else workspace_bytes
    _check(lib().moe_route_from_x(C.byref(shape), _ptr(x), _ptr(W_r), _ptr(logits), _ptr(topk_idx), _ptr(topk_w),
                                  _ptr(workspace), nbytes, _stream(stream)), "moe_route_from_x")


def moe_route_topk(shape, logits, topk_idx, topk_w, stream=None) -> None:
    _check(lib().moe_route_topk(C.byref(shape), _ptr(logits), _ptr(topk_idx), _ptr(topk_w), _stream(stream)),
           "moe_route_topk")


def moe_build_dispatch(shape, topk_idx, tables: DispatchTables, workspace, workspace_bytes=None, stream=None) -> None:
    nbytes = workspace.numel() * workspace.element_size() if workspace_bytes is None else workspace_bytes
    _check(lib().moe_build_dispatch(C.byref(shape), _ptr(topk_idx), C.byref(tables.struct), _ptr(workspace), nbytes,
                                    _stream(stream)), "moe_build_dispatch")


def moe_build_dispatch_noalloc(shape, topk_idx, tables: DispatchTables, stream=None) -> None:
    _check(lib().moe_build_dispatch_noalloc(C.byref(shape), _ptr(topk_idx), C.byref(tables.struct), _stream(stream)),
           "moe_build_dispatch_noalloc")


def moe_workspace_bytes(shape: moe_shape) -> int:
    return int(lib().moe_workspace_bytes(C.byref(shape)))


def moe_forward_status(workspace, stream=None) -> int:
    """0, or 1 if a wait inside the resident GEMM kernel of the last forward call on this workspace gave up.
    Synchronises with the stream."""
    flag = C.c_int32(-1)
    _check(lib().moe_forward_status(_ptr(workspace), C.byref(flag), _stream(stream)), "moe_forward_status")
    return int(flag.value)


def moe_fused_forward_bounded(shape, x, topk_idx, topk_w, tables, packed_gate_up, packed_down, y, workspace,
                              max_polls: int, wait_extra: int = 0, workspace_bytes=None, stream=None) -> None:
    nbytes = workspace.numel() * workspace.element_size() if workspace_bytes is None else workspace_bytes
    _check(lib().moe_fused_forward_bounded(C.byref(shape), _ptr(x), _ptr(topk_idx), _ptr(topk_w),
                                           C.byref(tables.struct), _ptr(packed_gate_up), _ptr(packed_down), _ptr(y),
                                           _ptr(workspace), nbytes, _stream(stream), int(max_polls),
                                           int(wait_extra)),
           "moe_fused_forward_bounded")


def moe_pack_weights(shape, W_gate, W_up, W_down, packed_gate_up, packed_down, stream=None) -> None:
    _check(lib().moe_pack_weights(C.byref(shape), _ptr(W_gate), _ptr(W_up), _ptr(W_down), _ptr(packed_gate_up),
                                  _ptr(packed_down), _stream(stream)), "moe_pack_weights")


def _forward(name, shape, x, topk_idx, topk_w, tables, packed_gate_up, packed_down, y, workspace, workspace_bytes,
             stream):
    nbytes = workspace.numel() * workspace.element_size() if workspace_bytes is None else workspace_bytes
    _check(getattr(lib(), name)(C.byref(shape), _ptr(x), _ptr(topk_idx), _ptr(topk_w), C.byref(tables.struct),
                                _ptr(packed_gate_up), _ptr(packed_down), _ptr(y), _ptr(workspace), nbytes,
                                _stream(stream)), name)


def moe_fused_forward(shape, x, topk_idx, topk_w, tables, packed_gate_up, packed_down, y, workspace,
                      workspace_bytes=None, stream=None) -> None:
    _forward("moe_fused_forward", shape, x, topk_idx, topk_w, tables, packed_gate_up, packed_down, y, workspace,
             workspace_bytes, stream)


def moe_fused_forward_timed(shape, x, topk_idx, topk_w, tables, packed_gate_up, packed_down, y, workspace, events,
                            workspace_bytes=None, stream=None) -> None:
    """`events`: five raw hipEvent_t handles (ints), e.g. ``torch.cuda.Event(enable_timing=True).cuda_event``."""
    nbytes = workspace.numel() * workspace.element_size() if workspace_bytes is None else workspace_bytes
    arr = (C.c_void_p * 5)(*[C.c_void_p(int(e)) if e else None for e in events])
    _check(lib().moe_fused_forward_timed(C.byref(shape), _ptr(x), _ptr(topk_idx), _ptr(topk_w),
                                         C.byref(tables.struct), _ptr(packed_gate_up), _ptr(packed_down), _ptr(y),
                                         _ptr(workspace), nbytes, _stream(stream), arr), "moe_fused_forward_timed")


def moe_forward_gemm_launches(shape) -> int:
    return int(lib().moe_forward_gemm_launches(C.byref(shape)))


def _forward_choice(name, shape, x, topk_idx, topk_w, tables, packed_gate_up, packed_down, y, workspace, events,
                    workspace_bytes, stream):
    nbytes = workspace.numel() * workspace.element_size() if workspace_bytes is None else workspace_bytes
    arr = None if events is None else (C.c_void_p * 5)(*[C.c_void_p(int(e)) if e else None for e in events])
    _check(getattr(lib(), name)(C.byref(shape), _ptr(x), _ptr(topk_idx), _ptr(topk_w), C.byref(tables.struct),
                                _ptr(packed_gate_up), _ptr(packed_down), _ptr(y), _ptr(workspace), nbytes,
                                _stream(stream), arr), name)


def moe_fused_forward_two_launch(shape, x, topk_idx, topk_w, tables, packed_gate_up, packed_down, y, workspace,
                                 events=None, workspace_bytes=None, stream=None) -> None:
    """`events`: None or five raw hipEvent_t handles as for moe_fused_forward_timed."""
    _forward_choice("moe_fused_forward_two_launch", shape, x, topk_idx, topk_w, tables, packed_gate_up, packed_down,
                    y, workspace, events, workspace_bytes, stream)


def moe_fused_forward_one_launch(shape, x, topk_idx, topk_w, tables, packed_gate_up, packed_down, y, workspace,
                                 events=None, workspace_bytes=None, stream=None) -> None:
    """`events`: None or five raw hipEvent_t handles as for moe_fused_forward_timed."""
    _forward_choice("moe_fused_forward_one_launch", shape, x, topk_idx, topk_w, tables, packed_gate_up, packed_down,
                    y, workspace, events, workspace_bytes, stream)


def moe_fused_forward_resident(shape, x, topk_idx, topk_w, tables, packed_gate_up, packed_down, y, workspace,
                               events=None, max_polls: int = 0, wait_extra: int = 0, workspace_bytes=None,
                               stream=None) -> None:
    """Tile table, then ONE launch for GEMM-1, GEMM-2 and Combine.  max_polls 0 = the library's default bound."""
    nbytes = workspace.numel() * workspace.element_size() if workspace_bytes is None else workspace_bytes
    arr = None if events is None else (C.c_void_p * 5)(*[C.c_void_p(int(e)) if e else None for e in events])
    _check(lib().moe_fused_forward_resident(C.byref(shape), _ptr(x), _ptr(topk_idx), _ptr(topk_w),
                                            C.byref(tables.struct), _ptr(packed_gate_up), _ptr(packed_down), _ptr(y),
                                            _ptr(workspace), nbytes, _stream(stream), arr, int(max_polls),
                                            int(wait_extra)), "moe_fused_forward_resident")


def moe_unfused_forward(shape, x, topk_idx, topk_w, tables, packed_gate_up, packed_down, y, workspace,
                        workspace_bytes=None, stream=None) -> None:
    _forward("moe_unfused_forward", shape, x, topk_idx, topk_w, tables, packed_gate_up, packed_down, y, workspace,
             workspace_bytes, stream)


MOE_GATE_SOFTMAX = 0
MOE_GATE_SIGMOID = 1


def moe_route_topk_gate(shape, logits, bias, gate, topk_idx, topk_w, stream=None) -> None:
    _check(lib().moe_route_topk_gate(C.byref(shape), _ptr(logits), _ptr(bias), int(gate), _ptr(topk_idx),
                                     _ptr(topk_w), _stream(stream)), "moe_route_topk_gate")


def moe_probe_mfma_rate(workgroups: int, iters: int, sink, stream=None) -> float:
    """Launches the matrix-core rate probe; returns the floating point operations of the launch."""
    flops = C.c_double(0.0)
    _check(lib().moe_probe_mfma_rate(workgroups, iters, _ptr(sink), sink.numel(), C.byref(flops), _stream(stream)),
           "moe_probe_mfma_rate")
    return float(flops.value)


def moe_route_backward(shape, topk_idx, topk_w, d_topk_w, dlogits, stream=None) -> None:
    _check(lib().moe_route_backward(C.byref(shape), _ptr(topk_idx), _ptr(topk_w), _ptr(d_topk_w), _ptr(dlogits),
                                    _stream(stream)), "moe_route_backward")


def moe_fp8_packed_weight_bytes(shape: moe_shape, which: int) -> int:
    return int(lib().moe_fp8_packed_weight_bytes(C.byref(shape), which))


def moe_fp8_forward_workspace_bytes(shape: moe_shape) -> int:
    return int(lib().moe_fp8_forward_workspace_bytes(C.byref(shape)))


def moe_fp8_pack_weights(shape, W_gate, W_up, W_down, packed_gate_up, packed_down, stream=None) -> None:
    _check(lib().moe_fp8_pack_weights(C.byref(shape), _ptr(W_gate), _ptr(W_up), _ptr(W_down), _ptr(packed_gate_up),
                                      _ptr(packed_down), _stream(stream)), "moe_fp8_pack_weights")


def moe_fp8_quantize_rows(rows: int, cols: int, x, codes, scales, stream=None) -> None:
    _check(lib().moe_fp8_quantize_rows(rows, cols, _ptr(x), _ptr(codes), _ptr(scales), _stream(stream)),
           "moe_fp8_quantize_rows")


def moe_fp8_fused_forward(shape, x, topk_idx, topk_w, tables, packed_gate_up, packed_down, h_scale, y, workspace,
                          events=None, workspace_bytes=None, stream=None) -> None:
    """`events`: None or five raw hipEvent_t handles as for moe_fused_forward_timed."""
    nbytes = workspace.numel() * workspace.element_size() if workspace_bytes is None else workspace_bytes
    arr = None if events is None else (C.c_void_p * 5)(*[C.c_void_p(int(e)) if e else None for e in events])
    _check(lib().moe_fp8_fused_forward(C.byref(shape), _ptr(x), _ptr(topk_idx), _ptr(topk_w), C.byref(tables.struct),
                                       _ptr(packed_gate_up), _ptr(packed_down), _ptr(h_scale), _ptr(y),
                                       _ptr(workspace), nbytes, _stream(stream), arr), "moe_fp8_fused_forward")


def _nbytes(t) -> int:
    return t.numel() * t.element_size()


def moe_train_kept_bytes(shape: moe_shape) -> int:
    return int(lib().moe_train_kept_bytes(C.byref(shape)))


def moe_backward_workspace_bytes(shape: moe_shape) -> int:
    return int(lib().moe_backward_workspace_bytes(C.byref(shape)))


def moe_backward_packed_weight_bytes(shape: moe_shape, which: int) -> int:
    return int(lib().moe_backward_packed_weight_bytes(C.byref(shape), which))


def moe_pack_weights_backward(shape, W_gate, W_up, W_down, packed_down_t, packed_gate_up_t, stream=None) -> None:
    _check(lib().moe_pack_weights_backward(C.byref(shape), _ptr(W_gate), _ptr(W_up), _ptr(W_down),
                                           _ptr(packed_down_t), _ptr(packed_gate_up_t), _stream(stream)),
           "moe_pack_weights_backward")


def moe_fused_forward_train(shape, x, topk_idx, topk_w, tables, packed_gate_up, packed_down, y, kept, workspace,
                            stream=None) -> None:
    _check(lib().moe_fused_forward_train(C.byref(shape), _ptr(x), _ptr(topk_idx), _ptr(topk_w),
                                         C.byref(tables.struct), _ptr(packed_gate_up), _ptr(packed_down), _ptr(y),
                                         _ptr(kept), _nbytes(kept), _ptr(workspace), _nbytes(workspace),
                                         _stream(stream)), "moe_fused_forward_train")


def moe_fused_backward(shape, x, dy, topk_idx, topk_w, tables, packed_down_t, packed_gate_up_t, kept, dx, d_topk_w,
                       dW_gate, dW_up, dW_down, workspace, stream=None) -> None:
    _check(lib().moe_fused_backward(C.byref(shape), _ptr(x), _ptr(dy), _ptr(topk_idx), _ptr(topk_w),
                                    C.byref(tables.struct), _ptr(packed_down_t), _ptr(packed_gate_up_t), _ptr(kept),
                                    _nbytes(kept), _ptr(dx), _ptr(d_topk_w), _ptr(dW_gate), _ptr(dW_up),
                                    _ptr(dW_down), _ptr(workspace), _nbytes(workspace), _stream(stream)),
           "moe_fused_backward")


def moe_dispatch_gather(shape, x, tables, xs, stream=None) -> None:
    _check(lib().moe_dispatch_gather(C.byref(shape), _ptr(x), C.byref(tables.struct), _ptr(xs), _stream(stream)),
           "moe_dispatch_gather")


def moe_combine_reduce(shape, rows, topk_idx, tables, y, stream=None) -> None:
    _check(lib().moe_combine_reduce(C.byref(shape), _ptr(rows), _ptr(topk_idx), C.byref(tables.struct), _ptr(y),
                                    _stream(stream)), "moe_combine_reduce")
