"""ctypes front end of the CPU oracle (``moe_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke()`` and by the
``cpu_baseline`` leg of ``bench.py``.  The GPU library never imports or links anything from here.

Two builds of the same source exist: ``libmoe_oracle.so`` accumulates in double (the reference used
for parity) and ``libmoe_oracle_f32.so`` accumulates in float (the "plain fp32 layer"; used to bound
the reference's own rounding error).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "moe_oracle.c")
_LIBS = {"f64": os.path.join(_HERE, "libmoe_oracle.so"), "f32": os.path.join(_HERE, "libmoe_oracle_f32.so")}
_loaded: dict = {}

ELT_F32 = 0
ELT_BF16 = 1


def build(force: bool = True) -> None:
    """Compile both variants with gcc."""
    for acc, out in _LIBS.items():
        if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(_SRC):
            continue
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
               "-DMOE_ACC_T=" + ("double" if acc == "f64" else "float"), _SRC, "-o", out, "-lm"]
        subprocess.run(cmd, check=True)


def _lib(acc: str = "f64") -> C.CDLL:
    if acc not in _loaded:
        if not os.path.exists(_LIBS[acc]):
            build(force=False)
        lib = C.CDLL(_LIBS[acc])
        assert lib.moe_oracle_acc_bytes() == (8 if acc == "f64" else 4)
        _loaded[acc] = lib
    return _loaded[acc]


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise ValueError(f"oracle {what} failed with status {rc}")


def max_threads() -> int:
    return int(_lib().moe_oracle_max_threads())


def router_logits(x: np.ndarray, W_r: np.ndarray, acc: str = "f64") -> np.ndarray:
    """Gate-network logits [T, E] (float64): x [T, d] times the rows of W_r [E, d].

    float32 arrays are taken as such; uint16 arrays as bf16 bit patterns (both operands alike)."""
    if x.dtype == np.uint16:
        elt = ELT_BF16
    elif x.dtype == np.float32:
        elt = ELT_F32
    else:
        raise TypeError("x must be float32 or uint16 (bf16 bits)")
    if W_r.dtype != x.dtype:
        raise TypeError("W_r must have the element type of x")
    x, W_r = np.ascontiguousarray(x), np.ascontiguousarray(W_r)
    T, d = x.shape
    E, d2 = W_r.shape
    assert d2 == d
    out = np.empty((T, E), dtype=np.float64)
    lib = _lib(acc)
    lib.moe_oracle_router_logits.argtypes = [C.c_int] * 4 + [C.c_void_p] * 3
    _check(lib.moe_oracle_router_logits(T, d, E, elt, _p(x), _p(W_r), _p(out)), "router_logits")
    return out


def route_topk(logits: np.ndarray, k: int):
    logits = np.ascontiguousarray(logits, dtype=np.float32)
    T, E = logits.shape
    idx = np.empty((T, k), dtype=np.int32)
    w = np.empty((T, k), dtype=np.float32)
    _check(_lib().moe_oracle_route_topk(T, E, k, _p(logits), _p(idx), _p(w)), "route_topk")
    return idx, w


GATE_SOFTMAX = 0
GATE_SIGMOID = 1


def route_topk_gate(logits: np.ndarray, k: int, gate: int, bias: Optional[np.ndarray] = None):
    """Routing with a softmax or sigmoid gate and an optional selection-only bias.  Returns (idx, w, sel): sel is
    the [T, E] float32 array of selection values."""
    logits = np.ascontiguousarray(logits, dtype=np.float32)
    T, E = logits.shape
    if bias is not None:
        bias = np.ascontiguousarray(bias, dtype=np.float32)
        assert bias.shape == (E,)
    idx = np.empty((T, k), dtype=np.int32)
    w = np.empty((T, k), dtype=np.float32)
    sel = np.empty((T, E), dtype=np.float32)
    _check(_lib().moe_oracle_route_topk_gate(T, E, k, _p(logits), _p(bias), int(gate), _p(idx), _p(w), _p(sel)),
           "route_topk_gate")
    return idx, w, sel


def build_tables(topk_idx: np.ndarray, E: int):
    topk_idx = np.ascontiguousarray(topk_idx, dtype=np.int32)
    T, k = topk_idx.shape
    counts = np.empty(E, dtype=np.int32)
    offsets = np.empty(E + 1, dtype=np.int32)
    perm = np.empty(T * k, dtype=np.int32)
    inv_perm = np.empty(T * k, dtype=np.int32)
    _check(_lib().moe_oracle_build_tables(T, E, k, _p(topk_idx), _p(counts), _p(offsets), _p(perm), _p(inv_perm)),
           "build_tables")
    return counts, offsets, perm, inv_perm


def build_dedup(topk_idx: np.ndarray, E: int, R: int):
    topk_idx = np.ascontiguousarray(topk_idx, dtype=np.int32)
    T, k = topk_idx.shape
    cap = T * min(k, R)
    rank_counts = np.empty(R, dtype=np.int32)
    rank_offsets = np.empty(R + 1, dtype=np.int32)
    dedup_tok = np.full(cap, -1, dtype=np.int32)
    dedup_mask = np.zeros(cap, dtype=np.uint32)
    pair_to_dedup = np.empty(T * k, dtype=np.int32)
    _check(_lib().moe_oracle_build_dedup(T, E, k, R, _p(topk_idx), _p(rank_counts), _p(rank_offsets),
                                         _p(dedup_tok), _p(dedup_mask), _p(pair_to_dedup)), "build_dedup")
    n = int(rank_offsets[R])
    return rank_counts, rank_offsets, dedup_tok[:n].copy(), dedup_mask[:n].copy(), pair_to_dedup


def forward(x: np.ndarray, topk_idx: np.ndarray, topk_w: np.ndarray, W_gate: np.ndarray, W_up: np.ndarray,
            W_down: np.ndarray, E: int, R: int, local_rank_begin: int, local_rank_end: int,
            tokens: Optional[np.ndarray] = None, acc: str = "f64") -> np.ndarray:
    """y rows (float64, [n_tok, d]) for the listed tokens (all tokens if ``tokens`` is None).

    Arrays of dtype float32 are taken as such; arrays of dtype uint16 are taken as bf16 bit patterns.
    """
    if x.dtype == np.uint16:
        elt = ELT_BF16
    elif x.dtype == np.float32:
        elt = ELT_F32
    else:
        raise TypeError("x must be float32 or uint16 (bf16 bits)")
    for a in (W_gate, W_up, W_down):
        if a.dtype != x.dtype:
            raise TypeError("weights must have the element type of x")
    x = np.ascontiguousarray(x)
    W_gate, W_up, W_down = (np.ascontiguousarray(a) for a in (W_gate, W_up, W_down))
    topk_idx = np.ascontiguousarray(topk_idx, dtype=np.int32)
    topk_w = np.ascontiguousarray(topk_w, dtype=np.float32)
    T, d = x.shape
    k = topk_idx.shape[1]
    El, d2, f = W_gate.shape
    assert d2 == d and W_up.shape == (El, d, f) and W_down.shape == (El, f, d)
    assert El == (local_rank_end - local_rank_begin) * (E // R)
    if tokens is not None:
        tokens = np.ascontiguousarray(tokens, dtype=np.int32)
        n_tok = int(tokens.shape[0])
    else:
        n_tok = T
    y = np.empty((n_tok, d), dtype=np.float64)
    lib = _lib(acc)
    lib.moe_oracle_forward.argtypes = [C.c_int] * 9 + [C.c_void_p] * 7 + [C.c_int, C.c_void_p]
    _check(lib.moe_oracle_forward(T, d, f, E, k, R, local_rank_begin, local_rank_end, elt, _p(x), _p(topk_idx),
                                  _p(topk_w), _p(W_gate), _p(W_up), _p(W_down), _p(tokens), n_tok, _p(y)),
           "forward")
    return y


def fp8_decode(codes: np.ndarray) -> np.ndarray:
    """Values (float64) of E4M3 codes (uint8); NaN codes give NaN."""
    lib = _lib()
    lib.moe_oracle_fp8_decode.restype = C.c_double
    lib.moe_oracle_fp8_decode.argtypes = [C.c_uint8]
    flat = np.ascontiguousarray(codes, dtype=np.uint8).ravel()
    table = np.array([lib.moe_oracle_fp8_decode(c) for c in range(256)], dtype=np.float64)
    return table[flat].reshape(np.shape(codes))


def fp8_encode(values: np.ndarray) -> np.ndarray:
    """E4M3 codes (uint8) of float32 values: nearest, ties to even, saturating at 448."""
    lib = _lib()
    lib.moe_oracle_fp8_encode.restype = C.c_uint8
    lib.moe_oracle_fp8_encode.argtypes = [C.c_float]
    flat = np.ascontiguousarray(values, dtype=np.float32).ravel()
    return np.array([lib.moe_oracle_fp8_encode(float(v)) for v in flat], dtype=np.uint8).reshape(np.shape(values))


def fp8_quantize(a: np.ndarray, axis: int):
    """Quantise a float32 array of 2 or 3 dimensions with one scale per group, a group running along ``axis`` of the
    last two dimensions (axis=-1: one scale per row, axis=-2: one scale per column; a leading dimension is a batch).
    Returns (codes uint8 of the same shape, scales float32 with ``axis`` removed)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    if a.ndim == 2:
        a3 = a[None]
    elif a.ndim == 3:
        a3 = a
    else:
        raise ValueError("2 or 3 dimensions")
    B, r, c = a3.shape
    codes = np.empty_like(a3, dtype=np.uint8)
    lib = _lib()
    lib.moe_oracle_fp8_quantize.argtypes = [C.c_void_p] + [C.c_int64] * 4 + [C.c_void_p, C.c_void_p]
    if axis in (-1, a.ndim - 1):
        scales = np.empty((B, r), dtype=np.float32)
        _check(lib.moe_oracle_fp8_quantize(_p(a3), B * r, c, c, 1, _p(codes), _p(scales)), "fp8_quantize")
    elif axis in (-2, a.ndim - 2):
        scales = np.empty((B, c), dtype=np.float32)
        for b in range(B):
            _check(lib.moe_oracle_fp8_quantize(_p(a3[b]), c, r, 1, c, _p(codes[b]), _p(scales[b])), "fp8_quantize")
    else:
        raise ValueError("axis must be one of the last two")
    if a.ndim == 2:
        return codes[0], scales[0]
    return codes, scales


def _as_f32(a: np.ndarray) -> np.ndarray:
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << 16).view(np.float32)  # bf16 bit patterns widened exactly
    if a.dtype == np.float32:
        return a
    raise TypeError("float32 or uint16 (bf16 bits)")


def forward_fp8(x: np.ndarray, topk_idx: np.ndarray, topk_w: np.ndarray, W_gate: np.ndarray, W_up: np.ndarray,
                W_down: np.ndarray, s_h: np.ndarray, E: int, R: int, local_rank_begin: int, local_rank_end: int,
                tokens: Optional[np.ndarray] = None, quantized=None) -> np.ndarray:
    """y rows (float64) of the layer with FP8 expert GEMMs (see moe_oracle.c for the scheme).  x and the weights are
    float32 or bf16 bit patterns; s_h [E_loc] float32.  ``quantized`` may carry the result of an earlier
    :func:`fp8_quantize_layer` call for the same x and weights."""
    q = quantized if quantized is not None else fp8_quantize_layer(x, W_gate, W_up, W_down)
    xq, sx, gq, sg, uq, su, dq, sd = q
    T, d = xq.shape
    El, _, f = gq.shape
    topk_idx = np.ascontiguousarray(topk_idx, dtype=np.int32)
    topk_w = np.ascontiguousarray(topk_w, dtype=np.float32)
    s_h = np.ascontiguousarray(s_h, dtype=np.float32)
    k = topk_idx.shape[1]
    assert s_h.shape == (El,) and El == (local_rank_end - local_rank_begin) * (E // R)
    if tokens is not None:
        tokens = np.ascontiguousarray(tokens, dtype=np.int32)
        n_tok = int(tokens.shape[0])
    else:
        n_tok = T
    y = np.empty((n_tok, d), dtype=np.float64)
    lib = _lib()
    lib.moe_oracle_forward_fp8.argtypes = [C.c_int] * 8 + [C.c_void_p] * 12 + [C.c_int, C.c_void_p]
    _check(lib.moe_oracle_forward_fp8(T, d, f, E, k, R, local_rank_begin, local_rank_end, _p(xq), _p(sx),
                                      _p(topk_idx), _p(topk_w), _p(gq), _p(sg), _p(uq), _p(su), _p(dq), _p(sd),
                                      _p(s_h), _p(tokens), n_tok, _p(y)), "forward_fp8")
    return y


def fp8_quantize_layer(x, W_gate, W_up, W_down):
    """Codes and scales of the operands: x per token, every weight matrix per expert and output column."""
    xq, sx = fp8_quantize(_as_f32(np.ascontiguousarray(x)), axis=-1)
    gq, sg = fp8_quantize(_as_f32(np.ascontiguousarray(W_gate)), axis=-2)
    uq, su = fp8_quantize(_as_f32(np.ascontiguousarray(W_up)), axis=-2)
    dq, sd = fp8_quantize(_as_f32(np.ascontiguousarray(W_down)), axis=-2)
    return xq, sx, gq, sg, uq, su, dq, sd


def _elt_of(a: np.ndarray) -> int:
    if a.dtype == np.uint16:
        return ELT_BF16
    if a.dtype == np.float32:
        return ELT_F32
    raise TypeError("float32 or uint16 (bf16 bits)")


def backward_tokens(x, dy, topk_idx, topk_w, W_gate, W_up, W_down, E: int, R: int, local_rank_begin: int,
                    local_rank_end: int, tokens: Optional[np.ndarray] = None):
    """Gradients with respect to x and to the gate weights for the listed tokens (all if None): (dx [n, d],
    d_topk_w [n, k]) in float64, given dy [T, d] (element type of x)."""
    elt = _elt_of(x)
    for a in (dy, W_gate, W_up, W_down):
        if a.dtype != x.dtype:
            raise TypeError("dy and the weights must have the element type of x")
    x, dy, W_gate, W_up, W_down = (np.ascontiguousarray(a) for a in (x, dy, W_gate, W_up, W_down))
    topk_idx = np.ascontiguousarray(topk_idx, dtype=np.int32)
    topk_w = np.ascontiguousarray(topk_w, dtype=np.float32)
    T, d = x.shape
    k = topk_idx.shape[1]
    El, _, f = W_gate.shape
    assert dy.shape == (T, d) and El == (local_rank_end - local_rank_begin) * (E // R)
    if tokens is not None:
        tokens = np.ascontiguousarray(tokens, dtype=np.int32)
        n = int(tokens.shape[0])
    else:
        n = T
    dx = np.empty((n, d), dtype=np.float64)
    dw = np.empty((n, k), dtype=np.float64)
    lib = _lib()
    lib.moe_oracle_backward_tokens.argtypes = [C.c_int] * 9 + [C.c_void_p] * 8 + [C.c_int, C.c_void_p, C.c_void_p]
    _check(lib.moe_oracle_backward_tokens(T, d, f, E, k, R, local_rank_begin, local_rank_end, elt, _p(x), _p(dy),
                                          _p(topk_idx), _p(topk_w), _p(W_gate), _p(W_up), _p(W_down), _p(tokens), n,
                                          _p(dx), _p(dw)), "backward_tokens")
    return dx, dw


def backward_weights(x, dy, topk_idx, topk_w, W_gate, W_up, W_down, E: int, R: int, local_rank_begin: int,
                     local_rank_end: int, le: int, n0: int = 0, n1: Optional[int] = None):
    """Weight gradients of local expert ``le`` for the hidden indices [n0, n1): (dW_gate[:, n0:n1],
    dW_up[:, n0:n1], dW_down[n0:n1, :]) in float64."""
    elt = _elt_of(x)
    x, dy, W_gate, W_up, W_down = (np.ascontiguousarray(a) for a in (x, dy, W_gate, W_up, W_down))
    topk_idx = np.ascontiguousarray(topk_idx, dtype=np.int32)
    topk_w = np.ascontiguousarray(topk_w, dtype=np.float32)
    T, d = x.shape
    k = topk_idx.shape[1]
    El, _, f = W_gate.shape
    n1 = f if n1 is None else n1
    dWg = np.empty((d, n1 - n0), dtype=np.float64)
    dWu = np.empty((d, n1 - n0), dtype=np.float64)
    dWd = np.empty((n1 - n0, d), dtype=np.float64)
    lib = _lib()
    lib.moe_oracle_backward_weights.argtypes = [C.c_int] * 9 + [C.c_void_p] * 7 + [C.c_int] * 3 + [C.c_void_p] * 3
    _check(lib.moe_oracle_backward_weights(T, d, f, E, k, R, local_rank_begin, local_rank_end, elt, _p(x), _p(dy),
                                           _p(topk_idx), _p(topk_w), _p(W_gate), _p(W_up), _p(W_down), le, n0, n1,
                                           _p(dWg), _p(dWu), _p(dWd)), "backward_weights")
    return dWg, dWu, dWd


def route_backward(logits: np.ndarray, topk_idx: np.ndarray, d_topk_w: np.ndarray) -> np.ndarray:
    """Gradient of the logits [T, E] (float64) from the gradient of the routing weights [T, k] of route_topk."""
    logits = np.ascontiguousarray(logits, dtype=np.float32)
    topk_idx = np.ascontiguousarray(topk_idx, dtype=np.int32)
    dw = np.ascontiguousarray(d_topk_w, dtype=np.float64)
    T, E = logits.shape
    k = topk_idx.shape[1]
    assert dw.shape == (T, k)
    out = np.empty((T, E), dtype=np.float64)
    _check(_lib().moe_oracle_route_backward(T, E, k, _p(logits), _p(topk_idx), _p(dw), _p(out)), "route_backward")
    return out
