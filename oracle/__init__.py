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
