"""NumPy re-derivations used to pin the oracle.  Each routine takes a different route from the oracle's
C loops (library sorts, sets, dense matmul in float64) so that an index, sign or transposition mistake in
the oracle cannot also be present here."""
import math

import numpy as np


def route_bruteforce(logits: np.ndarray, k: int):
    """Full stable descending sort of every row; weights = full fp64 softmax over all experts, then
    renormalised over the k picks."""
    logits = np.asarray(logits, dtype=np.float32)
    order = np.argsort(-logits.astype(np.float64), axis=1, kind="stable")[:, :k]
    z = logits.astype(np.float64)
    p = np.exp(z - z.max(axis=1, keepdims=True))
    p /= p.sum(axis=1, keepdims=True)
    sel = np.take_along_axis(p, order, axis=1)
    return order.astype(np.int32), sel / sel.sum(axis=1, keepdims=True)


def tables_bruteforce(topk_idx: np.ndarray, E: int):
    """Stable argsort of the flattened expert ids is the row -> pair map when a token's experts are distinct."""
    flat = np.asarray(topk_idx).ravel()
    perm = np.argsort(flat, kind="stable").astype(np.int32)
    inv = np.empty_like(perm)
    inv[perm] = np.arange(perm.size, dtype=np.int32)
    counts = np.bincount(flat, minlength=E).astype(np.int32)
    offsets = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    return counts, offsets, perm, inv


def dedup_bruteforce(topk_idx: np.ndarray, E: int, R: int):
    """Set of (rank, token) pairs by exhaustive enumeration; sorted tuples give the table order."""
    T, k = topk_idx.shape
    epr = E // R
    pairs = {}
    for t in range(T):
        for j in range(k):
            key = (int(topk_idx[t, j]) // epr, t)
            pairs[key] = pairs.get(key, 0) | (1 << j)
    keys = sorted(pairs)
    pos = {key: i for i, key in enumerate(keys)}
    tok = np.array([t for _, t in keys], dtype=np.int32)
    mask = np.array([pairs[key] for key in keys], dtype=np.uint32)
    rank_counts = np.array([sum(1 for r, _ in keys if r == rr) for rr in range(R)], dtype=np.int32)
    p2d = np.array([[pos[(int(topk_idx[t, j]) // epr, t)] for j in range(k)] for t in range(T)], dtype=np.int32)
    return rank_counts, tok, mask, p2d.ravel()


def ffn_dense(x, Wg, Wu, Wd):
    """One dense SwiGLU FFN in float64 with library matmuls."""
    x, Wg, Wu, Wd = (np.asarray(a, dtype=np.float64) for a in (x, Wg, Wu, Wd))
    g = x @ Wg
    return ((g / (1.0 + np.exp(-g))) * (x @ Wu)) @ Wd


def forward_bruteforce(x, logits, k, Wg, Wu, Wd, E, R, lrb, lre):
    """No tables at all: per token recompute the routing from the logits, loop over all experts and add the
    expert's dense FFN output if the expert is among the picks and local."""
    x = np.asarray(x, dtype=np.float64)
    T, d = x.shape
    idx, w = route_bruteforce(logits, k)
    epr = E // R
    y = np.zeros((T, d))
    for e in range(lrb * epr, lre * epr):
        le = e - lrb * epr
        out_e = ffn_dense(x, Wg[le], Wu[le], Wd[le])
        for t in range(T):
            for j in range(k):
                if idx[t, j] == e:
                    y[t] += w[t, j] * out_e[t]
    return y


def expected_unique_ranks_per_token(E: int, R: int, k: int) -> float:
    """E[#distinct ranks hit by a uniformly random k-subset of E experts] = R (1 - C(E-E/R, k) / C(E, k))."""
    epr = E // R
    return R * (1.0 - math.comb(E - epr, k) / math.comb(E, k))


# ---------------------------------------------------------------- FP8 (E4M3) through a library's conversions
def e4m3_values_closed_form():
    """The 256 code values from the format's definition: sign, 4 exponent bits with bias 7, 3 mantissa bits,
    subnormals m/8 * 2^-6, S.1111.111 = NaN, no infinities (OCP 8-bit floating point specification, E4M3)."""
    out = np.empty(256, dtype=np.float64)
    for c in range(256):
        s, e, m = c >> 7, (c >> 3) & 15, c & 7
        if e == 15 and m == 7:
            v = math.nan
        elif e == 0:
            v = m / 8.0 * 2.0 ** -6
        else:
            v = (1.0 + m / 8.0) * 2.0 ** (e - 7)
        out[c] = -v if s else v
    return out


def e4m3_round_library(v32: np.ndarray):
    """float32 -> nearest E4M3 value and code with PyTorch's CPU conversion (round to nearest even), after the
    saturation to +-448 that the conversion itself does not do."""
    import torch
    t = torch.from_numpy(np.clip(np.asarray(v32, dtype=np.float32), -448.0, 448.0)).to(torch.float8_e4m3fn)
    return t.to(torch.float32).numpy().astype(np.float64), t.view(torch.uint8).numpy()


def ffn_dense_fp8(x, Wg, Wu, Wd, s_h):
    """One dense SwiGLU FFN with E4M3 operands: per-row scale for x, per-column scales for the weights, a static
    scale for h; library conversions and float64 library matmuls."""
    x, Wg, Wu, Wd = (np.asarray(a, dtype=np.float32) for a in (x, Wg, Wu, Wd))

    def scale_of(amax):
        amax = amax.astype(np.float32)
        return np.where(amax > 0, amax / np.float32(448.0), np.float32(1.0)).astype(np.float32)

    sx = scale_of(np.abs(x).max(axis=1))
    xv, _ = e4m3_round_library(x / sx[:, None])
    sg, su, sd = (scale_of(np.abs(W).max(axis=0)) for W in (Wg, Wu, Wd))
    gv, _ = e4m3_round_library(Wg / sg[None, :])
    uv, _ = e4m3_round_library(Wu / su[None, :])
    dv, _ = e4m3_round_library(Wd / sd[None, :])
    g = (xv @ gv) * sx[:, None].astype(np.float64) * sg[None, :].astype(np.float64)
    u = (xv @ uv) * sx[:, None].astype(np.float64) * su[None, :].astype(np.float64)
    h32 = ((g / (1.0 + np.exp(-g))) * u).astype(np.float32)
    hv, _ = e4m3_round_library(h32 / np.float32(s_h))
    return (hv @ dv) * float(np.float32(s_h)) * sd[None, :].astype(np.float64)
