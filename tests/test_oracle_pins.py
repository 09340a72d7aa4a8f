"""Pins of the CPU oracle against things other than itself (CPU only).

Each test names the mistake it is there to catch.
"""
import json
import math
import os

import numpy as np
import pytest

import brute
from paper_2605_05607_amd import workloads as wl

GOLD = os.path.join(os.path.dirname(__file__), "golden", "hand_example_4tok.json")


def small_cfg(**kw):
    base = dict(name="s", T=24, d=16, f=24, E=8, k=3, R=4, local_rank_begin=1, local_rank_end=3, dtype=wl.F32,
                router="normal", seed=7)
    base.update(kw)
    return wl.MoEConfig(**base)


# ---------------------------------------------------------------- hand-worked example
def test_hand_example_tables(oracle):
    g = json.load(open(GOLD))
    logits = np.array(g["logits"], dtype=np.float32)
    idx, w = oracle.route_topk(logits, g["k"])
    assert idx.tolist() == g["topk_idx"]  # includes the e2 == e3 tie of token 2 -> lower index first
    np.testing.assert_allclose(w, np.array(g["topk_w"]), atol=1e-7)
    counts, offsets, perm, inv = oracle.build_tables(idx, g["E"])
    assert counts.tolist() == g["counts"] and offsets.tolist() == g["offsets"]
    assert perm.tolist() == g["perm"] and inv.tolist() == g["inv_perm"]
    rc, ro, tok, mask, p2d = oracle.build_dedup(idx, g["E"], g["R"])
    assert rc.tolist() == g["rank_counts"] and ro.tolist() == g["rank_offsets"]
    assert tok.tolist() == g["dedup_tok"] and mask.tolist() == g["dedup_mask"]
    assert p2d.tolist() == g["pair_to_dedup"]


def test_hand_example_forward_identical_experts(oracle):
    """Identical experts, local = rank 0 only: y[t] = (sum of local weights) * FFN(x_t); token 2 has no local slot."""
    g = json.load(open(GOLD))
    rng = np.random.default_rng(3)
    d, f = 8, 12
    x = rng.standard_normal((4, d)).astype(np.float32)
    Wg1, Wu1 = rng.standard_normal((2, d, f)).astype(np.float32) * 0.3
    Wd1 = rng.standard_normal((f, d)).astype(np.float32) * 0.3
    idx = np.array(g["topk_idx"], dtype=np.int32)
    w = np.array(g["topk_w"], dtype=np.float32)
    Wg, Wu, Wd = (np.stack([a, a]) for a in (Wg1, Wu1, Wd1))  # rank 0 hosts experts 0 and 1
    y = oracle.forward(x, idx, w, Wg, Wu, Wd, E=4, R=2, local_rank_begin=0, local_rank_end=1)
    ffn = brute.ffn_dense(x, Wg1, Wu1, Wd1)
    scale = np.zeros(4)
    for t, s in g["local_rank0"]["y_scale"].items():
        scale[int(t)] = s
    np.testing.assert_allclose(y, scale[:, None] * ffn, rtol=1e-6, atol=1e-7)
    assert np.all(y[2] == 0.0)


# ---------------------------------------------------------------- gate network
def test_router_logits_hand_example(oracle):
    # two tokens, three experts, worked by hand; a transposed operand or a swapped index changes every entry
    x = np.array([[1, 2, 3, 4], [0, -1, 0.5, 2]], dtype=np.float32)
    W = np.array([[1, 0, 0, 0], [0.5, 0.5, 0.5, 0.5], [-1, 2, -3, 4]], dtype=np.float32)
    want = [[1.0, 5.0, 10.0], [0.0, 0.75, 4.5]]
    assert oracle.router_logits(x, W).tolist() == want


@pytest.mark.parametrize("T,d,E", [(1, 1, 1), (7, 33, 5), (40, 257, 64)])
def test_router_logits_vs_library_matrix_product(oracle, T, d, E):
    rng = np.random.default_rng(T * 100 + d)
    x = rng.standard_normal((T, d)).astype(np.float32)
    W = rng.standard_normal((E, d)).astype(np.float32)
    ref = x.astype(np.float64) @ W.astype(np.float64).T
    got = oracle.router_logits(x, W)
    assert got.shape == (T, E)
    np.testing.assert_allclose(got, ref, rtol=0, atol=1e-12 * d)
    # unit-vector rows pick single columns of x: catches a row/column mix-up of W_r exactly
    sel = rng.integers(0, d, size=E)
    U = np.zeros((E, d), dtype=np.float32)
    U[np.arange(E), sel] = 1.0
    assert np.array_equal(oracle.router_logits(x, U), x[:, sel].astype(np.float64))


def test_router_logits_bf16_and_float_twin(oracle):
    rng = np.random.default_rng(3)
    x32 = rng.standard_normal((9, 96)).astype(np.float32)
    W32 = rng.standard_normal((6, 96)).astype(np.float32)
    xb, Wb = wl.f32_to_bf16_bits(x32), wl.f32_to_bf16_bits(W32)
    # bf16 bit patterns are widened exactly: same result as handing over the widened fp32 values
    assert np.array_equal(oracle.router_logits(xb, Wb),
                          oracle.router_logits(wl.bf16_bits_to_f32(xb), wl.bf16_bits_to_f32(Wb)))
    # the float-accumulating build stays within the textbook bound d * 2^-24 * sum |x w|
    a64, a32 = oracle.router_logits(x32, W32), oracle.router_logits(x32, W32, acc="f32")
    bound = 96 * 2.0 ** -24 * (np.abs(x32).astype(np.float64) @ np.abs(W32).astype(np.float64).T)
    assert np.all(np.abs(a64 - a32) <= bound) and np.any(a64 != a32)
    with pytest.raises(TypeError):
        oracle.router_logits(x32, Wb)


# ---------------------------------------------------------------- routing
@pytest.mark.parametrize("T,E,k", [(50, 8, 2), (33, 16, 16), (40, 5, 1), (64, 256, 8), (17, 3, 3)])
def test_route_vs_full_sort_and_full_softmax(oracle, T, E, k):
    rng = np.random.default_rng(T * 1000 + E)
    logits = rng.standard_normal((T, E)).astype(np.float32)
    logits[::3] = np.round(logits[::3] * 2) / 2  # plenty of exact ties
    idx, w = oracle.route_topk(logits, k)
    bidx, bw = brute.route_bruteforce(logits, k)
    assert np.array_equal(idx, bidx)
    np.testing.assert_allclose(w, bw, atol=2e-7)
    np.testing.assert_allclose(w.astype(np.float64).sum(axis=1), 1.0, atol=1e-6)


def test_route_special_cases(oracle):
    from scipy.special import softmax
    rng = np.random.default_rng(0)
    logits = rng.standard_normal((20, 6)).astype(np.float32)
    idx1, w1 = oracle.route_topk(logits, 1)
    assert np.array_equal(idx1[:, 0], logits.argmax(axis=1)) and np.all(w1 == 1.0)
    idxE, wE = oracle.route_topk(logits, 6)  # k = E: plain softmax, in descending-logit order
    sm = softmax(logits.astype(np.float64), axis=1)
    np.testing.assert_allclose(wE, np.take_along_axis(sm, idxE, axis=1), atol=2e-7)
    assert np.all(np.diff(np.take_along_axis(logits, idxE, axis=1), axis=1) <= 0)


def test_route_signed_zero_is_a_tie(oracle):
    logits = np.array([[-0.0, 0.0, -1.0], [0.0, -0.0, -1.0]], dtype=np.float32)
    idx, w = oracle.route_topk(logits, 2)
    assert idx.tolist() == [[0, 1], [0, 1]]
    np.testing.assert_allclose(w, 0.5)


def test_route_rejects_nonfinite(oracle):
    logits = np.array([[0.0, np.nan, 1.0]], dtype=np.float32)
    with pytest.raises(ValueError):
        oracle.route_topk(logits, 2)


# ---------------------------------------------------------------- dispatch tables
@pytest.mark.parametrize("T,E,k", [(1, 4, 2), (100, 8, 2), (257, 32, 8), (64, 4, 4), (90, 64, 1)])
def test_tables_vs_stable_argsort(oracle, T, E, k):
    rng = np.random.default_rng(E + k)
    logits = rng.standard_normal((T, E)).astype(np.float32)
    logits[:, : E // 2] -= 2.0  # skew: some experts (nearly) empty
    idx, _ = oracle.route_topk(logits, k)
    counts, offsets, perm, inv = oracle.build_tables(idx, E)
    bc, bo, bp, bi = brute.tables_bruteforce(idx, E)
    assert np.array_equal(counts, bc) and np.array_equal(offsets, bo)
    assert np.array_equal(perm, bp) and np.array_equal(inv, bi)
    # invariants: permutation, inverse, dense per-expert segments with strictly increasing token ids
    assert counts.sum() == T * k
    assert np.array_equal(np.sort(perm), np.arange(T * k))
    assert np.array_equal(perm[inv], np.arange(T * k))
    for e in range(E):
        seg = perm[offsets[e]:offsets[e + 1]]
        assert np.all(idx.ravel()[seg] == e)
        assert np.all(np.diff(seg // k) > 0)


def test_tables_empty_input(oracle):
    idx = np.zeros((0, 2), dtype=np.int32)
    counts, offsets, perm, inv = oracle.build_tables(idx, 4)
    assert counts.tolist() == [0] * 4 and offsets.tolist() == [0] * 5 and perm.size == 0


# ---------------------------------------------------------------- dedup
@pytest.mark.parametrize("T,E,k,R", [(60, 8, 2, 4), (40, 16, 4, 16), (40, 16, 4, 1), (55, 32, 8, 4), (30, 32, 32, 8),
                                     (25, 6, 1, 3)])
def test_dedup_vs_set_enumeration(oracle, T, E, k, R):
    rng = np.random.default_rng(T + R)
    idx, _ = oracle.route_topk(rng.standard_normal((T, E)).astype(np.float32), k)
    rc, ro, tok, mask, p2d = oracle.build_dedup(idx, E, R)
    brc, btok, bmask, bp2d = brute.dedup_bruteforce(idx, E, R)
    assert np.array_equal(rc, brc) and np.array_equal(tok, btok)
    assert np.array_equal(mask, bmask) and np.array_equal(p2d, bp2d)
    assert np.array_equal(ro, np.concatenate([[0], np.cumsum(rc)]))
    assert sum(bin(int(m)).count("1") for m in mask) == T * k
    if R == 1 or k == 1:
        assert ro[R] == T
    if R == E:
        assert ro[R] == T * k


@pytest.mark.parametrize("name", ["tiny", "deepseek_v3", "qwen3", "mixtral", "gpt_oss"])
def test_dedup_count_matches_closed_form_for_uniform_routing(oracle, name):
    """With iid continuous logits the top-k set is a uniform k-subset, so E[U_all]/T has a closed form."""
    cfg = wl.CONFIGS[name].scaled(router="normal", T=4096, d=8, dtype=wl.F32)
    w = wl.make_workload(cfg, weights=False)
    idx, _ = oracle.route_topk(w.logits, cfg.k)
    _, ro, *_ = oracle.build_dedup(idx, cfg.E, cfg.R)
    mean = brute.expected_unique_ranks_per_token(cfg.E, cfg.R, cfg.k)
    # per-token count lies in [1, min(k, R)]: its variance is at most (range/2)^2
    sigma = (min(cfg.k, cfg.R) - 1) / 2 / math.sqrt(cfg.T) + 1e-12
    assert abs(ro[cfg.R] / cfg.T - mean) <= 4 * sigma


def test_closed_form_values_quoted_for_the_configs():
    vals = {n: brute.expected_unique_ranks_per_token(c.E, c.R, c.k) for n, c in wl.CONFIGS.items()}
    assert abs(vals["tiny"] - 1.857) < 1e-3 and abs(vals["deepseek_v3"] - 5.295) < 1e-3
    assert abs(vals["qwen3"] - 5.339) < 1e-3 and abs(vals["mixtral"] - 2.0) < 1e-12
    assert abs(vals["gpt_oss"] - 2.754) < 1e-3
    # redundancy claim of Sec. II-B (256 experts, 32 GPUs): share of four-direction traffic that is redundant
    for k, lo in ((8, 0.40), (16, 0.44), (32, 0.46)):
        u = brute.expected_unique_ranks_per_token(256, 32, k)
        assert lo < (2 * u - 2) / (4 * u) < 0.5


# ---------------------------------------------------------------- forward
def _draw(cfg, seed=0):
    w = wl.make_workload(cfg)
    return w


def test_forward_single_expert_is_dense_ffn(oracle):
    """E = 1, k = 1: the layer is one dense SwiGLU FFN (catches transposed weights, wrong activation)."""
    cfg = small_cfg(E=1, k=1, R=1, local_rank_begin=0, local_rank_end=1, T=9, d=10, f=14)
    w = _draw(cfg)
    idx, tw = oracle.route_topk(w.logits, 1)
    y = oracle.forward(w.x, idx, tw, w.W_gate, w.W_up, w.W_down, 1, 1, 0, 1)
    np.testing.assert_allclose(y, brute.ffn_dense(w.x, w.W_gate[0], w.W_up[0], w.W_down[0]), rtol=1e-9, atol=1e-11)


@pytest.mark.parametrize("lr", [(0, 4), (1, 3), (3, 4)])
def test_forward_vs_table_free_bruteforce(oracle, lr):
    cfg = small_cfg(local_rank_begin=lr[0], local_rank_end=lr[1])
    w = _draw(cfg)
    idx, tw = oracle.route_topk(w.logits, cfg.k)
    y = oracle.forward(w.x, idx, tw, w.W_gate, w.W_up, w.W_down, cfg.E, cfg.R, *lr)
    yb = brute.forward_bruteforce(w.x, w.logits, cfg.k, w.W_gate, w.W_up, w.W_down, cfg.E, cfg.R, *lr)
    np.testing.assert_allclose(y, yb, rtol=1e-6, atol=1e-7)  # topk_w is stored in fp32


def test_forward_identical_experts_all_local_is_dense_ffn(oracle):
    cfg = small_cfg(local_rank_begin=0, local_rank_end=4)
    w = _draw(cfg)
    Wg, Wu, Wd = (np.repeat(a[:1], cfg.E, axis=0) for a in (w.W_gate, w.W_up, w.W_down))
    idx, tw = oracle.route_topk(w.logits, cfg.k)
    y = oracle.forward(w.x, idx, tw, Wg, Wu, Wd, cfg.E, cfg.R, 0, 4)
    np.testing.assert_allclose(y, brute.ffn_dense(w.x, Wg[0], Wu[0], Wd[0]), rtol=1e-6, atol=1e-7)


def test_forward_algebraic_properties(oracle):
    cfg = small_cfg(T=40, local_rank_begin=1, local_rank_end=2)
    w = _draw(cfg)
    idx, tw = oracle.route_topk(w.logits, cfg.k)
    args = (cfg.E, cfg.R, cfg.local_rank_begin, cfg.local_rank_end)
    y = oracle.forward(w.x, idx, tw, w.W_gate, w.W_up, w.W_down, *args)
    # linear in W_down
    y3 = oracle.forward(w.x, idx, tw, w.W_gate, w.W_up, (w.W_down * np.float32(4.0)), *args)
    np.testing.assert_allclose(y3, 4.0 * y, rtol=1e-12)
    # zero up-projection or zero gate (silu(0) = 0) kills the output
    assert np.all(oracle.forward(w.x, idx, tw, w.W_gate, np.zeros_like(w.W_up), w.W_down, *args) == 0)
    assert np.all(oracle.forward(w.x, idx, tw, np.zeros_like(w.W_gate), w.W_up, w.W_down, *args) == 0)
    # token-permutation equivariance
    p = np.random.default_rng(1).permutation(cfg.T)
    yp = oracle.forward(w.x[p], idx[p], tw[p], w.W_gate, w.W_up, w.W_down, *args)
    np.testing.assert_array_equal(yp, y[p])
    # token subset == rows of the full result; tokens without a local slot are exactly zero
    sel = np.array([5, 0, 17], dtype=np.int32)
    ys = oracle.forward(w.x, idx, tw, w.W_gate, w.W_up, w.W_down, *args, tokens=sel)
    np.testing.assert_array_equal(ys, y[sel])
    epr = cfg.E // cfg.R
    local = (idx // epr >= cfg.local_rank_begin) & (idx // epr < cfg.local_rank_end)
    assert np.all(y[~local.any(axis=1)] == 0) and (~local.any(axis=1)).any()
    # swapping gate and up changes the result (silu is applied to the gate branch only)
    ysw = oracle.forward(w.x, idx, tw, w.W_up, w.W_gate, w.W_down, *args)
    assert np.abs(ysw - y).max() > 1e-3


def test_forward_bf16_inputs_are_widened_exactly(oracle):
    cfg = small_cfg(dtype=wl.BF16)
    w = _draw(cfg)
    idx, tw = oracle.route_topk(w.logits, cfg.k)
    args = (cfg.E, cfg.R, cfg.local_rank_begin, cfg.local_rank_end)
    y16 = oracle.forward(w.x, idx, tw, w.W_gate, w.W_up, w.W_down, *args)
    y32 = oracle.forward(*(wl.bf16_bits_to_f32(a) for a in (w.x,)), idx, tw,
                         *(wl.bf16_bits_to_f32(a) for a in (w.W_gate, w.W_up, w.W_down)), *args)
    np.testing.assert_array_equal(y16, y32)


def test_forward_float_accumulation_twin(oracle):
    """fp32-accumulating build vs fp64-accumulating build: bounds the oracle's own rounding error."""
    cfg = small_cfg(T=16, d=256, f=128)
    w = _draw(cfg)
    idx, tw = oracle.route_topk(w.logits, cfg.k)
    args = (cfg.E, cfg.R, cfg.local_rank_begin, cfg.local_rank_end)
    y64 = oracle.forward(w.x, idx, tw, w.W_gate, w.W_up, w.W_down, *args, acc="f64")
    y32 = oracle.forward(w.x, idx, tw, w.W_gate, w.W_up, w.W_down, *args, acc="f32")
    assert np.abs(y64 - y32).max() <= 1e-5 * math.sqrt(cfg.d) * np.abs(y64).max()
    assert np.abs(y64 - y32).max() > 0


def test_bf16_rounding_helper_is_rne():
    import struct

    def bits(v):
        return struct.unpack("<I", struct.pack("<f", v))[0]

    vals = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, 1.0 + 2 ** -8 + 2 ** -20, -2.5, 0.0, 3.0e38], dtype=np.float32)
    got = wl.f32_to_bf16_bits(vals)
    # 1 + 2^-8 is a tie -> even (1.0); 1 + 3*2^-8 is a tie -> even (1 + 2^-6 = 0x3F82)
    assert got[0] == 0x3F80 and got[1] == 0x3F80 and got[2] == 0x3F82 and got[3] == 0x3F81
    assert got[4] == bits(-2.5) >> 16 and got[5] == 0
    back = wl.bf16_bits_to_f32(got)
    assert np.all(np.abs(back[:5] - vals[:5]) <= np.abs(vals[:5]) * 2 ** -8)


# ---------------------------------------------------------------- FP8 (E4M3) operands
def test_fp8_code_values_match_the_format_definition_and_a_library(oracle):
    """All 256 codes: against the closed form of the format and against PyTorch's CPU decoding."""
    import torch
    codes = np.arange(256, dtype=np.uint8)
    got = oracle.fp8_decode(codes)
    np.testing.assert_array_equal(got, brute.e4m3_values_closed_form())
    lib = torch.from_numpy(codes).view(torch.float8_e4m3fn).to(torch.float32).numpy().astype(np.float64)
    np.testing.assert_array_equal(got, lib)
    # the format's landmarks (OCP 8-bit floating point specification, E4M3 column of its table of encodings)
    assert got[0x7E] == 448.0 and got[0x08] == 2.0 ** -6 and got[0x07] == 0.875 * 2.0 ** -6 and got[0x01] == 2.0 ** -9
    assert np.isnan(got[0x7F]) and np.isnan(got[0xFF]) and got[0x38] == 1.0 and got[0xB8] == -1.0


def test_fp8_conversion_is_round_to_nearest_even_and_saturates(oracle):
    vals = brute.e4m3_values_closed_form()
    finite = np.array([c for c in range(256) if not math.isnan(vals[c])], dtype=np.uint8)
    # every code value converts to its own code (-0 and +0 keep their sign)
    np.testing.assert_array_equal(oracle.fp8_encode(vals[finite].astype(np.float32)), finite)
    # midpoints of neighbouring positive values go to the code with the even mantissa bit
    pos = np.arange(0, 0x7E, dtype=np.uint8)
    mid = ((vals[pos] + vals[pos + 1]) / 2).astype(np.float32)  # exact in fp32
    want = np.where(pos % 2 == 0, pos, pos + 1).astype(np.uint8)
    np.testing.assert_array_equal(oracle.fp8_encode(mid), want)
    np.testing.assert_array_equal(oracle.fp8_encode(-mid), want | 0x80)
    # just off the midpoints: the nearer neighbour
    np.testing.assert_array_equal(oracle.fp8_encode(np.nextafter(mid, np.float32(np.inf))), pos + 1)
    np.testing.assert_array_equal(oracle.fp8_encode(np.nextafter(mid, np.float32(0))), pos)
    # saturation and NaN
    big = np.array([448.0, 449.0, 464.0, 480.0, 1e30, np.inf], dtype=np.float32)
    np.testing.assert_array_equal(oracle.fp8_encode(big), np.full(6, 0x7E, dtype=np.uint8))
    np.testing.assert_array_equal(oracle.fp8_encode(-big), np.full(6, 0xFE, dtype=np.uint8))
    assert oracle.fp8_encode(np.array([np.nan], dtype=np.float32))[0] & 0x7F == 0x7F
    # random values, several magnitudes: same codes as the library's conversion
    rng = np.random.default_rng(5)
    v = np.concatenate([rng.standard_normal(20000) * s for s in (1e-3, 0.02, 1.0, 30.0, 200.0)]).astype(np.float32)
    _, lib_codes = brute.e4m3_round_library(v)
    np.testing.assert_array_equal(oracle.fp8_encode(v), lib_codes)


def test_fp8_quantize_rows_and_columns(oracle):
    rng = np.random.default_rng(6)
    a = (rng.standard_normal((7, 33)) * rng.uniform(0.01, 50, size=(7, 1))).astype(np.float32)
    a[3] = 0.0  # an all-zero group
    codes, scales = oracle.fp8_quantize(a, axis=-1)
    amax = np.abs(a).max(axis=1)
    np.testing.assert_array_equal(scales, np.where(amax > 0, amax / np.float32(448.0), np.float32(1.0)))
    _, lib_codes = brute.e4m3_round_library(a / scales[:, None])
    np.testing.assert_array_equal(codes, lib_codes)
    assert np.all(codes[3] == 0) and scales[3] == 1.0
    # the largest element of a group lands on +-448; the others within half a step (2^-4 relative for normal numbers)
    top = np.abs(a).argmax(axis=1)
    assert all((codes[r, top[r]] & 0x7F) == 0x7E for r in range(7) if r != 3)
    back = oracle.fp8_decode(codes) * scales[:, None]
    normal = np.abs(a) >= scales[:, None] * 2.0 ** -6
    assert np.all(np.abs(back - a)[normal] <= np.abs(a)[normal] * 2.0 ** -4 * (1 + 1e-6))
    assert np.all(np.abs(back - a)[~normal] <= scales[:, None].repeat(33, 1)[~normal] * 2.0 ** -10 * (1 + 1e-6))
    # columns of a matrix = rows of its transpose, also with a batch dimension
    b = rng.standard_normal((3, 12, 5)).astype(np.float32)
    cc, sc = oracle.fp8_quantize(b, axis=-2)
    for e in range(3):
        cr, sr = oracle.fp8_quantize(np.ascontiguousarray(b[e].T), axis=-1)
        np.testing.assert_array_equal(cc[e], cr.T)
        np.testing.assert_array_equal(sc[e], sr)


def test_fp8_forward_single_expert_vs_library_conversions(oracle):
    """E = 1, k = 1, weight 1: the FP8 layer written with PyTorch's conversions and float64 library products."""
    cfg = small_cfg(E=1, k=1, R=1, local_rank_begin=0, local_rank_end=1, T=12, d=24, f=20)
    w = _draw(cfg)
    idx, tw = oracle.route_topk(w.logits, 1)
    s_h = np.array([0.013], dtype=np.float32)
    y = oracle.forward_fp8(w.x, idx, tw, w.W_gate, w.W_up, w.W_down, s_h, 1, 1, 0, 1)
    want = brute.ffn_dense_fp8(w.x, w.W_gate[0], w.W_up[0], w.W_down[0], s_h[0])
    np.testing.assert_allclose(y, want, rtol=1e-9, atol=1e-12)
    # a scale for h that is far too small saturates every h to +-448 s_h: the layer still matches
    s_h = np.array([1e-6], dtype=np.float32)
    y = oracle.forward_fp8(w.x, idx, tw, w.W_gate, w.W_up, w.W_down, s_h, 1, 1, 0, 1)
    np.testing.assert_allclose(y, brute.ffn_dense_fp8(w.x, w.W_gate[0], w.W_up[0], w.W_down[0], s_h[0]),
                               rtol=1e-9, atol=1e-15)


def test_fp8_forward_properties(oracle):
    cfg = small_cfg(T=40, local_rank_begin=1, local_rank_end=3)
    w = _draw(cfg)
    idx, tw = oracle.route_topk(w.logits, cfg.k)
    El = w.W_gate.shape[0]
    s_h = (0.01 * (1 + np.arange(El) % 3)).astype(np.float32)
    args = (cfg.E, cfg.R, 1, 3)
    y = oracle.forward_fp8(w.x, idx, tw, w.W_gate, w.W_up, w.W_down, s_h, *args)
    # close to the unquantised layer (three roundings of 2^-4 relative per product, averaged over the sums) ...
    y0 = oracle.forward(w.x, idx, tw, w.W_gate, w.W_up, w.W_down, *args)
    rel = np.linalg.norm(y - y0) / np.linalg.norm(y0)
    assert 1e-3 < rel < 0.1
    # ... per-column scales absorb powers of two exactly: scaling W_down's columns scales y's columns
    factors = (2.0 ** (np.arange(w.W_down.shape[2]) % 7 - 3)).astype(np.float32)
    y2 = oracle.forward_fp8(w.x, idx, tw, w.W_gate, w.W_up, w.W_down * factors[None, None, :], s_h, *args)
    np.testing.assert_array_equal(y2, y * factors[None, :].astype(np.float64))
    y4 = oracle.forward_fp8(w.x, idx, tw, w.W_gate, w.W_up * np.float32(4), w.W_down, s_h * np.float32(4), *args)
    # u scaled by 4 and s_h by 4: the same h codes, so y is exactly 4 y
    np.testing.assert_array_equal(y4, 4.0 * y)
    # tokens without a local slot give zero rows; a token subset gives the same rows
    sub = np.array([5, 0, 17], dtype=np.int32)
    np.testing.assert_array_equal(oracle.forward_fp8(w.x, idx, tw, w.W_gate, w.W_up, w.W_down, s_h, *args, tokens=sub),
                                  y[sub])
    epr = cfg.E // cfg.R
    none_local = ~((idx >= epr) & (idx < 3 * epr)).any(axis=1)
    assert np.all(y[none_local] == 0)


def test_fp8_forward_vs_per_slot_bruteforce(oracle):
    """Several experts and ranks: every (token, local slot) as its own one-row dense FP8 FFN (a token's scale
    depends on its own row only), weighted and summed in slot order."""
    cfg = small_cfg(T=24, local_rank_begin=1, local_rank_end=3)
    w = _draw(cfg)
    idx, tw = oracle.route_topk(w.logits, cfg.k)
    El = w.W_gate.shape[0]
    epr = cfg.E // cfg.R
    s_h = (0.004 * (1 + np.arange(El))).astype(np.float32)
    y = oracle.forward_fp8(w.x, idx, tw, w.W_gate, w.W_up, w.W_down, s_h, cfg.E, cfg.R, 1, 3)
    want = np.zeros_like(y)
    for t in range(cfg.T):
        for j in range(cfg.k):
            le = int(idx[t, j]) - epr
            if 0 <= le < El:
                want[t] += float(tw[t, j]) * brute.ffn_dense_fp8(w.x[t:t + 1], w.W_gate[le], w.W_up[le], w.W_down[le],
                                                                 s_h[le])[0]
    np.testing.assert_allclose(y, want, rtol=1e-9, atol=1e-12)


# ---------------------------------------------------------------- gate variants (sigmoid gate, selection-only bias)
def _grid_logits(rng, T, E):
    """Logits on a grid of 1/4 and biases on a grid of 1/64: selection values are either exactly equal or far
    apart (no rounding can reorder them), so the picks have one right answer."""
    return (rng.integers(-12, 13, size=(T, E)) / 4.0).astype(np.float32)


@pytest.mark.parametrize("gate", [0, 1])
def test_gate_variants_vs_full_sort(oracle, gate):
    rng = np.random.default_rng(40 + gate)
    T, E, k = 60, 24, 5
    logits = _grid_logits(rng, T, E)
    bias = (rng.integers(-8, 9, size=E) / 64.0).astype(np.float32)
    idx, w, sel = oracle.route_topk_gate(logits, k, gate, bias)
    l64 = logits.astype(np.float64)
    s64 = 1.0 / (1.0 + np.exp(-l64))
    base = l64 if gate == 0 else s64
    want_sel = base + bias[None, :].astype(np.float64)
    np.testing.assert_allclose(sel, want_sel, rtol=3e-7, atol=1e-7)
    # stable sort of the fp32 selection values = pick order with ties to the lower index
    order = np.argsort(-sel.astype(np.float64), axis=1, kind="stable")[:, :k]
    np.testing.assert_array_equal(idx, order)
    # on this grid, fp32 rounding cannot have reordered anything: same picks from the exact values
    gaps = np.abs(want_sel[:, :, None] - want_sel[:, None, :])
    assert np.all((gaps == 0) | (gaps > 1e-4))
    np.testing.assert_array_equal(idx, np.argsort(-np.round(want_sel, 9), axis=1, kind="stable")[:, :k])
    # weights: from the logits alone (the bias steers the selection only)
    picked = np.take_along_axis(l64, idx.astype(np.int64), axis=1)
    if gate == 0:
        p = np.exp(picked - picked.max(axis=1, keepdims=True))
    else:
        p = 1.0 / (1.0 + np.exp(-picked))
    np.testing.assert_allclose(w, p / p.sum(axis=1, keepdims=True), rtol=2e-7)
    np.testing.assert_allclose(w.sum(axis=1), 1.0, atol=1e-6)


def test_gate_variants_special_cases(oracle):
    rng = np.random.default_rng(43)
    logits = rng.standard_normal((50, 16)).astype(np.float32)
    idx0, w0 = oracle.route_topk(logits, 4)
    # softmax gate without a bias is the plain routing
    idx, w, _ = oracle.route_topk_gate(logits, 4, 0, None)
    np.testing.assert_array_equal(idx, idx0)
    np.testing.assert_allclose(w, w0, rtol=1e-6)
    # the sigmoid is monotone: same picks without a bias (these logits are far from its saturation), other weights
    idx, w, _ = oracle.route_topk_gate(logits, 4, 1, None)
    np.testing.assert_array_equal(idx, idx0)
    assert np.abs(w - w0).max() > 1e-3
    # a large bias forces an expert into the first slot and leaves its weight a function of its logit only
    bias = np.zeros(16, dtype=np.float32)
    bias[11] = 100.0
    for gate in (0, 1):
        idx, w, _ = oracle.route_topk_gate(logits, 4, gate, bias)
        assert np.all(idx[:, 0] == 11)
        l = np.take_along_axis(logits.astype(np.float64), idx.astype(np.int64), axis=1)
        p = np.exp(l - l.max(axis=1, keepdims=True)) if gate == 0 else 1.0 / (1.0 + np.exp(-l))
        np.testing.assert_allclose(w, p / p.sum(axis=1, keepdims=True), rtol=2e-7)
    # k = E: every expert, in descending order of the selection value; sigmoid saturation makes exact ties
    sat = np.array([[30.0, 40.0, -1.0, 35.0]], dtype=np.float32)
    idx, w, sel = oracle.route_topk_gate(sat, 4, 1, None)
    assert sel[0, 0] == sel[0, 1] == sel[0, 3] == 1.0
    np.testing.assert_array_equal(idx[0], [0, 1, 3, 2])
    with pytest.raises(ValueError):
        oracle.route_topk_gate(np.array([[0.0, np.inf]], dtype=np.float32), 1, 1, None)


# ---------------------------------------------------------------- backward pass
def _loss(oracle, w, idx, tw, x, Wg, Wu, Wd, dy, cfg, lr):
    """L = sum(y * dy): its gradients are what the backward pass returns for the incoming gradient dy."""
    y = oracle.forward(x, idx, tw, Wg, Wu, Wd, cfg.E, cfg.R, *lr)
    return float((y * dy.astype(np.float64)).sum())


def test_backward_matches_finite_differences_of_the_forward(oracle):
    """Central differences of the (pinned) forward in float32-representable steps: every output of the backward."""
    cfg = small_cfg(T=7, d=6, f=5, E=4, k=2, R=2, local_rank_begin=0, local_rank_end=2, dtype=wl.F32)
    w = _draw(cfg)
    lr = (0, 2)
    idx, tw = oracle.route_topk(w.logits, cfg.k)
    rng = np.random.default_rng(3)
    dy = rng.standard_normal((cfg.T, cfg.d)).astype(np.float32)
    dx, dw = oracle.backward_tokens(w.x, dy, idx, tw, w.W_gate, w.W_up, w.W_down, cfg.E, cfg.R, *lr)
    eps = np.float32(2.0 ** -7)

    def fd(arr, pos):
        a, b = arr.copy(), arr.copy()
        a[pos] += eps
        b[pos] -= eps
        return a, b, float(a[pos] - b[pos])

    def check(got, arr, make_args, n_probe=12, tol=2e-3):
        for _ in range(n_probe):
            pos = tuple(int(rng.integers(0, s)) for s in arr.shape)
            a, b, step = fd(arr, pos)
            want = (_loss(oracle, w, idx, tw, *make_args(a), dy, cfg, lr)
                    - _loss(oracle, w, idx, tw, *make_args(b), dy, cfg, lr)) / step
            assert abs(got(pos) - want) <= tol * (1 + abs(want)), (pos, got(pos), want)

    check(lambda p: dx[p], w.x, lambda a: (a, w.W_gate, w.W_up, w.W_down))
    grads = [oracle.backward_weights(w.x, dy, idx, tw, w.W_gate, w.W_up, w.W_down, cfg.E, cfg.R, *lr, le)
             for le in range(cfg.E)]
    check(lambda p: grads[p[0]][0][p[1], p[2]], w.W_gate, lambda a: (w.x, a, w.W_up, w.W_down))
    check(lambda p: grads[p[0]][1][p[1], p[2]], w.W_up, lambda a: (w.x, w.W_gate, a, w.W_down))
    check(lambda p: grads[p[0]][2][p[1], p[2]], w.W_down, lambda a: (w.x, w.W_gate, w.W_up, a))
    # gate weights: the forward is linear in them, so a difference of any size is exact
    for _ in range(8):
        t, j = int(rng.integers(0, cfg.T)), int(rng.integers(0, cfg.k))
        a, b = tw.copy(), tw.copy()
        a[t, j] += 0.25
        b[t, j] -= 0.25
        want = (_loss(oracle, w, idx, a, w.x, w.W_gate, w.W_up, w.W_down, dy, cfg, lr)
                - _loss(oracle, w, idx, b, w.x, w.W_gate, w.W_up, w.W_down, dy, cfg, lr)) / 0.5
        assert abs(dw[t, j] - want) <= 1e-9 * (1 + abs(want))


def test_backward_local_slots_only_and_ranges(oracle):
    cfg = small_cfg(T=30, local_rank_begin=1, local_rank_end=3)
    w = _draw(cfg)
    lr = (1, 3)
    idx, tw = oracle.route_topk(w.logits, cfg.k)
    rng = np.random.default_rng(4)
    dy = wl.f32_to_bf16_bits(rng.standard_normal((cfg.T, cfg.d)).astype(np.float32)) if w.x.dtype == np.uint16 \
        else rng.standard_normal((cfg.T, cfg.d)).astype(np.float32)
    dx, dw = oracle.backward_tokens(w.x, dy, idx, tw, w.W_gate, w.W_up, w.W_down, cfg.E, cfg.R, *lr)
    epr = cfg.E // cfg.R
    local = (idx >= epr) & (idx < 3 * epr)
    assert np.all(dw[~local] == 0) and np.all(dw[local] != 0)
    assert np.all(dx[~local.any(axis=1)] == 0)
    sub = np.array([9, 2, 21], dtype=np.int32)
    dxs, dws = oracle.backward_tokens(w.x, dy, idx, tw, w.W_gate, w.W_up, w.W_down, cfg.E, cfg.R, *lr, tokens=sub)
    np.testing.assert_array_equal(dxs, dx[sub])
    np.testing.assert_array_equal(dws, dw[sub])
    # a hidden-index range of the weight gradients is the slice of the whole
    full = oracle.backward_weights(w.x, dy, idx, tw, w.W_gate, w.W_up, w.W_down, cfg.E, cfg.R, *lr, 1)
    part = oracle.backward_weights(w.x, dy, idx, tw, w.W_gate, w.W_up, w.W_down, cfg.E, cfg.R, *lr, 1, 3, 9)
    np.testing.assert_array_equal(part[0], full[0][:, 3:9])
    np.testing.assert_array_equal(part[1], full[1][:, 3:9])
    np.testing.assert_array_equal(part[2], full[2][3:9, :])
    # dw = <o, dy>: the unweighted expert output against the incoming gradient (forward with weight 1 on one slot)
    t = int(np.nonzero(local.any(axis=1))[0][0])
    j = int(np.nonzero(local[t])[0][0])
    one = np.zeros_like(tw)
    one[t, j] = 1.0
    o = oracle.forward(w.x, idx, one, w.W_gate, w.W_up, w.W_down, cfg.E, cfg.R, *lr, tokens=np.array([t], np.int32))[0]
    dyf = wl.bf16_bits_to_f32(dy) if dy.dtype == np.uint16 else dy
    np.testing.assert_allclose(dw[t, j], float((o * dyf[t].astype(np.float64)).sum()), rtol=1e-10)


def test_route_backward_vs_finite_differences_and_closed_form(oracle):
    rng = np.random.default_rng(50)
    T, E, k = 9, 12, 4
    logits = rng.standard_normal((T, E)).astype(np.float32)
    idx, w = oracle.route_topk(logits, k)
    dw = rng.standard_normal((T, k))
    dl = oracle.route_backward(logits, idx, dw)
    # closed form through the full Jacobian of a softmax over the picked logits (NumPy, float64)
    for t in range(T):
        l = logits[t, idx[t]].astype(np.float64)
        p = np.exp(l - l.max())
        p /= p.sum()
        J = np.diag(p) - np.outer(p, p)
        want = np.zeros(E)
        want[idx[t]] = J @ dw[t]
        np.testing.assert_allclose(dl[t], want, rtol=1e-12, atol=1e-15)
    # central differences of the routing weights themselves (picks unchanged for a small step)
    eps = np.float32(2.0 ** -9)
    for _ in range(10):
        t, e = int(rng.integers(0, T)), int(rng.integers(0, E))
        a, b = logits.copy(), logits.copy()
        a[t, e] += eps
        b[t, e] -= eps
        ia, wa = oracle.route_topk(a, k)
        ib, wb = oracle.route_topk(b, k)
        if not (np.array_equal(ia[t], idx[t]) and np.array_equal(ib[t], idx[t])):
            continue
        want = float(((wa[t].astype(np.float64) - wb[t].astype(np.float64)) * dw[t]).sum()) / float(a[t, e] - b[t, e])
        assert abs(dl[t, e] - want) <= 2e-4 * (1 + abs(want))  # the weights are stored in fp32
    # the gradients of a row sum to zero (the weights sum to one) and vanish off the picks
    np.testing.assert_allclose(dl.sum(axis=1), 0.0, atol=1e-14)
    mask = np.zeros((T, E), bool)
    np.put_along_axis(mask, idx.astype(np.int64), True, axis=1)
    assert np.all(dl[~mask] == 0)


def test_fp8_landmarks_from_the_format_specification(oracle):
    with open(os.path.join(os.path.dirname(__file__), "golden", "e4m3_landmarks.json")) as f:
        gold = json.load(f)
    codes = np.array([int(c, 16) for c in gold["codes"]], dtype=np.uint8)
    np.testing.assert_array_equal(oracle.fp8_decode(codes), np.array(list(gold["codes"].values())))
    assert np.isnan(oracle.fp8_decode(np.array([int(c, 16) for c in gold["nan_codes"]], dtype=np.uint8))).all()
    for case in gold["round_to_nearest_even"]:
        got = int(oracle.fp8_encode(np.array([case["value"]], dtype=np.float32))[0])
        assert got == int(case["code"], 16), case


# ---------------------------------------------------------------- load models of the synthetic routers (inputs only)
@pytest.mark.parametrize("std", [0.01, 0.032, 0.05])
def test_loadstd_router_spreads_the_load_as_requested(oracle, std):
    """The training-load router: the pairs an expert receives follow its drawn share p_e (top-k of ln p + Gumbel
    noise = draws without replacement in proportion to p), so the measured spread of the load grows with the
    requested standard deviation and the measured shares correlate with the drawn ones."""
    cfg = wl.CONFIGS["table1_m"].scaled(router="loadstd", load_std=std, T=8192)
    w = wl.make_workload(cfg, weights=False)
    idx, _ = oracle.route_topk(w.logits, cfg.k)
    share = np.bincount(idx.ravel(), minlength=cfg.E) / idx.size
    p = wl.expert_load_fractions(cfg.E, std, np.random.SeedSequence(cfg.seed).spawn(7)[2])
    assert abs(p.sum() - 1) < 1e-12 and p.min() > 0
    cv_want = std / 0.125
    cv_got = share.std() / share.mean()
    assert 0.6 * cv_want < cv_got < 1.3 * cv_want + 0.03, (cv_want, cv_got)
    assert np.corrcoef(share, p)[0, 1] > 0.8  # 512 pairs per expert: a few per cent of sampling noise


def test_hot_rank_router_puts_nearly_all_pairs_on_rank_zero(oracle):
    cfg = wl.CONFIGS["deepseek_v3"].scaled(router="zipf_hot", T=1024)
    w = wl.make_workload(cfg, weights=False)
    idx, _ = oracle.route_topk(w.logits, cfg.k)
    on_rank0 = (idx // cfg.epr == 0).mean()
    assert on_rank0 > 0.85
