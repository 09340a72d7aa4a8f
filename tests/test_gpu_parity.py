"""GPU parity: every step of the hot path, called through the C ABI, against the CPU oracle on the same seeded
inputs.  Integer tables bit-exact; routing weights |err| <= 1e-6; y within the stated tolerance."""
import numpy as np
import pytest

import gpu_util as G
from paper_2605_05607_amd import binding as B
from paper_2605_05607_amd import layer as L
from paper_2605_05607_amd import workloads as wl

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)


def cfg_of(**kw):
    base = dict(name="t", T=300, d=128, f=192, E=16, k=4, R=4, local_rank_begin=1, local_rank_end=3, dtype=wl.BF16,
                router="normal", seed=11)
    base.update(kw)
    return wl.MoEConfig(**base)


# scaled-down layers with the structure of the five named ones: several M tiles per expert, ragged tails,
# empty experts (zipf), all-local and one-rank-local, column and reduction tails
SMALL = {
    "tiny_f32": wl.CONFIGS["tiny"],
    "deepseek_like": cfg_of(T=700, d=448, f=320, E=64, k=8, R=8, local_rank_begin=0, local_rank_end=1,
                            router="zipf", seed=21),
    "qwen_like": cfg_of(T=900, d=256, f=192, E=32, k=8, R=8, local_rank_begin=2, local_rank_end=3, seed=22),
    "mixtral_like": cfg_of(T=520, d=256, f=896, E=8, k=2, R=8, local_rank_begin=0, local_rank_end=8, seed=23),
    "gpt_oss_like": cfg_of(T=1100, d=360, f=360, E=32, k=4, R=4, local_rank_begin=0, local_rank_end=1,
                           router="forced", seed=24),
    "f32_ragged": cfg_of(T=130, d=72, f=88, E=6, k=3, R=3, local_rank_begin=1, local_rank_end=3, dtype=wl.F32, seed=25),
    "k_tail_bf16": cfg_of(T=77, d=72, f=40, E=4, k=2, R=2, local_rank_begin=0, local_rank_end=2, seed=26),
    # the wider top-k columns of the evaluation's model table (16 and 32 picks): many slots per token on one rank
    "table1_like_k16": cfg_of(T=400, d=256, f=128, E=64, k=16, R=8, local_rank_begin=3, local_rank_end=4, seed=27),
    "table1_like_k32": cfg_of(T=260, d=192, f=64, E=64, k=32, R=8, local_rank_begin=0, local_rank_end=2, seed=28),
}


# ---------------------------------------------------------------- routing + tables
@pytest.mark.parametrize("T,E,k,R", [(1, 4, 2, 2), (63, 8, 2, 4), (64, 8, 8, 8), (257, 256, 8, 8), (1000, 128, 4, 4),
                                     (300, 16, 1, 16), (129, 32, 32, 4), (200, 6, 3, 1), (4096, 256, 8, 8),
                                     (90, 4096, 5, 64), (70, 12, 7, 3), (150, 4096, 3, 4096),
                                     (5000, 48, 6, 8), (777, 512, 8, 8), (333, 65, 9, 5), (2100, 640, 8, 8)])
def test_route_and_tables_bit_exact(oracle, T, E, k, R):
    say(f"route/tables T={T} E={E} k={k} R={R}")
    rng = np.random.default_rng(T * 7 + E)
    logits = rng.standard_normal((T, E)).astype(np.float32)
    logits[::5] = np.round(logits[::5] * 2) / 2      # exact ties
    logits[1::7, : max(1, E // 3)] -= 3.0             # skew: empty experts
    if T > 2:
        logits[2, :2] = (-0.0, 0.0)
    cfg = cfg_of(T=T, E=E, k=k, R=R, d=8, f=8, local_rank_begin=0, local_rank_end=R)
    lay, got = G.run_tables(cfg, logits)
    G.assert_tables_equal(got, oracle, logits, cfg)


@pytest.mark.parametrize("name", ["tiny", "deepseek_v3", "qwen3", "mixtral", "gpt_oss", "table1_s", "table1_m"])
def test_route_and_tables_full_size_configs(oracle, name):
    say(f"route/tables full size {name}")
    cfg = wl.CONFIGS[name]
    w = wl.make_workload(cfg, weights=False)
    lay, got = G.run_tables(cfg, w.logits)
    G.assert_tables_equal(got, oracle, w.logits, cfg)
    # properties that hold at any size
    assert got["counts"].sum() == cfg.T * cfg.k
    assert np.array_equal(np.sort(got["perm"]), np.arange(cfg.T * cfg.k))


def test_tables_empty_layer():
    import torch
    cfg = cfg_of(T=0, d=8, f=8)
    lay = L.MoELayer(cfg)
    lay.tables.counts.fill_(7)
    lay.tables.offsets.fill_(7)
    lay.tables.rank_offsets.fill_(7)
    lay.route(lay.topk_w)  # any non-null pointer; T = 0 touches nothing
    lay.build_dispatch()
    torch.cuda.synchronize()
    assert lay.tables.counts.abs().sum().item() == 0 and lay.tables.offsets.abs().sum().item() == 0
    assert lay.tables.rank_offsets.abs().sum().item() == 0
    lay.load_weights(*(np.zeros(sh, np.uint16) for sh in ((cfg.E_loc, 8, 8),) * 3))
    lay.forward(lay.y)
    torch.cuda.synchronize()


# ---------------------------------------------------------------- forward, whole output
def run_forward(cfg, oracle, tokens=None):
    import torch
    w = wl.make_workload(cfg)
    lay = L.MoELayer(cfg)
    lay.load_weights(w.W_gate, w.W_up, w.W_down)
    x = L.to_device(w.x)
    lg = L.to_device(w.logits)
    lay.y.fill_(float("nan"))  # every row has to be written by this call, whichever kernel owns it
    lay.step(lg, x)
    torch.cuda.synchronize()
    got = G.tables_to_host(lay)
    idx, tw = G.assert_tables_equal(got, oracle, w.logits, cfg)
    y = lay.y_host()
    ref = oracle.forward(w.x, idx, tw, w.W_gate, w.W_up, w.W_down, cfg.E, cfg.R, cfg.local_rank_begin,
                         cfg.local_rank_end, tokens=tokens)
    return w, lay, x, lg, idx, tw, y, ref


@pytest.mark.parametrize("name", list(SMALL))
def test_forward_matches_oracle_small(oracle, name):
    cfg = SMALL[name]
    say(f"forward small {name}: T={cfg.T} d={cfg.d} f={cfg.f} E={cfg.E} k={cfg.k}")
    w, lay, x, lg, idx, tw, y, ref = run_forward(cfg, oracle)
    mx, mean = G.check_y(y, ref, cfg.dtype)
    say(f"  max rel {mx:.2e} mean rel {mean:.2e}")
    epr = cfg.epr
    local = (idx // epr >= cfg.local_rank_begin) & (idx // epr < cfg.local_rank_end)
    assert np.all(y[~local.any(axis=1)] == 0)


@pytest.mark.parametrize("kw", [dict(T=1), dict(k=1), dict(E=4, k=4, R=2, local_rank_begin=0, local_rank_end=2),
                                dict(R=1, local_rank_begin=0, local_rank_end=1),
                                dict(R=16, local_rank_begin=3, local_rank_end=4),
                                dict(T=129, E=2, k=1, R=2, local_rank_begin=1, local_rank_end=2),
                                dict(T=257, E=1, k=1, R=1, local_rank_begin=0, local_rank_end=1, d=64, f=64),
                                # many local experts: the tile table's per-expert scans, its rank sort (up to 1024
                                # experts) and the expert-order fallback beyond
                                dict(T=600, E=512, k=4, R=1, local_rank_begin=0, local_rank_end=1, d=64, f=64),
                                dict(T=900, E=2048, k=3, R=2, local_rank_begin=0, local_rank_end=2, d=64, f=64,
                                     router="zipf"),
                                dict(T=3000, E=4096, k=2, R=4096, local_rank_begin=100, local_rank_end=1400, d=32,
                                     f=32)])
def test_forward_edge_shapes(oracle, kw):
    cfg = cfg_of(**kw)
    say(f"forward edge {kw}")
    w, lay, x, lg, idx, tw, y, ref = run_forward(cfg, oracle)
    G.check_y(y, ref, cfg.dtype)


def test_forward_is_deterministic_and_leaves_inputs_alone(oracle):
    import torch
    cfg = SMALL["deepseek_like"]
    w, lay, x, lg, idx, tw, y, ref = run_forward(cfg, oracle)
    x0 = x.clone()
    y0 = lay.y.clone()
    lay.y.fill_(123.0)
    lay.forward_ws.fill_(0xFF)  # scratch contents must not matter
    lay.step(lg, x)
    torch.cuda.synchronize()
    assert torch.equal(lay.y, y0), "two runs differ: an order-dependent reduction is on the path"
    assert torch.equal(x, x0)


# ---------------------------------------------------------------- forward, full-size configs, whole output
def check_rows(y, ref, local):
    """Row by row: the error of every token row against the norm of ITS reference row, so that a wrong row of a small
    expert cannot hide behind the largest value of the whole output.  One bf16 rounding of h and one of y put the
    relative L2 error of a row near 3e-3; 5e-2 leaves room for rows that are sums of partials of opposite sign."""
    err = np.linalg.norm(y - ref, axis=1)
    nrm = np.linalg.norm(ref, axis=1)
    bad = err > 5e-2 * nrm + 1e-6
    assert not bad.any(), f"{int(bad.sum())} rows off, first token {int(np.nonzero(bad)[0][0])}"
    assert np.all(y[~local] == 0)


def full_size_forward_case(oracle, cfg):
    """Runs the layer at full size in every launch form the library has and compares EVERY element of y with the
    oracle (one oracle pass over all tokens: seconds to half a minute on the host cores)."""
    import time

    import torch
    w = wl.make_workload(cfg)
    lay = L.MoELayer(cfg)
    lay.load_weights(w.W_gate, w.W_up, w.W_down)
    x, lg = L.to_device(w.x), L.to_device(w.logits)
    lay.y.fill_(float("nan"))
    lay.step(lg, x)
    torch.cuda.synchronize()
    got = G.tables_to_host(lay)
    idx, tw = G.assert_tables_equal(got, oracle, w.logits, cfg)
    t0 = time.time()
    ref = oracle.forward(w.x, idx, tw, w.W_gate, w.W_up, w.W_down, cfg.E, cfg.R, cfg.local_rank_begin,
                         cfg.local_rank_end)
    say(f"  oracle over all {cfg.T} tokens: {time.time() - t0:.1f} s")
    local = ((idx // cfg.epr >= cfg.local_rank_begin) & (idx // cfg.epr < cfg.local_rank_end)).any(axis=1)
    y = lay.y_host()
    mx, mean = G.check_y(y, ref, cfg.dtype)
    check_rows(y, ref, local)
    say(f"  {cfg.name} k={cfg.k}: all {cfg.T} x {cfg.d} elements, max rel {mx:.2e}, mean rel {mean:.2e}, "
        f"{int(local.sum())} tokens with a local slot")
    assert np.isfinite(y).all() and np.abs(y[local]).max(axis=1).min() > 0
    y_auto = lay.y.clone()
    if cfg.dtype == wl.BF16:  # the other launch form of the GEMMs: same tiles, same arithmetic, same bits
        for fwd in (lay.forward_two_launch, lay.forward_one_launch, lay.forward_resident):
            lay.y.fill_(float("nan"))
            lay.forward_ws.fill_(0xFF)
            fwd(x)
            torch.cuda.synchronize()
            assert torch.equal(lay.y, y_auto) and ws_error_flag(lay) == 0
    return w, lay, x, lg, idx, tw, ref


@pytest.mark.parametrize("name", ["deepseek_v3", "qwen3", "mixtral", "gpt_oss", "table1_s", "table1_m"])
def test_forward_full_size_whole_output(oracle, name):
    cfg = wl.CONFIGS[name]
    say(f"forward full size, whole output: {name}")
    full_size_forward_case(oracle, cfg)


@pytest.mark.parametrize("name,k", [("deepseek_v3", 16), ("deepseek_v3", 32), ("table1_m", 16), ("table1_m", 32)])
def test_forward_table1_topk_columns_whole_output(oracle, name, k):
    """The top-k 16 and 32 columns of the evaluation's model table at its Large (the DeepSeek shape) and Medium
    shapes, near-uniform load as in the table's training setting: every element of y."""
    cfg = wl.CONFIGS[name].scaled(k=k, router="normal")
    say(f"forward full size, whole output: {name} with top-{k}, uniform load")
    full_size_forward_case(oracle, cfg)


# ---------------------------------------------------------------- phase-split entry points and the unfused path
def test_dispatch_gather_and_combine_reduce(oracle):
    import torch
    for name in ("deepseek_like", "mixtral_like", "tiny_f32"):
        cfg = SMALL[name]
        say(f"phase split {name}")
        w = wl.make_workload(cfg, weights=False)
        lay, got = G.run_tables(cfg, w.logits)
        s = lay.shape
        x = L.to_device(w.x)
        P_cap = cfg.T * min(cfg.k, cfg.E_loc)
        xs = torch.zeros((P_cap, cfg.d), dtype=lay.elt_dtype, device="cuda")
        B.moe_dispatch_gather(s, x, lay.tables, xs)
        base = int(got["offsets"][cfg.first_local_expert])
        P = int(got["offsets"][cfg.first_local_expert + cfg.E_loc]) - base
        tok_of_row = got["perm"][base:base + P] // cfg.k
        torch.cuda.synchronize()
        assert torch.equal(xs[:P], x[torch.from_numpy(tok_of_row).cuda().long()])
        assert xs[P:].abs().sum().item() == 0
        rows = torch.from_numpy(np.random.default_rng(1).standard_normal((P_cap, cfg.d)).astype(np.float32)).cuda()
        B.moe_combine_reduce(s, rows, lay.topk_idx, lay.tables, lay.y)
        torch.cuda.synchronize()
        ref = np.zeros((cfg.T, cfg.d))
        rows_h = rows.cpu().numpy().astype(np.float64)
        for r in range(P):
            ref[tok_of_row[r]] += rows_h[r]
        y = lay.y_host()
        tol = 2 ** -8 if cfg.dtype == wl.BF16 else 1e-6
        assert np.all(np.abs(y - ref) <= tol * np.maximum(1.0, np.abs(ref)))


@pytest.mark.parametrize("name", ["deepseek_v3", "gpt_oss"])
def test_dispatch_gather_and_combine_reduce_full_size(oracle, name):
    """Phase-split Dispatch and Combine at the sizes bench.py times, against the oracle's own tables."""
    import torch
    cfg = wl.CONFIGS[name]
    say(f"phase split full size {name}")
    w = wl.make_workload(cfg, weights=False)
    lay, got = G.run_tables(cfg, w.logits)
    idx, _ = oracle.route_topk(w.logits, cfg.k)
    counts, offsets, perm, inv = oracle.build_tables(idx, cfg.E)
    base = int(offsets[cfg.first_local_expert])
    P = int(offsets[cfg.first_local_expert + cfg.E_loc]) - base
    tok_of_row = torch.from_numpy((perm[base:base + P] // cfg.k).astype(np.int64)).cuda()
    x = L.to_device(w.x)
    P_cap = cfg.T * min(cfg.k, cfg.E_loc)
    xs = torch.zeros((P_cap, cfg.d), dtype=lay.elt_dtype, device="cuda")
    B.moe_dispatch_gather(lay.shape, x, lay.tables, xs)
    torch.cuda.synchronize()
    assert torch.equal(xs[:P], x[tok_of_row])          # every layout row holds its token's row, bit for bit
    assert xs[P:].abs().sum().item() == 0              # nothing beyond the local segment is touched
    del xs
    # Combine: integer-valued rows make the fp32 sums exact, so the result is unique whatever the order
    g = torch.Generator(device="cuda").manual_seed(7)
    rows = torch.randint(-8, 9, (P, cfg.d), generator=g, device="cuda").to(torch.float32)
    lay.y.fill_(float("nan"))
    B.moe_combine_reduce(lay.shape, rows, lay.topk_idx, lay.tables, lay.y)
    torch.cuda.synchronize()
    want = torch.zeros((cfg.T, cfg.d), dtype=torch.float32, device="cuda").index_add_(0, tok_of_row, rows)
    assert torch.equal(lay.y.to(torch.float32), want)  # |sums| <= 8 k = 64: exact in bf16 as well


# ---------------------------------------------------------------- the two forms of the GEMM-1 => GEMM-2 hand-over
def ws_error_flag(lay):
    return B.moe_forward_status(lay.forward_ws)


@pytest.mark.parametrize("name", ["deepseek_like", "qwen_like", "mixtral_like", "gpt_oss_like", "k_tail_bf16",
                                  "table1_like_k16", "table1_like_k32"])
def test_one_and_two_launch_forward_match_oracle_and_each_other(oracle, name):
    import torch
    cfg = SMALL[name]
    say(f"one/two-launch small {name}")
    w, lay, x, lg, idx, tw, y, ref = run_forward(cfg, oracle)
    y_auto = lay.y.clone()
    for rep in range(2):  # the second round starts from the counters and tickets the first one left
        for fwd in (lay.forward_two_launch, lay.forward_one_launch, lay.forward_resident):
            lay.y.fill_(float("nan"))
            fwd(x)
            torch.cuda.synchronize()
            G.check_y(lay.y_host(), ref, cfg.dtype)
            # same tiles, same arithmetic per tile: bit-identical whichever way the GEMMs are launched
            assert torch.equal(lay.y, y_auto)
            assert ws_error_flag(lay) == 0, "a wait inside the resident kernel gave up"
    # The hand-over inside the resident kernel, many times over a workspace whose previous contents (h included)
    # are trashed before every call: a GEMM-2 tile that reads h before its producers' rows are visible would see
    # the trash (a repeat over an untouched workspace would see the previous call's identical h and hide it).
    for rep in range(40):
        lay.y.fill_(float("nan"))
        lay.forward_ws.fill_(0xFF if rep % 2 else 0x3C)
        lay.forward_one_launch(x)
        torch.cuda.synchronize()
        assert torch.equal(lay.y, y_auto), f"hand-over call {rep} differs"
    # the same for the second hand-over (GEMM-2 => Combine) of the launch that also reduces the tokens: a token summed
    # before its rows are visible would pick up the trash
    for rep in range(40):
        lay.y.fill_(float("nan"))
        lay.forward_ws.fill_(0xFF if rep % 2 else 0x3C)
        lay.forward_resident(x)
        torch.cuda.synchronize()
        assert torch.equal(lay.y, y_auto), f"resident call {rep} differs"


@pytest.mark.parametrize("kw", [dict(T=1, E=8, k=2, R=2, local_rank_begin=0, local_rank_end=1, d=64, f=64),
                                dict(T=7, E=8, k=8, R=1, local_rank_begin=0, local_rank_end=1, d=520, f=72),  # all tokens, all experts
                                dict(T=300, E=16, k=4, R=4, d=136, f=200, router="zipf"),
                                dict(T=513, E=64, k=6, R=8, d=1032, f=264, local_rank_begin=2, local_rank_end=5),
                                dict(T=64, E=8, k=1, R=2, local_rank_begin=0, local_rank_end=2, d=256, f=128),  # sole rows only
                                dict(T=2000, E=4, k=2, R=1, local_rank_begin=0, local_rank_end=1, d=264, f=128)])  # full M tiles
def test_resident_forward_with_combine_edge_shapes(oracle, kw):
    """GEMM-1, GEMM-2 and Combine in one launch against the oracle and, bit for bit, against the form with kernel
    boundaries, on shapes with ragged tails, empty experts, tokens without a local slot and more tokens than waves."""
    import torch
    cfg = cfg_of(**kw)
    say(f"resident forward edge {kw}")
    w, lay, x, lg, idx, tw, y, ref = run_forward(cfg, oracle)
    y_auto = lay.y.clone()
    for rep in range(3):
        lay.y.fill_(float("nan"))
        lay.forward_ws.fill_(0xA5)
        lay.forward_resident(x)
        torch.cuda.synchronize()
        G.check_y(lay.y_host(), ref, cfg.dtype)
        assert torch.equal(lay.y, y_auto) and ws_error_flag(lay) == 0


def test_resident_forward_combine_wait_gives_up_cleanly(oracle):
    """As the give-up test of the GEMM-2 wait, for the launch that also runs Combine: every wait (GEMM-2 items for h,
    tokens for their rows) expects one more finished tile than exists and gives up after a handful of polls."""
    import torch
    cfg = SMALL["deepseek_like"]
    say("resident kernel with Combine: forced give-up")
    w, lay, x, lg, idx, tw, y, ref = run_forward(cfg, oracle)
    y_good = lay.y.clone()
    lay.y.fill_(123.0)
    B.moe_fused_forward_resident(lay.shape, x, lay.topk_idx, lay.topk_w, lay.tables, lay.packed_gate_up,
                                 lay.packed_down, lay.y, lay.forward_ws, max_polls=4, wait_extra=1)
    torch.cuda.synchronize()
    assert B.moe_forward_status(lay.forward_ws) == 1
    local = ((idx // cfg.epr >= cfg.local_rank_begin) & (idx // cfg.epr < cfg.local_rank_end)).any(axis=1)
    yb = lay.y[: cfg.T].float().cpu().numpy()
    assert np.isnan(yb[local]).all(), "a row computed after a wait gave up is not marked"
    assert np.all(yb[~local] == 0)
    lay.y.fill_(float("nan"))
    lay.forward_resident(x)
    torch.cuda.synchronize()
    assert B.moe_forward_status(lay.forward_ws) == 0
    assert torch.equal(lay.y, y_good)


def test_resident_kernel_wait_gives_up_cleanly(oracle):
    """The bounded wait of the GEMM-1 => GEMM-2 hand-over, forced from the host: every GEMM-2 tile waits for one more
    GEMM-1 tile than exists and the bound is a handful of polls, so every wait gives up.  All kernels still exit,
    the call returns, the status word reads 1 and nothing computed from the incomplete tiles looks like a result
    (NaN rows); the next ordinary call on the same workspace is correct again and the status word reads 0."""
    import torch
    cfg = SMALL["deepseek_like"]
    say("resident kernel: forced give-up")
    w, lay, x, lg, idx, tw, y, ref = run_forward(cfg, oracle)
    y_good = lay.y.clone()
    assert B.moe_forward_status(lay.forward_ws) == 0
    lay.y.fill_(123.0)
    B.moe_fused_forward_bounded(lay.shape, x, lay.topk_idx, lay.topk_w, lay.tables, lay.packed_gate_up,
                                lay.packed_down, lay.y, lay.forward_ws, max_polls=4, wait_extra=1)
    torch.cuda.synchronize()
    assert B.moe_forward_status(lay.forward_ws) == 1
    local = ((idx // cfg.epr >= cfg.local_rank_begin) & (idx // cfg.epr < cfg.local_rank_end)).any(axis=1)
    yb = lay.y[: cfg.T].float().cpu().numpy()
    assert np.isnan(yb[local]).all(), "a row computed after a wait gave up is not marked"
    assert np.all(yb[~local] == 0)
    # an ample bound and the real count: the ordinary result
    lay.y.fill_(float("nan"))
    B.moe_fused_forward_bounded(lay.shape, x, lay.topk_idx, lay.topk_w, lay.tables, lay.packed_gate_up,
                                lay.packed_down, lay.y, lay.forward_ws, max_polls=1 << 22, wait_extra=0)
    torch.cuda.synchronize()
    assert B.moe_forward_status(lay.forward_ws) == 0
    assert torch.equal(lay.y, y_good)


def test_one_launch_forward_rejects_fp32_layers():
    cfg = SMALL["f32_ragged"]
    w = wl.make_workload(cfg)
    lay = L.MoELayer(cfg)
    lay.load_weights(w.W_gate, w.W_up, w.W_down)
    lay.step(L.to_device(w.logits), L.to_device(w.x))
    with pytest.raises(B.MoeError) as err:
        lay.forward_one_launch(L.to_device(w.x))
    assert err.value.status == B.MOE_ERR_UNSUPPORTED
    assert B.moe_forward_gemm_launches(lay.shape) == 2


# ---------------------------------------------------------------- the whole step inside a HIP graph
@pytest.mark.parametrize("name", ["deepseek_like", "gpt_oss_like"])
def test_step_replays_from_a_hip_graph(oracle, name):
    """route + tables + forward captured once and replayed: every launch takes its sizes from device memory, so a
    replay follows whatever logits and tokens the input buffers hold at that moment.  Replays alternate with eager
    work and are checked against eager results and the oracle."""
    import torch
    cfg = SMALL[name]
    say(f"graph replay {name}")
    w, lay, x, lg, idx, tw, y, ref = run_forward(cfg, oracle)   # eager, also warms up one-off attribute calls
    y_first = lay.y.clone()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        lay.step(lg, x)
    # second input set: other tokens and another routing, written into the same buffers before a replay
    w2 = wl.make_workload(cfg.scaled(seed=cfg.seed + 100))
    x_b, lg_b = L.to_device(w2.x), L.to_device(w2.logits)
    x_a, lg_a = x.clone(), lg.clone()
    idx2, tw2 = oracle.route_topk(w2.logits, cfg.k)
    ref2 = oracle.forward(w2.x, idx2, tw2, w.W_gate, w.W_up, w.W_down, cfg.E, cfg.R, cfg.local_rank_begin,
                          cfg.local_rank_end)
    for rep in range(3):
        for (xi, lgi, want, first) in ((x_b, lg_b, ref2, None), (x_a, lg_a, ref, y_first)):
            x.copy_(xi)
            lg.copy_(lgi)
            lay.y.fill_(float("nan"))
            lay.forward_ws.fill_(0xFF)
            graph.replay()
            torch.cuda.synchronize()
            G.check_y(lay.y_host(), want, cfg.dtype)
            if first is not None:
                assert torch.equal(lay.y, first), "replay differs from the eager run on the same inputs"
            assert ws_error_flag(lay) == 0


def test_unfused_path_full_size_agrees_with_fused():
    """The comparison path of bench.py at full size: same GEMM tiles, but an atomic fp32 scatter-add instead of the
    ordered reduction, so it agrees with the fused result to fp32 reordering plus one bf16 rounding, not bit for bit."""
    import torch
    cfg = wl.CONFIGS["deepseek_v3"]
    say("unfused full size deepseek_v3")
    w = wl.make_workload(cfg)
    lay = L.MoELayer(cfg, unfused=True)
    lay.load_weights(w.W_gate, w.W_up, w.W_down)
    x, lg = L.to_device(w.x), L.to_device(w.logits)
    lay.route(lg)
    lay.build_dispatch()
    lay.forward(x)
    torch.cuda.synchronize()
    y_fused = lay.y.to(torch.float32).clone()
    lay.y.fill_(float("nan"))
    lay.forward_unfused(x)
    torch.cuda.synchronize()
    y_unf = lay.y.to(torch.float32)
    assert torch.isfinite(y_unf).all()
    scale = y_fused.abs().max().item()
    assert (y_unf - y_fused).abs().max().item() <= 2 ** -7 * scale   # at most one bf16 ulp of the largest value
    assert (y_unf != y_fused).float().mean().item() < 0.05            # and rarely different at all


@pytest.mark.parametrize("name", ["deepseek_like", "tiny_f32"])
def test_unfused_path_matches_oracle(oracle, name):
    import torch
    cfg = SMALL[name]
    say(f"unfused {name}")
    w = wl.make_workload(cfg)
    lay = L.MoELayer(cfg, unfused=True)
    lay.load_weights(w.W_gate, w.W_up, w.W_down)
    x, lg = L.to_device(w.x), L.to_device(w.logits)
    lay.route(lg)
    lay.build_dispatch()
    lay.forward_unfused(x)
    torch.cuda.synchronize()
    idx, tw = oracle.route_topk(w.logits, cfg.k)
    ref = oracle.forward(w.x, idx, tw, w.W_gate, w.W_up, w.W_down, cfg.E, cfg.R, cfg.local_rank_begin,
                         cfg.local_rank_end)
    G.check_y(lay.y_host(), ref, cfg.dtype)


# ---------------------------------------------------------------- gate network ahead of the routing
def router_case(T, d, E, k, dtype, seed):
    rng = np.random.default_rng(seed)
    x32 = rng.standard_normal((T, d)).astype(np.float32)
    W32 = (rng.standard_normal((E, d)) * d ** -0.5).astype(np.float32)
    if dtype == wl.BF16:
        return wl.f32_to_bf16_bits(x32), wl.f32_to_bf16_bits(W32)
    return x32, W32


def check_router(oracle, T, d, E, k, dtype, seed, rows=None):
    import torch
    x, W = router_case(T, d, E, k, dtype, seed)
    cfg = cfg_of(T=T, d=d, f=8, E=E, k=k, R=1, local_rank_begin=0, local_rank_end=1, dtype=dtype)
    s = B.shape_of(cfg)
    xd, Wd = L.to_device(x), L.to_device(W)
    logits = torch.full((T, E), float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.full((B.moe_router_workspace_bytes(s),), 0xFF, dtype=torch.uint8, device="cuda")
    B.moe_router_logits(s, xd, Wd, logits, ws)
    again = torch.empty_like(logits)
    B.moe_router_logits(s, xd, Wd, again, ws)
    torch.cuda.synchronize()
    assert torch.equal(logits, again), "the gate network is not reproducible"
    got = logits.cpu().numpy().astype(np.float64)
    sel = np.arange(T) if rows is None else rows
    ref = oracle.router_logits(np.ascontiguousarray(x[sel]), W)
    xf = (wl.bf16_bits_to_f32(x[sel]) if dtype == wl.BF16 else x[sel]).astype(np.float64)
    Wf = (wl.bf16_bits_to_f32(W) if dtype == wl.BF16 else W).astype(np.float64)
    # fp32 accumulation of d exact products (bf16) or d fused multiply-adds (fp32), in any order
    tol = d * 2.0 ** -23 * (np.abs(xf) @ np.abs(Wf).T) + 1e-30
    assert np.all(np.abs(got[sel] - ref) <= tol), f"max excess {(np.abs(got[sel] - ref) / tol).max():.3f}"
    # routing on the GPU's logits: with eps the largest deviation actually seen in a token's row, two logits
    # further apart than 2 eps keep their order, so the picks must equal the oracle's wherever the oracle's own
    # margins (among its k + 1 largest logits) exceed 2 eps, and must be a valid top-k within 2 eps everywhere
    idx = torch.empty((T, k), dtype=torch.int32, device="cuda")
    wts = torch.empty((T, k), dtype=torch.float32, device="cuda")
    B.moe_route_topk(s, logits, idx, wts)
    torch.cuda.synchronize()
    idx = idx.cpu().numpy()[sel]
    ridx, _ = oracle.route_topk(ref.astype(np.float32), k)
    order = np.argsort(-ref, axis=1, kind="stable")
    srt = np.take_along_axis(ref, order, axis=1)
    tmax = np.abs(got[sel] - ref).max(axis=1)
    top = srt[:, :min(k + 1, E)]
    safe = (top[:, :-1] - top[:, 1:]).min(axis=1) > 2 * tmax if top.shape[1] > 1 else np.ones(len(sel), bool)
    assert np.array_equal(idx[safe], ridx[safe])
    kth = srt[:, k - 1]
    picked = np.take_along_axis(ref, idx.astype(np.int64), axis=1)
    assert np.all(picked >= (kth - 2 * tmax)[:, None])
    assert all(len(set(r)) == k for r in idx.tolist())
    return int(safe.sum()), len(sel)


@pytest.mark.parametrize("T,d,E,k,dtype", [(1, 8, 1, 1, wl.BF16), (70, 72, 6, 3, wl.BF16), (130, 24, 65, 4, wl.BF16),
                                           (300, 520, 128, 8, wl.BF16), (90, 136, 300, 4, wl.BF16),
                                           (2100, 64, 16, 2, wl.BF16), (33, 40, 12, 2, wl.F32)])
def test_router_logits_small(oracle, T, d, E, k, dtype):
    say(f"router logits T={T} d={d} E={E} dtype={dtype}")
    n_safe, n = check_router(oracle, T, d, E, k, dtype, seed=T + d)
    say(f"  {n_safe} of {n} tokens with margins above the tolerance compared index by index")


def test_router_logits_deepseek_shape_all_tokens(oracle):
    cfg = wl.CONFIGS["deepseek_v3"]
    say("router logits at the DeepSeek shape, every logit")
    n_safe, n = check_router(oracle, cfg.T, cfg.d, cfg.E, cfg.k, wl.BF16, seed=77)
    say(f"  {n_safe} of {n} tokens compared index by index")
    assert n_safe > n // 2


def check_route_from_x(oracle, T, d, E, k, dtype, seed, want_logits):
    """The fused call against the two-call form on the GPU (bit for bit: same partial products, same order) and
    against the oracle (picks equal wherever the oracle's margins exceed the fp32 deviation, valid elsewhere)."""
    import torch
    x, W = router_case(T, d, E, k, dtype, seed)
    cfg = cfg_of(T=T, d=d, f=8, E=E, k=k, R=1, local_rank_begin=0, local_rank_end=1, dtype=dtype)
    s = B.shape_of(cfg)
    xd, Wd = L.to_device(x), L.to_device(W)
    logits2 = torch.empty((T, E), dtype=torch.float32, device="cuda")
    ws2 = torch.full((B.moe_router_workspace_bytes(s),), 0xFF, dtype=torch.uint8, device="cuda")
    idx2 = torch.empty((T, k), dtype=torch.int32, device="cuda")
    w2 = torch.empty((T, k), dtype=torch.float32, device="cuda")
    B.moe_router_logits(s, xd, Wd, logits2, ws2)
    B.moe_route_topk(s, logits2, idx2, w2)
    ws = torch.full((B.moe_route_from_x_workspace_bytes(s),), 0xFF, dtype=torch.uint8, device="cuda")
    idx = torch.full((T, k), -1, dtype=torch.int32, device="cuda")
    w = torch.full((T, k), float("nan"), dtype=torch.float32, device="cuda")
    logits = torch.full((T, E), float("nan"), dtype=torch.float32, device="cuda") if want_logits else None
    B.moe_route_from_x(s, xd, Wd, logits, idx, w, ws)
    torch.cuda.synchronize()
    assert torch.equal(idx, idx2) and torch.equal(w, w2), "fused and two-call routing differ"
    if want_logits:
        assert torch.equal(logits, logits2)
    # against the oracle
    ref = oracle.router_logits(x, W)
    got = logits2.cpu().numpy().astype(np.float64)
    ridx, rw = oracle.route_topk(ref.astype(np.float32), k)
    order = np.argsort(-ref, axis=1, kind="stable")
    srt = np.take_along_axis(ref, order, axis=1)
    tmax = np.abs(got - ref).max(axis=1)
    top = srt[:, :min(k + 1, E)]
    safe = (top[:, :-1] - top[:, 1:]).min(axis=1) > 2 * tmax if top.shape[1] > 1 else np.ones(T, bool)
    ih, wh = idx.cpu().numpy(), w.cpu().numpy()
    assert np.array_equal(ih[safe], ridx[safe])
    assert np.abs(wh[safe] - rw[safe]).max() <= 1e-5 if safe.any() else True  # weights follow logits that differ by tmax
    picked = np.take_along_axis(ref, ih.astype(np.int64), axis=1)
    assert np.all(picked >= (srt[:, k - 1] - 2 * tmax)[:, None])
    assert all(len(set(r)) == k for r in ih.tolist())
    return int(safe.sum())


@pytest.mark.parametrize("T,d,E,k,dtype,want_logits", [(1, 8, 1, 1, wl.BF16, True), (70, 72, 6, 3, wl.BF16, False),
                                                       (130, 24, 65, 4, wl.BF16, True),
                                                       (300, 520, 128, 8, wl.BF16, False),
                                                       (90, 136, 300, 4, wl.BF16, True),
                                                       (700, 64, 640, 6, wl.BF16, True),    # beyond a wave's registers
                                                       (2100, 64, 16, 2, wl.BF16, False),
                                                       (33, 40, 12, 2, wl.F32, True)])
def test_route_from_x_small(oracle, T, d, E, k, dtype, want_logits):
    say(f"route from x T={T} d={d} E={E} k={k} dtype={dtype} logits={want_logits}")
    n_safe = check_route_from_x(oracle, T, d, E, k, dtype, seed=T + d + 1, want_logits=want_logits)
    say(f"  {n_safe} of {T} tokens compared pick by pick with the oracle")


@pytest.mark.parametrize("name", ["deepseek_v3", "qwen3", "gpt_oss"])
def test_route_from_x_full_size(oracle, name):
    cfg = wl.CONFIGS[name]
    say(f"route from x at the {name} shape, every token")
    n_safe = check_route_from_x(oracle, cfg.T, cfg.d, cfg.E, cfg.k, wl.BF16, seed=78, want_logits=False)
    say(f"  {n_safe} of {cfg.T} tokens compared pick by pick with the oracle")
    assert n_safe > cfg.T // 2


# ---------------------------------------------------------------- FP8 form of the expert GEMMs
@pytest.mark.parametrize("rows,cols", [(1, 8), (37, 72), (300, 448), (64, 7168)])
def test_fp8_quantize_rows_bit_exact(oracle, rows, cols):
    import torch
    say(f"fp8 quantize rows {rows} x {cols}")
    rng = np.random.default_rng(rows + cols)
    a = rng.standard_normal((rows, cols)) * 10.0 ** rng.uniform(-3, 2, size=(rows, 1))
    a[:, ::5] *= 1e-3                               # small against the row maximum: subnormal codes and zeros
    if rows > 2:
        a[1] = 0.0                                  # a zero row: scale 1
        a[2, :] = np.arange(cols) % 17 * 28.0       # multiples of amax / 16: exact ties between codes
    bits = wl.f32_to_bf16_bits(a.astype(np.float32))
    x = L.to_device(bits)
    codes = torch.full((rows, cols), 0xAA, dtype=torch.uint8, device="cuda")
    scales = torch.full((rows,), float("nan"), dtype=torch.float32, device="cuda")
    B.moe_fp8_quantize_rows(rows, cols, x, codes, scales)
    torch.cuda.synchronize()
    want_codes, want_scales = oracle.fp8_quantize(wl.bf16_bits_to_f32(bits), axis=-1)
    assert np.array_equal(scales.cpu().numpy(), want_scales)
    got = codes.cpu().numpy()
    # -0 and +0 are the same value: compare codes up to the sign of zero
    same = (got == want_codes) | (((got | want_codes) & 0x7F) == 0)
    assert same.all(), f"{(~same).sum()} codes differ"


FP8_SMALL = {
    "deepseek_like": SMALL["deepseek_like"],
    "qwen_like": SMALL["qwen_like"],
    "mixtral_like": SMALL["mixtral_like"],
    "table1_like_k16": SMALL["table1_like_k16"],
    # reduction tails (368 = 2 x 128 + 112, 336 = 2 x 128 + 80), column tails, forced routing
    "tails": cfg_of(T=1100, d=368, f=336, E=32, k=4, R=4, local_rank_begin=0, local_rank_end=1, router="forced",
                    seed=31),
    # more than one M tile of rows per expert on average: the GEMMs run as two launches
    "two_launch": cfg_of(T=1200, d=256, f=256, E=16, k=4, R=4, local_rank_begin=1, local_rank_end=2, seed=32),
}


def run_forward_fp8(cfg, oracle, tokens=None):
    import torch
    w = wl.make_workload(cfg)
    s_h = wl.fp8_h_scale(cfg)
    lay = L.MoELayer(cfg)
    lay.load_weights_fp8(w.W_gate, w.W_up, w.W_down, s_h)
    x = L.to_device(w.x)
    lg = L.to_device(w.logits)
    lay.y.fill_(float("nan"))
    lay.fp8_ws.fill_(0xFF)
    lay.route(lg)
    lay.build_dispatch()
    lay.forward_fp8(x)
    torch.cuda.synchronize()
    got = G.tables_to_host(lay)
    idx, tw = G.assert_tables_equal(got, oracle, w.logits, cfg)
    y = lay.y_host()
    ref = oracle.forward_fp8(w.x, idx, tw, w.W_gate, w.W_up, w.W_down, s_h, cfg.E, cfg.R, cfg.local_rank_begin,
                             cfg.local_rank_end, tokens=tokens)
    return w, lay, x, idx, tw, y, ref


@pytest.mark.parametrize("name", list(FP8_SMALL))
def test_fp8_forward_matches_oracle_small(oracle, name):
    import torch
    cfg = FP8_SMALL[name]
    say(f"fp8 forward small {name}: T={cfg.T} d={cfg.d} f={cfg.f} E={cfg.E} k={cfg.k} "
        f"launches={B.moe_forward_gemm_launches(B.shape_of(cfg))}")
    w, lay, x, idx, tw, y, ref = run_forward_fp8(cfg, oracle)
    mx, mean = G.check_y(y, ref, cfg.dtype)
    say(f"  max rel {mx:.2e} mean rel {mean:.2e}")
    local = (idx // cfg.epr >= cfg.local_rank_begin) & (idx // cfg.epr < cfg.local_rank_end)
    assert np.all(y[~local.any(axis=1)] == 0)
    # the quantised layer is a different function from the bf16 one (the test would not notice a bf16 fallback
    # otherwise) and still close to it
    ref16 = oracle.forward(w.x, idx, tw, w.W_gate, w.W_up, w.W_down, cfg.E, cfg.R, cfg.local_rank_begin,
                           cfg.local_rank_end)
    rel = np.linalg.norm(y - ref16) / np.linalg.norm(ref16)
    assert 5e-3 < rel < 0.1, rel
    # rerun over a trashed workspace: bit-identical
    y0 = lay.y.clone()
    lay.fp8_ws.fill_(0x5A)
    lay.y.fill_(7.0)
    lay.forward_fp8(x)
    torch.cuda.synchronize()
    assert torch.equal(lay.y, y0)


def test_fp8_rejects_what_it_does_not_cover():
    cfg = cfg_of(d=72, f=40)  # rows are not whole 16-code chunks
    lay = L.MoELayer(cfg)
    with pytest.raises(B.MoeError):
        lay.load_weights_fp8(*(np.zeros(sh, np.uint16) for sh in ((cfg.E_loc, 72, 40),) * 2),
                             np.zeros((cfg.E_loc, 40, 72), np.uint16), wl.fp8_h_scale(cfg))


@pytest.mark.parametrize("name", ["deepseek_v3", "qwen3", "mixtral", "gpt_oss"])
def test_fp8_forward_full_size_whole_output(oracle, name):
    """Every element of y of the FP8 layer at full size (5-20 s of oracle time per layer)."""
    cfg = wl.CONFIGS[name]
    say(f"fp8 forward full size, whole output: {name}")
    w, lay, x, idx, tw, y, ref = run_forward_fp8(cfg, oracle)
    local = ((idx // cfg.epr >= cfg.local_rank_begin) & (idx // cfg.epr < cfg.local_rank_end)).any(axis=1)
    mx, mean = G.check_y(y, ref, cfg.dtype)
    check_rows(y, ref, local)
    say(f"  {name}: all {cfg.T} tokens, max rel {mx:.2e}, mean rel {mean:.2e}")
    assert np.isfinite(y).all()


# ---------------------------------------------------------------- gate variants: sigmoid gate, selection-only bias
@pytest.mark.parametrize("T,E,k,gate,with_bias", [(257, 256, 8, 1, True), (1000, 128, 4, 1, False), (300, 64, 6, 0, True),
                                                  (90, 4096, 5, 1, True), (64, 8, 8, 1, True), (1, 4, 2, 0, True),
                                                  (4096, 256, 8, 1, True)])
def test_route_gate_variants(oracle, T, E, k, gate, with_bias):
    import torch
    say(f"route gate={gate} bias={with_bias} T={T} E={E} k={k}")
    rng = np.random.default_rng(T + E + gate)
    logits = rng.standard_normal((T, E)).astype(np.float32) * 2
    logits[::5] = np.round(logits[::5] * 2) / 2       # exact ties
    logits[3::11] += 30.0                             # the sigmoid saturates: many equal selection values
    bias = (rng.standard_normal(E) * 0.1).astype(np.float32) if with_bias else None
    if with_bias:
        bias[::3] = 0.125                             # equal biases keep the exact ties
    cfg = cfg_of(T=T, E=E, k=k, R=1, d=8, f=8, local_rank_begin=0, local_rank_end=1)
    s = B.shape_of(cfg)
    idx = torch.full((T, k), -1, dtype=torch.int32, device="cuda")
    w = torch.full((T, k), float("nan"), dtype=torch.float32, device="cuda")
    B.moe_route_topk_gate(s, L.to_device(logits), None if bias is None else L.to_device(bias), gate, idx, w)
    torch.cuda.synchronize()
    idx, w = idx.cpu().numpy(), w.cpu().numpy()
    ridx, rw, sel = oracle.route_topk_gate(logits, k, gate, bias)
    # Where the gap between the k-th and the (k+1)-th selection value and between consecutive picks exceeds what
    # two exp implementations can differ by (a few ulp of a value <= 1 plus the bias), the picks are unique: exact
    # comparison.  Elsewhere: the picks must be k distinct experts whose values are within that slack of the oracle's.
    srt = -np.sort(-sel.astype(np.float64), axis=1)
    slack = 4e-7 * (1.0 + np.abs(srt[:, :1]))
    gaps = srt[:, :-1] - srt[:, 1:] if E > 1 else np.ones((T, 1))
    lim = min(k, E - 1)
    decisive = (gaps[:, :lim] > slack) | (gaps[:, :lim] == 0)
    # an exact tie (gap 0) is only decisive if both implementations see it as one: true when gate == 0 (no exp)
    safe = (gaps[:, :lim] > slack).all(axis=1) if gate == 1 else decisive.all(axis=1)
    assert safe.sum() >= T // 4 or T < 8
    assert np.array_equal(idx[safe], ridx[safe])
    assert np.abs(w[safe] - rw[safe]).max() <= 1e-6 if safe.any() else True
    picked = np.take_along_axis(sel.astype(np.float64), idx.astype(np.int64), axis=1)
    assert np.all(picked >= srt[:, k - 1:k] - slack)
    assert np.all(np.diff(picked, axis=1) <= slack)  # slot order = descending selection value
    assert all(len(set(r)) == k for r in idx.tolist())
    assert np.allclose(w.sum(axis=1), 1.0, atol=1e-5) and np.isfinite(w).all()


# ---------------------------------------------------------------- training path: forward that keeps g, u, o; backward
BWD_SMALL = {
    "deepseek_like": cfg_of(T=700, d=448, f=320, E=64, k=8, R=8, local_rank_begin=0, local_rank_end=1, router="zipf",
                            seed=21),
    "qwen_like": SMALL["qwen_like"],
    "mixtral_like": SMALL["mixtral_like"],
    "ragged": cfg_of(T=333, d=200, f=128, E=12, k=3, R=3, local_rank_begin=1, local_rank_end=3, seed=41),
    "table1_like_k16": SMALL["table1_like_k16"],
    # 80 pairs over 64 experts: many local experts without a row (their gradients are zero), others with one or two
    "empty_experts": cfg_of(T=40, d=64, f=64, E=64, k=2, R=2, local_rank_begin=0, local_rank_end=1, seed=42),
    # several hundred local experts: the block scan and the block -> expert search of the weight-gradient path
    "many_experts": cfg_of(T=500, d=64, f=64, E=512, k=4, R=1, local_rank_begin=0, local_rank_end=1, seed=43),
}


def dy_for(cfg, seed=9):
    rng = np.random.default_rng(seed + cfg.seed)
    return wl.f32_to_bf16_bits(rng.standard_normal((cfg.T, cfg.d)).astype(np.float32))


def run_backward(cfg, oracle, wgrad):
    import torch
    w = wl.make_workload(cfg)
    lay = L.MoELayer(cfg)
    lay.load_weights(w.W_gate, w.W_up, w.W_down)
    lay.enable_training(w.W_gate, w.W_up, w.W_down, wgrad=wgrad)
    x, lg = L.to_device(w.x), L.to_device(w.logits)
    dy_bits = dy_for(cfg)
    dy = L.to_device(dy_bits)
    lay.route(lg)
    lay.build_dispatch()
    lay.y.fill_(float("nan"))
    lay.forward_train(x)
    lay.dx.fill_(float("nan"))
    lay.d_topk_w.fill_(float("nan"))
    lay.backward_ws.fill_(0xFF)
    if wgrad:
        for t in (lay.dW_gate, lay.dW_up, lay.dW_down):
            t.fill_(float("nan"))
    lay.backward(x, dy)
    torch.cuda.synchronize()
    got = G.tables_to_host(lay)
    idx, tw = G.assert_tables_equal(got, oracle, w.logits, cfg)
    return w, lay, x, dy, dy_bits, idx, tw


@pytest.mark.parametrize("name", list(BWD_SMALL))
def test_backward_tokens_matches_oracle_small(oracle, name):
    import torch
    cfg = BWD_SMALL[name]
    say(f"backward (dx, d_topk_w) small {name}: T={cfg.T} d={cfg.d} f={cfg.f} E={cfg.E} k={cfg.k}")
    w, lay, x, dy, dy_bits, idx, tw = run_backward(cfg, oracle, wgrad=False)
    lr = (cfg.local_rank_begin, cfg.local_rank_end)
    # the training forward gives the same y as the plain forward's oracle
    ref_y = oracle.forward(w.x, idx, tw, w.W_gate, w.W_up, w.W_down, cfg.E, cfg.R, *lr)
    G.check_y(lay.y_host(), ref_y, cfg.dtype)
    ref_dx, ref_dw = oracle.backward_tokens(w.x, dy_bits, idx, tw, w.W_gate, w.W_up, w.W_down, cfg.E, cfg.R, *lr)
    dx = lay.dx[: cfg.T].to(torch.float64).cpu().numpy()
    mx, mean = G.check_y(dx, ref_dx, cfg.dtype)
    dw = lay.d_topk_w[: cfg.T * cfg.k].cpu().numpy().astype(np.float64).reshape(cfg.T, cfg.k)
    local = (idx // cfg.epr >= lr[0]) & (idx // cfg.epr < lr[1])
    assert np.all(dw[~local] == 0) and np.all(dx[~local.any(axis=1)] == 0)
    err = np.abs(dw - ref_dw).max() / np.abs(ref_dw).max()
    say(f"  dx max rel {mx:.2e} mean rel {mean:.2e}; d_topk_w max err / max {err:.2e}")
    assert err <= 2e-2
    # rerun over a trashed workspace: bit-identical
    dx0, dw0 = lay.dx.clone(), lay.d_topk_w.clone()
    lay.backward_ws.fill_(0x5A)
    lay.dx.fill_(3.0)
    lay.backward(x, dy)
    torch.cuda.synchronize()
    assert torch.equal(lay.dx, dx0) and torch.equal(lay.d_topk_w, dw0)


def check_weight_grads(oracle, cfg, w, lay, dy_bits, idx, tw, experts, n0, n1):
    import torch
    lr = (cfg.local_rank_begin, cfg.local_rank_end)
    worst = 0.0
    for le in experts:
        rg, ru, rd = oracle.backward_weights(w.x, dy_bits, idx, tw, w.W_gate, w.W_up, w.W_down, cfg.E, cfg.R, *lr, le,
                                             n0, n1)
        got = (lay.dW_gate[le, :, n0:n1], lay.dW_up[le, :, n0:n1], lay.dW_down[le, n0:n1, :])
        for name, gt, ref in zip(("dW_gate", "dW_up", "dW_down"), got, (rg, ru, rd)):
            g = gt.to(torch.float64).cpu().numpy()
            assert np.isfinite(g).all(), name
            if np.abs(ref).max() == 0:
                assert np.all(g == 0), name
                continue
            mx, mean = G.check_y(g, ref, cfg.dtype)
            worst = max(worst, mean)
    return worst


@pytest.mark.parametrize("name", list(BWD_SMALL))
def test_backward_weight_gradients_match_oracle_small(oracle, name):
    import torch
    cfg = BWD_SMALL[name]
    say(f"backward (weight gradients) small {name}: T={cfg.T} d={cfg.d} f={cfg.f} E={cfg.E} k={cfg.k}")
    w, lay, x, dy, dy_bits, idx, tw = run_backward(cfg, oracle, wgrad=True)
    counts = np.bincount(idx.ravel(), minlength=cfg.E)[cfg.first_local_expert:cfg.first_local_expert + cfg.E_loc]
    worst = check_weight_grads(oracle, cfg, w, lay, dy_bits, idx, tw, range(cfg.E_loc), 0, cfg.f)
    say(f"  rows per local expert {counts.min()}..{counts.max()}, worst mean rel {worst:.2e}")
    # an expert without rows has zero gradients (checked above through the all-zero reference); dx is unchanged by
    # the presence of the weight-gradient outputs
    ref_dx, _ = oracle.backward_tokens(w.x, dy_bits, idx, tw, w.W_gate, w.W_up, w.W_down, cfg.E, cfg.R,
                                       cfg.local_rank_begin, cfg.local_rank_end)
    G.check_y(lay.dx[: cfg.T].to(torch.float64).cpu().numpy(), ref_dx, cfg.dtype)
    g0 = [t.clone() for t in (lay.dW_gate, lay.dW_up, lay.dW_down)]
    lay.backward_ws.fill_(0xA5)
    lay.backward(x, dy)
    torch.cuda.synchronize()
    assert all(torch.equal(a, b) for a, b in zip(g0, (lay.dW_gate, lay.dW_up, lay.dW_down)))


@pytest.mark.parametrize("name", ["deepseek_v3", "qwen3", "mixtral", "gpt_oss"])
def test_backward_full_size_whole_output(oracle, name):
    """Full-size layers.  dx and d_topk_w: every element (7-31 s of oracle time per layer).  Weight gradients: a
    64-wide range of hidden indices from EVERY non-empty local expert (all of the three matrices would be minutes of
    oracle time on the largest layers), experts without rows exactly zero, everything finite."""
    import time

    import torch
    cfg = wl.CONFIGS[name]
    say(f"backward full size, whole dx and d_topk_w: {name}")
    w, lay, x, dy, dy_bits, idx, tw = run_backward(cfg, oracle, wgrad=True)
    lr = (cfg.local_rank_begin, cfg.local_rank_end)
    local = (idx // cfg.epr >= lr[0]) & (idx // cfg.epr < lr[1])
    t0 = time.time()
    ref_dx, ref_dw = oracle.backward_tokens(w.x, dy_bits, idx, tw, w.W_gate, w.W_up, w.W_down, cfg.E, cfg.R, *lr)
    say(f"  oracle backward over all {cfg.T} tokens: {time.time() - t0:.1f} s")
    dx = lay.dx[: cfg.T].to(torch.float64).cpu().numpy()
    dw = lay.d_topk_w[: cfg.T * cfg.k].cpu().numpy().astype(np.float64).reshape(cfg.T, cfg.k)
    mx, mean = G.check_y(dx, ref_dx, cfg.dtype)
    check_rows(dx, ref_dx, local.any(axis=1))
    err = np.abs(dw - ref_dw).max() / np.abs(ref_dw).max()
    say(f"  dx: max rel {mx:.2e} mean rel {mean:.2e}; d_topk_w {err:.2e}")
    assert err <= 2e-2
    assert np.isfinite(dx).all() and np.all(dw[~local] == 0) and np.isfinite(dw).all()
    counts = np.bincount(idx.ravel(), minlength=cfg.E)[cfg.first_local_expert:cfg.first_local_expert + cfg.E_loc]
    n0 = (cfg.f // 2) // 64 * 64 + 24
    nonempty = [int(e) for e in np.nonzero(counts > 0)[0]]
    t0 = time.time()
    worst = check_weight_grads(oracle, cfg, w, lay, dy_bits, idx, tw, nonempty, n0, n0 + 64)
    say(f"  weight gradients of all {len(nonempty)} non-empty experts ({counts[counts > 0].min()}..{counts.max()} rows), "
        f"hidden indices {n0}..{n0 + 63}: worst mean rel {worst:.2e} ({time.time() - t0:.1f} s of oracle)")
    for le in np.nonzero(counts == 0)[0]:
        assert lay.dW_gate[le].abs().max().item() == 0 and lay.dW_up[le].abs().max().item() == 0
        assert lay.dW_down[le].abs().max().item() == 0
    for t in (lay.dW_gate, lay.dW_up, lay.dW_down):
        assert torch.isfinite(t.float()).all()


@pytest.mark.parametrize("name", ["ragged", "empty_experts"])
def test_backward_replays_from_a_hip_graph(oracle, name):
    """The backward call forks part of its work to a stream of the library's own and joins it before it returns, so
    a capture of the caller's stream takes in all of it.  Replays alternate with eager calls and synchronisations and
    must give the eager call's bits every time."""
    import torch
    cfg = BWD_SMALL[name]
    say(f"backward graph replay {name}")
    w, lay, x, dy, dy_bits, idx, tw = run_backward(cfg, oracle, wgrad=True)   # eager; also the one-off set-up calls
    outs = lambda: (lay.dx, lay.d_topk_w, lay.dW_gate, lay.dW_up, lay.dW_down)
    want = [t.clone() for t in outs()]
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        lay.backward(x, dy)
    for rep in range(3):
        for t in outs():
            t.fill_(float("nan"))
        lay.backward_ws.fill_(0x3C + rep)
        graph.replay()
        torch.cuda.synchronize()
        assert all(torch.equal(a, b) for a, b in zip(want, outs())), f"replay {rep} differs from the eager call"
        lay.backward(x, dy)   # eager work between the replays
        torch.cuda.synchronize()
        assert all(torch.equal(a, b) for a, b in zip(want, outs()))


def test_backward_from_two_host_threads(oracle):
    """Two host threads, each with its own layer, workspace and stream, call the backward at the same time.  The
    library's side stream and its events are shared per device, so it serialises the two callers' enqueueing; each
    must get the bits of its own single-threaded call."""
    import threading

    import torch
    names = ["ragged", "deepseek_like"]
    say(f"backward from two host threads: {names}")
    runs = [run_backward(BWD_SMALL[n], oracle, wgrad=True) for n in names]   # eager, one after the other
    outs = lambda lay: (lay.dx, lay.d_topk_w, lay.dW_gate, lay.dW_up, lay.dW_down)
    want = [[t.clone() for t in outs(r[1])] for r in runs]
    torch.cuda.synchronize()
    errors = []

    def work(i):
        try:
            lay, x, dy = runs[i][1], runs[i][2], runs[i][3]
            stream = torch.cuda.Stream()
            with torch.cuda.stream(stream):
                for _ in range(25):
                    lay.backward(x, dy)
            stream.synchronize()
        except Exception as exc:   # reported by the main thread
            errors.append(exc)

    threads = [threading.Thread(target=work, args=(i,)) for i in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join(timeout=100)
    assert not any(t.is_alive() for t in threads) and not errors, errors
    torch.cuda.synchronize()
    for i, r in enumerate(runs):
        assert all(torch.equal(a, b) for a, b in zip(want[i], outs(r[1]))), names[i]


def test_backward_empty_layer_zeroes_the_weight_gradients():
    import torch
    cfg = cfg_of(T=0, d=64, f=64)
    lay = L.MoELayer(cfg)
    z = np.zeros((cfg.E_loc, 64, 64), np.uint16)
    lay.load_weights(z, z, z)
    lay.enable_training(z, z, z, wgrad=True)
    for t in (lay.dW_gate, lay.dW_up, lay.dW_down):
        t.fill_(float("nan"))
    lay.forward_train(lay.y)   # any non-null pointers; T = 0 touches nothing
    lay.backward(lay.y, lay.y)
    torch.cuda.synchronize()
    assert all(t.abs().max().item() == 0 for t in (lay.dW_gate, lay.dW_up, lay.dW_down))


@pytest.mark.parametrize("T,E,k", [(1, 4, 2), (257, 256, 8), (300, 64, 1), (129, 640, 32), (4096, 256, 8)])
def test_route_backward(oracle, T, E, k):
    import torch
    say(f"route backward T={T} E={E} k={k}")
    rng = np.random.default_rng(T + E + k)
    logits = rng.standard_normal((T, E)).astype(np.float32) * 2
    dw = rng.standard_normal((T, k)).astype(np.float32)
    cfg = cfg_of(T=T, E=E, k=k, R=1, d=8, f=8, local_rank_begin=0, local_rank_end=1)
    lay, got = G.run_tables(cfg, logits)
    idx, w = oracle.route_topk(logits, k)
    assert np.array_equal(got["topk_idx"].reshape(T, k), idx)
    dl = torch.full((T, E), float("nan"), dtype=torch.float32, device="cuda")
    B.moe_route_backward(lay.shape, lay.topk_idx, lay.topk_w, L.to_device(dw), dl)
    torch.cuda.synchronize()
    ref = oracle.route_backward(logits, idx, dw.astype(np.float64))
    out = dl.cpu().numpy().astype(np.float64)
    mask = np.zeros((T, E), bool)
    np.put_along_axis(mask, idx.astype(np.int64), True, axis=1)
    assert np.all(out[~mask] == 0)
    assert np.abs(out - ref).max() <= 1e-5 * max(1.0, np.abs(ref).max())  # fp32 weights and sums of k <= 32 terms


def test_training_path_without_any_local_row():
    """Routing that sends nothing to this GPU's experts: y, dx, d_topk_w and every weight gradient are zero."""
    import torch
    cfg = cfg_of(T=200, d=64, f=64, E=16, k=2, R=4, local_rank_begin=1, local_rank_end=2)
    w = wl.make_workload(cfg)
    logits = w.logits.copy()
    logits[:, cfg.first_local_expert:cfg.first_local_expert + cfg.E_loc] = -50.0
    lay = L.MoELayer(cfg)
    lay.load_weights(w.W_gate, w.W_up, w.W_down)
    lay.enable_training(w.W_gate, w.W_up, w.W_down, wgrad=True)
    x, dy = L.to_device(w.x), L.to_device(dy_for(cfg))
    lay.route(L.to_device(logits))
    lay.build_dispatch()
    for t in (lay.y, lay.dx, lay.d_topk_w, lay.dW_gate, lay.dW_up, lay.dW_down):
        t.fill_(float("nan"))
    lay.forward_train(x)
    lay.backward(x, dy)
    torch.cuda.synchronize()
    for t in (lay.y, lay.dx, lay.d_topk_w, lay.dW_gate, lay.dW_up, lay.dW_down):
        assert t.float().abs().max().item() == 0
