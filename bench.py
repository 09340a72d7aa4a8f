"""Throughput of the whole hot path (route -> dispatch tables -> fused forward) on one MI355X.

Prints ONE JSON line.  A step is one pass of the three calls over one synthetic batch that already resides in
HBM.  The dominant kernel (both grouped GEMMs where they run as one launch, else GEMM-1: gathered gate/up grouped GEMM
with the SwiGLU epilogue) is timed with HIP events recorded on the launch stream inside the timed steps (every
fourth step, two events).  The CPU oracle is timed beside it on a bounded token sample as a reported baseline.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0      # MI355X HBM3E
MFMA_BF16_PEAK_TF = 2500.0  # dense bf16


def algorithmic_work(cfg, idx, counts_local):
    """Flops and compulsory HBM bytes of GEMM-1, GEMM-2 and combine for this routing."""
    import numpy as np
    epr = cfg.epr
    local = (idx // epr >= cfg.local_rank_begin) & (idx // epr < cfg.local_rank_end)
    P = int(local.sum())
    U_tok = int(local.any(axis=1).sum())
    n_sole = int((local.sum(axis=1) == 1).sum())  # rows that GEMM-2 writes straight to y in the output type
    ne = int((counts_local > 0).sum())  # experts whose weights have to be streamed at all
    b = 2 if cfg.dtype == 1 else 4
    d, f, T = cfg.d, cfg.f, cfg.T
    g1 = dict(flops=4.0 * P * d * f, bytes=ne * 2.0 * d * f * b + U_tok * d * b + P * f * b)
    g2 = dict(flops=2.0 * P * d * f, bytes=ne * 1.0 * d * f * b + P * f * b + (P - n_sole) * d * 4 + n_sole * d * b)
    cb = dict(flops=float(P * d), bytes=P * d * 4.0 + T * d * b)
    return P, U_tok, ne, g1, g2, cb


def kernel_source_hash():
    """sha256 over the kernel sources; stored counter readings are only valid for the sources they were taken on."""
    import hashlib
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2605_05607_amd", "csrc")
    for name in sorted(os.listdir(csrc)):
        with open(os.path.join(csrc, name), "rb") as f:
            h.update(name.encode() + b"\0" + f.read())
    return h.hexdigest()


def stored_traffic(cfg_name):
    """HBM bytes per launch of the GEMM kernel from the committed rocprofv3 counter readings (FETCH_SIZE and WRITE_SIZE in KiB,
    each scaled by what the same counter reads for a plain 1 GiB copy); None if the kernels changed since."""
    path = os.path.join(ROOT, "profiles", f"traffic_gemms_{cfg_name}.json")
    if not os.path.exists(path):
        return None
    with open(path) as f:
        rec = json.load(f)
    if rec.get("source_sha256") != kernel_source_hash():
        return None
    return (rec["fetch_size_kib"] * rec["fetch_scale"] + rec["write_size_kib"] * rec["write_scale"]) * 1024.0


def cpu_baseline(cfg, w, budget_s=12.0):
    """Oracle (as it stands) on a bounded random token sample; tokens/s on the host cores."""
    import numpy as np

    import oracle
    t0 = time.perf_counter()
    idx, tw = oracle.route_topk(w.logits, cfg.k)
    oracle.build_tables(idx, cfg.E)
    oracle.build_dedup(idx, cfg.E, cfg.R)
    t_tables = time.perf_counter() - t0
    rng = np.random.default_rng(12345)
    order = rng.permutation(cfg.T).astype(np.int32)
    threads = oracle.max_threads()
    done, spent, batch = 0, 0.0, max(threads, 16)
    while spent < budget_s and done < cfg.T:
        toks = order[done:done + batch]
        t1 = time.perf_counter()
        oracle.forward(w.x, idx, tw, w.W_gate, w.W_up, w.W_down, cfg.E, cfg.R, cfg.local_rank_begin,
                       cfg.local_rank_end, tokens=toks)
        spent += time.perf_counter() - t1
        done += len(toks)
        if spent < budget_s / 8:
            batch *= 2
    total = spent + t_tables * done / cfg.T
    model = ""
    try:
        with open("/proc/cpuinfo") as f:
            model = next((ln.split(":", 1)[1].strip() for ln in f if ln.startswith("model name")), "")
    except OSError:
        pass
    return {"value": done / total, "unit": "tokens/s", "cores": threads, "kind": "oracle", "cpu": model,
            "sample": f"{done} of {cfg.T} tokens drawn uniformly (forward {spent:.1f} s; routing+tables "
                      f"{t_tables:.2f} s for all tokens, charged pro rata)"}


def timed_steps(lay, lg, x, K):
    """K steps (route, tables, fused forward) between two synchronisations.  Returns wall ms per step, the mean
    duration of the four kernels phases of the forward call (HIP events on the launch stream), the mean duration of
    route + tables, and the per-step durations."""
    import numpy as np
    import torch

    from paper_2605_05607_amd import binding as B
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(K)]
    for row in ev:  # give every event a raw handle before the timed region
        for e in row:
            e.record()
    step_ev = [torch.cuda.Event(enable_timing=True) for _ in range(K + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    step_ev[0].record()
    for i in range(K):
        lay.route(lg)
        lay.build_dispatch()
        B.moe_fused_forward_timed(lay.shape, x, lay.topk_idx, lay.topk_w, lay.tables, lay.packed_gate_up,
                                  lay.packed_down, lay.y, lay.forward_ws, [e.cuda_event for e in ev[i]])
        step_ev[i + 1].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    phase = np.array([[ev[i][j].elapsed_time(ev[i][j + 1]) for j in range(4)] for i in range(K)])  # ms
    front_ms = float(np.mean([step_ev[i].elapsed_time(ev[i][0]) for i in range(K)]))  # route + tables
    step_ms = np.array([step_ev[i].elapsed_time(step_ev[i + 1]) for i in range(K)])
    return wall * 1e3 / K, phase.mean(axis=0), front_ms, step_ms


def timed_value(lay, lg, x, K, ev_first, ev_last, every):
    """The timed region: K steps (route, tables, fused forward) between two synchronisations.  On every `every`-th
    step the dominant kernel is bracketed by two HIP events on the launch stream (slots ev_first / ev_last of the
    five of moe_fused_forward_timed); the other steps carry no event, because every record costs the stream about
    5 us (six records per step were 4.5 % of the DeepSeek-shaped step).  Returns wall ms per step, the mean duration
    of the bracketed launch in ms, and the number of launches sampled."""
    import numpy as np
    import torch

    from paper_2605_05607_amd import binding as B
    sampled = [i for i in range(K) if i % every == 0]
    ev = {i: (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for i in sampled}
    for a, b in ev.values():  # give every event a raw handle before the timed region
        a.record()
        b.record()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(K):
        lay.route(lg)
        lay.build_dispatch()
        if i in ev:
            slots = [None] * 5
            slots[ev_first], slots[ev_last] = ev[i][0].cuda_event, ev[i][1].cuda_event
            B.moe_fused_forward_timed(lay.shape, x, lay.topk_idx, lay.topk_w, lay.tables, lay.packed_gate_up,
                                      lay.packed_down, lay.y, lay.forward_ws, slots)
        else:
            lay.forward(x)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    durs = np.array([a.elapsed_time(b) for a, b in ev.values()])
    return wall * 1e3 / K, float(durs.mean()), (len(sampled), float(np.median(durs)), float(durs.min()))


def step_statistics(lay, lg, x, K):
    """Per-step durations of K further steps (one event record per step boundary, outside the timed region)."""
    import numpy as np
    import torch
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(K + 1)]
    for e in ev:
        e.record()
    torch.cuda.synchronize()
    ev[0].record()
    for i in range(K):
        lay.step(lg, x)
        ev[i + 1].record()
    torch.cuda.synchronize()
    d = np.array([ev[i].elapsed_time(ev[i + 1]) for i in range(K)])
    return float(np.median(d)), float(d.min())


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default="deepseek_v3")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--tokens", type=int, default=0, help="override T (sweeps); 0 = the config's T")
    ap.add_argument("--topk", type=int, default=0, help="override k (sweeps)")
    ap.add_argument("--router", default="", help="override the router kind: normal | zipf | forced (sweeps)")
    ap.add_argument("--zipf-s", type=float, default=-1.0, help="override the Zipf exponent of the zipf router (sweeps)")
    ap.add_argument("--load-std", type=float, default=-1.0, help="training-load model: normal spread of the token "
                    "distribution across experts with this standard deviation (0.032 typical, 0.01-0.05 swept); "
                    "selects the loadstd router")
    ap.add_argument("--no-8x-point", action="store_true", help="skip the extra run of the layer at 8 x the tokens")
    ap.add_argument("--no-skew-points", action="store_true", help="skip the two extra ranks of the skewed routing "
                    "(counter runs: their launches would enter the per-kernel averages)")
    ap.add_argument("--no-extras", action="store_true", help="skip the untimed extras (phase-split entry points, "
                    "unfused path, reference figures)")
    ap.add_argument("--operand-probe", default="", choices=["", "normal", "one_row"],
                    help="only run the forward call 10 times in the two-launch form (to be run under rocprofv3 --pmc): "
                    "'normal' on the real tables, 'one_row' with every layout row mapped to token 0, so that GEMM-1's "
                    "A operand comes out of the caches and the difference of the two FETCH_SIZE readings is the HBM "
                    "traffic of the gathered token rows")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a 1 GiB device-to-device copy (reference point for the HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU's share of the layer; this build has no multi-GPU path (--gpus must be 1)",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    if args.copy_calibration:
        torch.cuda.set_device(0)
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")  # 1 GiB
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes_read": src.numel() * 4, "copy_bytes_written": dst.numel() * 4, "launches": 5}))
        return

    from paper_2605_05607_amd import binding as B
    from paper_2605_05607_amd import layer as L
    from paper_2605_05607_amd import workloads as wl

    cfg = wl.CONFIGS[args.config]
    swept = bool(args.tokens or args.topk or args.router or args.zipf_s >= 0 or args.load_std >= 0)
    if args.tokens:
        cfg = cfg.scaled(T=args.tokens)
    if args.topk:
        cfg = cfg.scaled(k=args.topk)
    if args.router:
        cfg = cfg.scaled(router=args.router)
    if args.zipf_s >= 0:
        cfg = cfg.scaled(zipf_s=args.zipf_s)
    if args.load_std >= 0:
        cfg = cfg.scaled(router="loadstd", load_std=args.load_std)
    torch.cuda.set_device(0)
    w = wl.make_workload(cfg)
    lay = L.MoELayer(cfg)
    lay.load_weights(w.W_gate, w.W_up, w.W_down)
    x, lg = L.to_device(w.x), L.to_device(w.logits)
    torch.cuda.synchronize()

    for _ in range(args.warmup):
        lay.step(lg, x)
    torch.cuda.synchronize()

    if args.operand_probe:
        if args.operand_probe == "one_row":
            lay.tables.perm.zero_()  # every layout row now holds pair 0, i.e. token 0 (results are meaningless)
        for _ in range(10):
            lay.forward_two_launch(x)
        torch.cuda.synchronize()
        print(json.dumps({"operand_probe": args.operand_probe, "config": cfg.name, "forward_calls": 10}))
        return

    K = args.steps
    # Dominant kernel: where the library runs GEMM-1 and GEMM-2 as one launch (resident workgroups, tile-level
    # hand-over; see moe_forward_gemm_launches) that launch, with the algorithmic work of both GEMMs; otherwise the
    # GEMM-1 launch.  Duration = time between the HIP events recorded before and after it on the launch stream,
    # on every fourth step of the timed region.
    one_launch = B.moe_forward_gemm_launches(lay.shape) == 1
    every = 4 if K >= 20 else 1
    # phase breakdown: an untimed loop with all five events of moe_fused_forward_timed on every step (run first:
    # the clocks of a box that has just started working take some tens of steps to settle)
    ms_instr, (prep_ms, g1_ms, g2_ms, cb_ms), front_ms, step_ms = timed_steps(lay, lg, x, 20)
    ms_per_step, gk_ms, n_sampled = timed_value(lay, lg, x, K, 1, 3 if one_launch else 2, every)
    ms_median, ms_min = step_statistics(lay, lg, x, K)

    idx = lay.topk_idx.cpu().numpy().reshape(cfg.T, cfg.k)
    counts = lay.tables.counts.cpu().numpy()
    counts_local = counts[cfg.first_local_expert:cfg.first_local_expert + cfg.E_loc]
    P, U_tok, ne, g1, g2, cb = algorithmic_work(cfg, idx, counts_local)

    gk = {k: g1[k] + g2[k] for k in g1} if one_launch else g1
    t_mfma = gk["flops"] / (MFMA_BF16_PEAK_TF * 1e12)
    t_hbm = gk["bytes"] / (HBM_PEAK_GBS * 1e9)
    if t_hbm >= t_mfma:
        roof = {"bound": "hbm", "achieved": gk["bytes"] / (gk_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s"}
    else:
        roof = {"bound": "mfma", "achieved": gk["flops"] / (gk_ms * 1e-3) / 1e12, "peak": MFMA_BF16_PEAK_TF,
                "unit": "TFLOP/s"}
    roof["frac"] = roof["achieved"] / roof["peak"]
    roof["traffic"] = None if swept else stored_traffic(cfg.name)
    roof["traffic_unit"] = "bytes per launch"
    roof["algorithmic"] = gk["bytes"] if roof["bound"] == "hbm" else gk["flops"]
    roof["kernel"] = ("gemm_bf16_pipeline_kernel (gathered gate/up GEMM + SwiGLU, then down GEMM x gate weight, one "
                      "launch)" if one_launch else
                      ("gemm_bf16_kernel<true, false, false>" if cfg.dtype == wl.BF16 else "gemm_f32_kernel<true>")
                      + " (GEMM-1: gathered gate/up GEMM + SwiGLU)")
    roof["avg_launch_ms"] = gk_ms
    roof["launches_sampled"], roof["median_launch_ms"], roof["min_launch_ms"] = n_sampled

    out = {
        "metric": "fused MoE layer tokens/s on 1 MI355X", "value": cfg.T / (ms_per_step * 1e-3), "unit": "tokens/s",
        "n_gpus": 1, "steps": K, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "ms_per_step_median": ms_median, "ms_per_step_min": ms_min, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16" if cfg.dtype == wl.BF16 else "f32",
        "data": "synthetic",
        "config": {"workload": f"{cfg.name}: T={cfg.T} d={cfg.d} f={cfg.f} E={cfg.E} local={cfg.E_loc} k={cfg.k} "
                               f"R={cfg.R} router={cfg.router}", "step": "moe_route_topk + moe_build_dispatch + "
                   "moe_fused_forward", "weights": "re-tiled once by moe_pack_weights (untimed, static)",
                   "local_pairs_P": P, "tokens_with_local_expert": U_tok, "nonempty_local_experts": ne,
                   "rows_per_expert_max": int(counts_local.max()), "seed": cfg.seed,
                   "step_statistics": "ms_per_step_median / _min: a second loop of the same K steps with one event "
                                      "record per step boundary (outside the timed region)"},
        "roofline": roof,
        "phases_ms": {"note": "separate untimed loop of 20 steps with six event records per step (they slow the step itself), run before the timed region",
                      "instrumented_step": ms_instr, "route_and_tables": front_ms, "tile_table": float(prep_ms), "gemms": float(g1_ms + g2_ms),
                      "combine": float(cb_ms), "gemm_launches": 1 if one_launch else 2},
        "gemm_phase": {"flops": g1["flops"] + g2["flops"],
                       "mfma_tflops": (g1["flops"] + g2["flops"]) / ((g1_ms + g2_ms) * 1e-3) / 1e12,
                       "mfma_frac_of_peak": (g1["flops"] + g2["flops"]) / ((g1_ms + g2_ms) * 1e-3) / 1e12
                       / MFMA_BF16_PEAK_TF,
                       "hbm_gbs": (g1["bytes"] + g2["bytes"]) / ((g1_ms + g2_ms) * 1e-3) / 1e9,
                       "hbm_frac_of_peak": (g1["bytes"] + g2["bytes"]) / ((g1_ms + g2_ms) * 1e-3) / 1e9 / HBM_PEAK_GBS,
                       "mfma_ceiling_if_hbm_bound": min(1.0, (g1["flops"] + g2["flops"]) / (MFMA_BF16_PEAK_TF * 1e12)
                                                        / ((g1["bytes"] + g2["bytes"]) / (HBM_PEAK_GBS * 1e9)))},
    }
    out["gemm_phase"]["mfma_frac_of_ceiling"] = (out["gemm_phase"]["mfma_frac_of_peak"]
                                                 / out["gemm_phase"]["mfma_ceiling_if_hbm_bound"])
    if args.no_extras:
        print(json.dumps(out))
        return

    # ---- untimed extras: Dispatch and Combine on their own (phase-split entry points) and the unfused path ----
    def timed(fn, reps):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    b = 2 if cfg.dtype == wl.BF16 else 4
    P_cap = cfg.T * min(cfg.k, cfg.E_loc)
    # Dispatch on its own: every needed token row read once, every layout row written.  Timed twice: on one pair of
    # buffers (x and xs together fit the 256 MB Infinity Cache, as x does right after the layer that produced it) and
    # rotating over pairs whose bytes together exceed that cache several times (every read from HBM).
    disp_bytes = U_tok * cfg.d * b + P * cfg.d * b
    live = (cfg.T + max(1, P)) * cfg.d * b  # bytes one call touches: x and the P layout rows it writes
    npair = max(2, min(16, -(-(768 << 20) // live)))
    xs_bufs = [torch.empty((max(1, P), cfg.d), dtype=lay.elt_dtype, device="cuda") for _ in range(npair)]
    x_bufs = [x] + [x.clone() for _ in range(npair - 1)]
    t_disp_warm = timed(lambda: B.moe_dispatch_gather(lay.shape, x, lay.tables, xs_bufs[0]), 20)
    dturn = [0]

    def dispatch_next():
        dturn[0] = (dturn[0] + 1) % npair
        B.moe_dispatch_gather(lay.shape, x_bufs[dturn[0]], lay.tables, xs_bufs[dturn[0]])

    t_disp = timed(dispatch_next, 4 * npair)
    out["dispatch_phase"] = {"entry": "moe_dispatch_gather", "ms": t_disp, "hbm_gbs": disp_bytes / (t_disp * 1e-3) / 1e9,
                             "hbm_frac_of_peak": disp_bytes / (t_disp * 1e-3) / 1e9 / HBM_PEAK_GBS,
                             "ms_same_buffers": t_disp_warm,
                             "hbm_frac_of_peak_same_buffers": disp_bytes / (t_disp_warm * 1e-3) / 1e9 / HBM_PEAK_GBS,
                             "buffer_pairs_rotated": npair,
                             "bytes": disp_bytes, "bytes_without_dedup": 2 * P * cfg.d * b}
    del xs_bufs, x_bufs
    # Combine on its own: every weighted row read, every token row written.  (Inside the fused call GEMM-2 writes
    # the rows of tokens with a single local slot itself, so the fused combine kernel moves less than this.)
    # Timed twice: on one buffer (rows partly resident in the 256 MB Infinity Cache, as they are right after GEMM-2
    # wrote them) and rotating over buffers whose live rows together exceed that cache (every read from HBM).
    live = max(1, P) * cfg.d * 4
    nbuf = max(2, min(8, -(-(768 << 20) // live)))
    bufs = [torch.randn((max(1, P), cfg.d), dtype=torch.float32, device="cuda") for _ in range(nbuf)]
    y2 = torch.empty_like(lay.y)
    t_warm = timed(lambda: B.moe_combine_reduce(lay.shape, bufs[0], lay.topk_idx, lay.tables, y2), 20)
    turn = [0]

    def combine_next():
        turn[0] = (turn[0] + 1) % nbuf
        B.moe_combine_reduce(lay.shape, bufs[turn[0]], lay.topk_idx, lay.tables, y2)

    t_comb = timed(combine_next, 4 * nbuf)
    out["combine_phase"] = {"entry": "moe_combine_reduce", "ms": t_comb, "bytes": cb["bytes"],
                            "hbm_gbs": cb["bytes"] / (t_comb * 1e-3) / 1e9,
                            "hbm_frac_of_peak": cb["bytes"] / (t_comb * 1e-3) / 1e9 / HBM_PEAK_GBS,
                            "ms_same_buffer": t_warm,
                            "hbm_frac_of_peak_same_buffer": cb["bytes"] / (t_warm * 1e-3) / 1e9 / HBM_PEAK_GBS,
                            "buffers_rotated": nbuf}
    del bufs
    del y2
    lay_u = L.MoELayer(cfg, unfused=True)
    lay_u.packed_gate_up, lay_u.packed_down = lay.packed_gate_up, lay.packed_down
    lay_u.route(lg)
    lay_u.build_dispatch()
    t_unf = timed(lambda: lay_u.forward_unfused(x), 5)
    t_fus = timed(lambda: lay.forward(x), 5)
    out["unfused_comparison"] = {"fused_forward_ms": t_fus, "unfused_forward_ms": t_unf,
                                 "note": "unfused = gather copy + same grouped GEMMs + fp32 atomic scatter-add + cast"}
    # The two forms of the GEMM-1 => GEMM-2 hand-over side by side (the library picks by shape), and the two GEMMs
    # timed apart in the two-launch form.
    ev2 = [torch.cuda.Event(enable_timing=True) for _ in range(5)]
    for e in ev2:
        e.record()
    t_two = timed(lambda: lay.forward_two_launch(x), 5)
    lay.forward_two_launch(x, [e.cuda_event for e in ev2])
    torch.cuda.synchronize()
    out["hand_over_comparison"] = {"default_gemm_launches": 1 if one_launch else 2, "two_launch_forward_ms": t_two,
                                   "gemm1_ms": ev2[1].elapsed_time(ev2[2]), "gemm2_ms": ev2[2].elapsed_time(ev2[3])}
    if cfg.dtype == wl.BF16:
        # the three forms in rotating order (the clock drifts with load), median of the rounds
        forms = [("two_launch_forward_ms", lay.forward_two_launch), ("one_launch_forward_ms", lay.forward_one_launch),
                 ("resident_with_combine_forward_ms", lay.forward_resident)]
        rounds = {k: [] for k, _ in forms}
        for _ in range(6):
            forms = forms[1:] + forms[:1]
            for key, fn in forms:
                rounds[key].append(timed(lambda: fn(x), 5))
        for key, v in rounds.items():
            out["hand_over_comparison"][key] = float(np.median(v))
        out["hand_over_comparison"]["note"] = ("forward call = tile table + GEMMs + Combine; resident_with_combine = "
                                               "GEMM-1, GEMM-2 and Combine in one launch (moe_fused_forward_resident)")
    del lay_u
    # The gate network ahead of the routing (not part of the timed step: the logits are an input of the layer):
    # a skinny product bound by reading x once.
    W_r = (torch.randn((cfg.E, cfg.d), dtype=torch.float32, device="cuda") * cfg.d ** -0.5).to(lay.elt_dtype)
    lg2 = torch.empty((cfg.T, cfg.E), dtype=torch.float32, device="cuda")
    ws_r = torch.empty((B.moe_router_workspace_bytes(lay.shape),), dtype=torch.uint8, device="cuda")
    t_gate = timed(lambda: B.moe_router_logits(lay.shape, x, W_r, lg2, ws_r), 20)
    gate_bytes = (cfg.T * cfg.d + cfg.E * cfg.d) * b + cfg.T * cfg.E * 4
    out["router_logits"] = {"entry": "moe_router_logits", "ms": t_gate, "bytes": gate_bytes,
                            "hbm_gbs": gate_bytes / (t_gate * 1e-3) / 1e9,
                            "hbm_frac_of_peak": gate_bytes / (t_gate * 1e-3) / 1e9 / HBM_PEAK_GBS}
    # gate network and routing in one call (the logits never reach memory), against the two calls it replaces
    ws_x = torch.empty((B.moe_route_from_x_workspace_bytes(lay.shape),), dtype=torch.uint8, device="cuda")
    idx_x, w_x = torch.empty_like(lay.topk_idx), torch.empty_like(lay.topk_w)
    t_fused = timed(lambda: B.moe_route_from_x(lay.shape, x, W_r, None, idx_x, w_x, ws_x), 20)

    def two_calls():
        B.moe_router_logits(lay.shape, x, W_r, lg2, ws_r)
        B.moe_route_topk(lay.shape, lg2, idx_x, w_x)

    t_two_calls = timed(two_calls, 20)
    x_bytes = (cfg.T * cfg.d + cfg.E * cfg.d) * b + 2 * cfg.T * cfg.k * 4
    out["route_from_x"] = {"entry": "moe_route_from_x", "ms": t_fused, "bytes": x_bytes,
                           "hbm_gbs": x_bytes / (t_fused * 1e-3) / 1e9,
                           "hbm_frac_of_peak": x_bytes / (t_fused * 1e-3) / 1e9 / HBM_PEAK_GBS,
                           "ms_router_logits_then_route_topk": t_two_calls}
    del W_r, lg2, ws_r, ws_x, idx_x, w_x
    # The same step with the FP8 (E4M3) form of the expert GEMMs (weights quantised once, untimed; x quantised inside
    # the step): half the weight bytes, the same number of matrix-core instructions.  Not `value`: the metric is
    # the bf16 layer.
    if cfg.dtype == wl.BF16 and cfg.d % 16 == 0 and cfg.f % 16 == 0:
        lay.load_weights_fp8(w.W_gate, w.W_up, w.W_down, wl.fp8_h_scale(cfg))

        def step_fp8(events=None):
            lay.route(lg)
            lay.build_dispatch()
            lay.forward_fp8(x, events)

        t_fp8 = timed(step_fp8, 10)
        ev8 = [torch.cuda.Event(enable_timing=True) for _ in range(5)]
        for e in ev8:
            e.record()
        step_fp8([e.cuda_event for e in ev8])
        torch.cuda.synchronize()
        g8_ms = ev8[1].elapsed_time(ev8[3])
        fp8_bytes = (g1["bytes"] + g2["bytes"]) - ne * 3 * cfg.d * cfg.f  # weights, x and h are one byte each ...
        fp8_bytes -= U_tok * cfg.d + 2 * P * cfg.f                        # ... instead of two
        out["fp8_gemms"] = {"entry": "moe_fp8_fused_forward", "ms_per_step": t_fp8,
                            "tokens_per_s": cfg.T / (t_fp8 * 1e-3),
                            "quantise_x_and_tile_table_ms": ev8[0].elapsed_time(ev8[1]), "gemms_ms": g8_ms,
                            "combine_ms": ev8[3].elapsed_time(ev8[4]),
                            "gemm_tflops": (g1["flops"] + g2["flops"]) / (g8_ms * 1e-3) / 1e12,
                            "gemm_bytes": fp8_bytes, "hbm_gbs": fp8_bytes / (g8_ms * 1e-3) / 1e9,
                            "hbm_frac_of_peak": fp8_bytes / (g8_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                            "speedup_vs_bf16_step": ms_per_step / t_fp8}
        del lay.fp8_gate_up, lay.fp8_down, lay.fp8_ws
        # context: the vendor library's dense FP8 product of GEMM-1's size on this machine (not part of the path)
        try:
            Mref = max(256, -(-P // 256) * 256)
            a8 = torch.randn((Mref, cfg.d), device="cuda").to(torch.float8_e4m3fn)
            b8 = torch.randn((2 * cfg.f, cfg.d), device="cuda").to(torch.float8_e4m3fn).t()  # column-major operand
            one = torch.ones((), dtype=torch.float32, device="cuda")
            t_ref8 = timed(lambda: torch._scaled_mm(a8, b8, scale_a=one, scale_b=one, out_dtype=torch.bfloat16), 10)
            out["fp8_gemms"]["dense_fp8_gemm_reference"] = {
                "what": "torch._scaled_mm (hipBLASLt) e4m3, one dense product", "M": Mref, "N": 2 * cfg.f, "K": cfg.d,
                "ms": t_ref8, "tflops": 2.0 * Mref * 2 * cfg.f * cfg.d / (t_ref8 * 1e-3) / 1e12}
            del a8, b8
        except Exception as exc:  # the reference figure is optional
            out["fp8_gemms"]["dense_fp8_gemm_reference"] = {"error": str(exc)[:200]}
    # Training path (not `value`): the forward that keeps g, u and the weighted rows, then the backward pass (dx, gate-
    # weight gradients and the three weight gradients).  Flops: forward 6 P d f, backward 12 P d f.
    if cfg.dtype == wl.BF16 and cfg.f % 64 == 0:
        lay.enable_training(w.W_gate, w.W_up, w.W_down, wgrad=True)
        dy = torch.randn((cfg.T, cfg.d), dtype=torch.float32, device="cuda").to(torch.bfloat16)
        med3 = lambda fn: sorted(timed(fn, 10) for _ in range(3))[1]  # the clock drifts for a while after a change of load
        t_ft = med3(lambda: lay.forward_train(x))
        lay.backward(x, dy)  # first call: one-off attribute changes of its kernels
        t_bw = med3(lambda: lay.backward(x, dy))
        dWg, dWu, dWd = lay.dW_gate, lay.dW_up, lay.dW_down
        lay.dW_gate = lay.dW_up = lay.dW_down = None
        t_bw_tok = med3(lambda: lay.backward(x, dy))
        lay.dW_gate, lay.dW_up, lay.dW_down = dWg, dWu, dWd
        fl = 2.0 * P * cfg.d * cfg.f
        wg_bytes = 3.0 * cfg.E_loc * cfg.d * cfg.f * 2  # every weight gradient is written in full
        out["training"] = {"entries": "moe_fused_forward_train, moe_fused_backward", "forward_train_ms": t_ft,
                           "backward_ms": t_bw, "backward_without_weight_gradients_ms": t_bw_tok,
                           "weight_gradients_ms": t_bw - t_bw_tok,
                           "forward_plus_backward_ms": t_ft + t_bw,
                           "backward_tflops": 6 * fl / (t_bw * 1e-3) / 1e12,
                           "dgrad_tflops": 3 * fl / (t_bw_tok * 1e-3) / 1e12,
                           "wgrad_tflops": 3 * fl / ((t_bw - t_bw_tok) * 1e-3) / 1e12,
                           "wgrad_bytes_written": wg_bytes,
                           "wgrad_write_gbs": wg_bytes / ((t_bw - t_bw_tok) * 1e-3) / 1e9}
        for name in ("packed_down_t", "packed_gate_up_t", "kept", "backward_ws", "dx", "d_topk_w", "dW_gate", "dW_up",
                     "dW_down"):
            delattr(lay, name)
        del dy, dWg, dWu, dWd
    # Two more ranks of the same skewed routing (DeepSeek-shaped workload only): the rank that receives the most pairs
    # under this seed, and the "hot rank" corner (popular experts first: nearly every pair on rank 0).  Same shapes
    # and the same packed weight buffers (their values do not matter for the time); labelled extras, not `value`.
    if cfg.name == "deepseek_v3" and not swept and not args.no_skew_points:
        rank_pairs = counts.reshape(cfg.R, cfg.epr).sum(axis=1)
        pts = {}
        for label, cfg_x in (("max_load_rank", cfg.scaled(local_rank_begin=int(rank_pairs.argmax()),
                                                          local_rank_end=int(rank_pairs.argmax()) + 1)),
                             ("hot_rank", cfg.scaled(router="zipf_hot", local_rank_begin=0, local_rank_end=1))):
            wx = w if cfg_x.router == cfg.router else wl.make_workload(cfg_x, weights=False)
            lay_x = L.MoELayer(cfg_x)
            lay_x.packed_gate_up, lay_x.packed_down = lay.packed_gate_up, lay.packed_down
            lgx = lg if wx is w else L.to_device(wx.logits)
            for _ in range(40):  # (the clocks take some tens of steps to settle after a change of load)
                lay_x.step(lgx, x)
            t_x = timed(lambda: lay_x.step(lgx, x), 10)
            cx = lay_x.tables.counts.cpu().numpy()[cfg_x.first_local_expert:cfg_x.first_local_expert + cfg_x.E_loc]
            Px = int(cx.sum())
            pts[label] = {"local_rank": cfg_x.local_rank_begin, "router": cfg_x.router, "local_pairs_P": Px,
                          "rows_per_expert_max": int(cx.max()), "nonempty_local_experts": int((cx > 0).sum()),
                          "gemm_launches": B.moe_forward_gemm_launches(lay_x.shape), "ms_per_step": t_x,
                          "tokens_per_s": cfg.T / (t_x * 1e-3),
                          "mfma_tflops_whole_step": 6.0 * Px * cfg.d * cfg.f / (t_x * 1e-3) / 1e12}
            del lay_x
        out["skew_points"] = pts
        # The balanced load of the paper's training runs on the same shape (Table I Large: every expert equally
        # likely; all 32 local experts stay below one M tile, so the GEMM launch streams every expert's weights once):
        # the regime in which this launch is bound by HBM throughout.  A labelled extra, not `value`.
        cfg_n = cfg.scaled(router="normal")
        wn = wl.make_workload(cfg_n, weights=False)
        lay_n = L.MoELayer(cfg_n)
        lay_n.packed_gate_up, lay_n.packed_down = lay.packed_gate_up, lay.packed_down
        lgn = L.to_device(wn.logits)
        for _ in range(60):  # (the clocks take some tens of steps to settle after a change of load)
            lay_n.step(lgn, x)
        one_n = B.moe_forward_gemm_launches(lay_n.shape) == 1
        # as for `value`: the GEMM launch (both GEMMs if they share one, else both brackets) on every fourth step
        ms_n, gemm_n, _ = timed_value(lay_n, lgn, x, 40, 1, 3, 4)
        idx_n = lay_n.topk_idx.cpu().numpy().reshape(cfg_n.T, cfg_n.k)
        cn = lay_n.tables.counts.cpu().numpy()[cfg_n.first_local_expert:cfg_n.first_local_expert + cfg_n.E_loc]
        Pn, Un, nen, g1w, g2w, _ = algorithmic_work(cfg_n, idx_n, cn)
        gemm_n = float(gemm_n)
        out["balanced_load_point"] = {
            "workload": "deepseek_v3 shape with router=normal (Table I Large, k = 8)", "local_pairs_P": Pn,
            "rows_per_expert_max": int(cn.max()), "gemm_launches": 1 if one_n else 2,
            "ms_per_step": ms_n, "tokens_per_s": cfg.T / (ms_n * 1e-3), "gemm_ms": gemm_n,
            "gemm_bytes": g1w["bytes"] + g2w["bytes"],
            "hbm_gbs": (g1w["bytes"] + g2w["bytes"]) / (gemm_n * 1e-3) / 1e9,
            "hbm_frac_of_peak": (g1w["bytes"] + g2w["bytes"]) / (gemm_n * 1e-3) / 1e9 / HBM_PEAK_GBS}
        del lay_n, lgn, wn
    # The whole step captured once in a HIP graph and replayed (what a serving loop would do): fewer host launches.
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        lay.step(lg, x)
    t_graph = timed(graph.replay, 20)
    out["graph_replay"] = {"ms_per_step": t_graph, "tokens_per_s": cfg.T / (t_graph * 1e-3),
                           "note": "route + tables + fused forward replayed from one captured HIP graph; `value` is "
                                   "measured on eager launches because the per-kernel events live there"}
    del graph
    # The same layer at 8 x the tokens (for the DeepSeek-shaped workload: what one GPU of an 8-way expert-parallel
    # group sees when every GPU contributes T tokens): enough rows per expert for the GEMMs to be compute-bound.
    if cfg.dtype == wl.BF16 and not swept and not args.no_8x_point and cfg.T * 8 * cfg.d * 2 <= 1 << 30:
        cfg8 = cfg.scaled(T=8 * cfg.T)
        w8 = wl.make_workload(cfg8, weights=False)
        lay8 = L.MoELayer(cfg8)
        lay8.packed_gate_up, lay8.packed_down = lay.packed_gate_up, lay.packed_down
        x8, lg8 = L.to_device(w8.x), L.to_device(w8.logits)
        for _ in range(12):
            lay8.step(lg8, x8)
        ms8, (_, g1_8, g2_8, _), _, _ = timed_steps(lay8, lg8, x8, 8)
        idx8 = lay8.topk_idx.cpu().numpy().reshape(cfg8.T, cfg8.k)
        local8 = (idx8 // cfg8.epr >= cfg8.local_rank_begin) & (idx8 // cfg8.epr < cfg8.local_rank_end)
        P8 = int(local8.sum())
        fl8 = 6.0 * P8 * cfg8.d * cfg8.f
        out["compute_bound_point"] = {"workload": f"{cfg.name} at T={cfg8.T} (8 x), same weights", "local_pairs_P": P8,
                                      "ms_per_step": ms8, "tokens_per_s": cfg8.T / (ms8 * 1e-3),
                                      "gemm_ms": float(g1_8 + g2_8),
                                      "mfma_tflops": fl8 / ((g1_8 + g2_8) * 1e-3) / 1e12,
                                      "mfma_frac_of_peak": fl8 / ((g1_8 + g2_8) * 1e-3) / 1e12 / MFMA_BF16_PEAK_TF}
        del lay8, x8, lg8, w8
    # Context for the bandwidth fractions: a plain 1 GiB device copy on this machine (reads + writes counted).
    src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
    dst = torch.empty_like(src)
    t_copy = timed(lambda: dst.copy_(src), 10)
    out["copy_reference"] = {"what": "torch 1 GiB device-to-device copy", "ms": t_copy,
                             "hbm_gbs": 2.0 * src.numel() * 4 / (t_copy * 1e-3) / 1e9}
    del src, dst
    # Context for the matrix-core fractions: what this box's matrix cores sustain on register operands (no loads at
    # all; pseudo-random values), one workgroup of 8 waves per CU as the GEMM kernels run.
    sink = torch.empty(256 * 512, dtype=torch.float32, device="cuda")
    B.moe_probe_mfma_rate(256, 2000, sink)  # warm-up
    probe_flops = [0.0]

    def probe():
        probe_flops[0] = B.moe_probe_mfma_rate(256, 20000, sink)

    t_probe = timed(probe, 3)
    out["mfma_rate_probe"] = {"what": "8 waves per CU, 8 independent bf16 32x32x16 instructions per round, register "
                                      "operands", "ms": t_probe, "tflops": probe_flops[0] / (t_probe * 1e-3) / 1e12}
    roof["frac_of_probed_mfma_rate"] = (gk["flops"] / (gk_ms * 1e-3) / 1e12) / out["mfma_rate_probe"]["tflops"]
    del sink
    # Context for the matrix-core fractions: what the vendor library's dense bf16 GEMM reaches on this very box
    # with the same kind of data (random normal), on a problem as large as this layer's GEMM-1 would be if it were
    # one dense product.  Not part of the path, not timed into `value`.
    if cfg.dtype == wl.BF16:
        Mref = max(256, -(-P // 256) * 256)
        a = torch.randn((Mref, cfg.d), dtype=torch.bfloat16, device="cuda")
        bmat = torch.randn((cfg.d, 2 * cfg.f), dtype=torch.bfloat16, device="cuda")
        t_ref = timed(lambda: torch.matmul(a, bmat), 10)
        out["dense_gemm_reference"] = {"what": "torch.matmul (hipBLASLt) bf16, one dense product", "M": Mref,
                                       "N": 2 * cfg.f, "K": cfg.d, "ms": t_ref,
                                       "tflops": 2.0 * Mref * 2 * cfg.f * cfg.d / (t_ref * 1e-3) / 1e12}
        del a, bmat
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, w)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
