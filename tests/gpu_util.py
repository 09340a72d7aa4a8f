"""Helpers of the GPU parity tests: run the library on a workload and bring every output back to the host."""
import numpy as np

from paper_2605_05607_amd import binding as B
from paper_2605_05607_amd import layer as L
from paper_2605_05607_amd import workloads as wl

# tolerances (stated by the target; derivation of the fp32 one: sums of <= 14336 fp32 products, reordered)
BF16_MAX_REL = 2e-2      # max |err| <= 2e-2 * max |ref|
BF16_MEAN_REL = 5e-3     # mean |err| / mean |ref| <= 5e-3
F32_MAX_REL = 1e-4       # fp32 layers: max |err| <= 1e-4 * max |ref|
W_ATOL = 1e-6            # routing weights


def run_tables(cfg, logits):
    """route + build on the GPU; returns host copies of every table."""
    import torch
    lay = L.MoELayer(cfg)
    lg = L.to_device(logits)
    lay.route(lg)
    lay.build_dispatch()
    torch.cuda.synchronize()
    return lay, tables_to_host(lay)


def tables_to_host(lay):
    s = lay.shape
    tb = lay.tables
    out = {n: getattr(tb, n).cpu().numpy() for n in ("counts", "offsets", "perm", "inv_perm", "rank_counts",
                                                      "rank_offsets", "dedup_tok", "dedup_mask", "pair_to_dedup")}
    n = s.T * s.k
    out["perm"] = out["perm"][:n]
    out["inv_perm"] = out["inv_perm"][:n]
    out["pair_to_dedup"] = out["pair_to_dedup"][:n]
    u = int(out["rank_offsets"][s.R])
    out["dedup_tok"] = out["dedup_tok"][:u]
    out["dedup_mask"] = out["dedup_mask"][:u].view(np.uint32)
    out["topk_idx"] = lay.topk_idx.cpu().numpy()[:n].reshape(s.T, s.k)
    out["topk_w"] = lay.topk_w.cpu().numpy()[:n].reshape(s.T, s.k)
    return out


def assert_tables_equal(got, oracle_mod, logits, cfg):
    idx, w = oracle_mod.route_topk(logits, cfg.k)
    assert np.array_equal(got["topk_idx"], idx), "topk_idx"
    np.testing.assert_allclose(got["topk_w"], w, atol=W_ATOL, rtol=0)
    counts, offsets, perm, inv = oracle_mod.build_tables(idx, cfg.E)
    rc, ro, tok, mask, p2d = oracle_mod.build_dedup(idx, cfg.E, cfg.R)
    for name, ref in (("counts", counts), ("offsets", offsets), ("perm", perm), ("inv_perm", inv),
                      ("rank_counts", rc), ("rank_offsets", ro), ("dedup_tok", tok), ("dedup_mask", mask),
                      ("pair_to_dedup", p2d)):
        assert np.array_equal(got[name], ref), name
    return idx, w


def check_y(y, ref, dtype):
    err = np.abs(y - ref)
    scale = np.abs(ref).max()
    if scale == 0:
        assert err.max() == 0
        return 0.0, 0.0
    if dtype == wl.BF16:
        mean_rel = err.mean() / np.abs(ref).mean()
        assert err.max() <= BF16_MAX_REL * scale, f"max err {err.max():.3e} vs scale {scale:.3e}"
        assert mean_rel <= BF16_MEAN_REL, f"mean rel err {mean_rel:.3e}"
        return err.max() / scale, mean_rel
    assert err.max() <= F32_MAX_REL * scale, f"max err {err.max():.3e} vs scale {scale:.3e}"
    return err.max() / scale, err.mean() / np.abs(ref).mean()
