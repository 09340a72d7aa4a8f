"""The entry point that allocates nothing (static device scratch) against the workspace form of the same call,
through the C ABI: every table bit for bit, on two calls in a row, the second on a smaller input."""
import numpy as np
import pytest

import gpu_util as G
from paper_2605_05607_amd import binding as B
from paper_2605_05607_amd import layer as L
from paper_2605_05607_amd import workloads as wl

pytestmark = pytest.mark.gpu

NAMES = ("counts", "offsets", "perm", "inv_perm", "rank_counts", "rank_offsets", "dedup_tok", "dedup_mask",
         "pair_to_dedup")


def tables_of(cfg, logits, noalloc):
    import torch
    lay = L.MoELayer(cfg)
    lay.route(L.to_device(logits))
    for n in NAMES:  # whatever the call does not write must not look like a result
        getattr(lay.tables, n).fill_(-7)
    if noalloc:
        B.moe_build_dispatch_noalloc(lay.shape, lay.topk_idx, lay.tables)
    else:
        lay.build_dispatch()
    torch.cuda.synchronize()
    return G.tables_to_host(lay)


def test_noalloc_dispatch_matches_workspace_form_twice(oracle):
    import torch
    big = wl.CONFIGS["deepseek_v3"]
    small = wl.MoEConfig("t", T=333, d=8, f=8, E=48, k=6, R=8, local_rank_begin=0, local_rank_end=8, dtype=wl.BF16,
                         router="zipf", seed=5)
    before = torch.cuda.memory_allocated()
    for cfg in (big, small):  # the second call finds the first one's histograms in the static scratch
        print(f"no-alloc dispatch T={cfg.T} E={cfg.E} k={cfg.k} R={cfg.R}", flush=True)
        w = wl.make_workload(cfg, weights=False)
        want = tables_of(cfg, w.logits, noalloc=False)
        got = tables_of(cfg, w.logits, noalloc=True)
        for n in NAMES + ("topk_idx",):
            assert np.array_equal(got[n], want[n]), n
        # and both equal the oracle's tables
        G.assert_tables_equal(got, oracle, w.logits, cfg)
    assert torch.cuda.memory_allocated() <= before + (1 << 20)  # nothing of the calls' own stays allocated


def test_noalloc_dispatch_empty_layer_and_limit():
    import torch
    cfg = wl.MoEConfig("t", T=0, d=8, f=8, E=16, k=2, R=4, local_rank_begin=0, local_rank_end=4, dtype=wl.BF16,
                       router="normal", seed=1)
    lay = L.MoELayer(cfg)
    lay.tables.counts.fill_(9)
    lay.tables.offsets.fill_(9)
    B.moe_build_dispatch_noalloc(lay.shape, lay.topk_idx, lay.tables)
    torch.cuda.synchronize()
    assert lay.tables.counts.abs().sum().item() == 0 and lay.tables.offsets.abs().sum().item() == 0
    over = wl.MoEConfig("t", T=8, d=8, f=8, E=1024, k=2, R=1, local_rank_begin=0, local_rank_end=1, dtype=wl.BF16,
                        router="normal", seed=1)
    lay = L.MoELayer(over)
    with pytest.raises(B.MoeError) as err:
        B.moe_build_dispatch_noalloc(lay.shape, lay.topk_idx, lay.tables)
    assert err.value.status == B.MOE_ERR_UNSUPPORTED
