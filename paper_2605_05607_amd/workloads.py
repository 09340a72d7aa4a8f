"""Seeded synthetic MoE-layer workloads (inputs only; none of the method's arithmetic lives here).

The shapes follow the model table of the paper's methodology section (hidden size, MoE hidden size,
number of experts, top-k; Table I "Large" = DeepSeek-V3, and the discussion section's table for
GPT-OSS-120B and Qwen3-235B) and its load models (near-uniform load for training, power-law skew for
inference).  Every array is produced on the host from ``numpy.random.SeedSequence`` children, so the
same bits reach the CPU oracle and the GPU library.  The generator knows nothing about routing,
dispatch tables or expert computation: router logits are an *input* of the layer.

Large tensors are drawn in fixed-size chunks, each chunk from its own child seed, so the result does
not depend on how many threads fill it.
"""
from __future__ import annotations

import dataclasses
from concurrent.futures import ThreadPoolExecutor
from typing import Optional

import numpy as np

F32 = 0
BF16 = 1

_CHUNK = 1 << 22  # elements per independently seeded chunk


@dataclasses.dataclass(frozen=True)
class MoEConfig:
    """One synthetic layer.  ``router`` selects how the logits are made:

    ``"xwr"``     logits = x @ W_r with W_r ~ N(0, 0.02^2), computed once here in fp32
    ``"normal"``  logits ~ N(0, 1)                          (uniform expected load)
    ``"zipf"``    N(0, 1) + bias[e], bias[e] = -s * ln(1 + pi(e)), pi a seeded permutation of the experts
    ``"forced"``  N(0, 1); a Bernoulli(force_p) subset of tokens gets +16 on every logit of one uniformly
                  drawn virtual rank, so all of its top-k picks fall on that rank
    ``"zipf_hot"`` as ``"zipf"`` with the identity permutation: the popular experts are the first ones, so nearly all
                  pairs land on rank 0 (the "hot rank" corner of the skewed load)
    ``"loadstd"`` the training-load model of the evaluation (token distribution across experts ~ normal, quoted by its
                  standard deviation, 0.032 for a typical job, swept over 0.01-0.05): expert load fractions
                  p_e = (1 + c z_e) / E with z_e ~ N(0, 1) and c = load_std / 0.125 (the figure is quoted for groups of
                  eight experts, where the mean fraction is 1/8), clipped at 0.05 / E and renormalised; logits =
                  ln p_e + Gumbel noise, so the k picks of a token are draws without replacement in proportion to p
    """

    name: str
    T: int
    d: int
    f: int
    E: int
    k: int
    R: int
    local_rank_begin: int
    local_rank_end: int
    dtype: int
    router: str
    seed: int
    zipf_s: float = 1.1
    force_p: float = 0.1
    load_std: float = 0.032

    @property
    def epr(self) -> int:
        return self.E // self.R

    @property
    def E_loc(self) -> int:
        return (self.local_rank_end - self.local_rank_begin) * self.epr

    @property
    def first_local_expert(self) -> int:
        return self.local_rank_begin * self.epr

    def scaled(self, **kw) -> "MoEConfig":
        return dataclasses.replace(self, **kw)


CONFIGS = {
    "tiny": MoEConfig("tiny", T=256, d=512, f=1024, E=8, k=2, R=4, local_rank_begin=0, local_rank_end=4,
                      dtype=F32, router="xwr", seed=1000),
    # local rank 4 is the rank that hosts the most popular expert under this seed's Zipf permutation: its load
    # (about 5.3 k of the 32768 pairs, one expert with ~4 k rows, a dozen empty experts) is the one closest to the
    # mean rank load T*k/R = 4096; the other ranks range from 0.1 k to 7 k pairs.
    "deepseek_v3": MoEConfig("deepseek_v3", T=4096, d=7168, f=2048, E=256, k=8, R=8, local_rank_begin=4,
                             local_rank_end=5, dtype=BF16, router="zipf", seed=1001),
    "qwen3": MoEConfig("qwen3", T=8192, d=4096, f=1536, E=128, k=8, R=8, local_rank_begin=0,
                       local_rank_end=1, dtype=BF16, router="normal", seed=1002),
    "mixtral": MoEConfig("mixtral", T=2048, d=4096, f=14336, E=8, k=2, R=8, local_rank_begin=0,
                         local_rank_end=8, dtype=BF16, router="normal", seed=1003),
    "gpt_oss": MoEConfig("gpt_oss", T=16384, d=2880, f=2880, E=128, k=4, R=4, local_rank_begin=0,
                         local_rank_end=1, dtype=BF16, router="forced", seed=1004),
    # "Small" and "Medium" rows of the evaluation's model table (its "Large" row is deepseek_v3 above); one rank of
    # eight is local and the load is uniform, top-k 8 (16 and 32 are the table's other columns: MoEConfig.scaled(k=...))
    "table1_s": MoEConfig("table1_s", T=2048, d=2048, f=512, E=64, k=8, R=8, local_rank_begin=0, local_rank_end=1,
                          dtype=BF16, router="normal", seed=1005),
    "table1_m": MoEConfig("table1_m", T=4096, d=4096, f=1024, E=128, k=8, R=8, local_rank_begin=0, local_rank_end=1,
                          dtype=BF16, router="normal", seed=1006),
}


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 to bfloat16 (round-to-nearest-even) and return the 16-bit patterns (finite inputs)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = (u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns to the fp32 values they denote (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _fill_normal(shape, std: float, ss: np.random.SeedSequence, dtype: int, threads: int = 8) -> np.ndarray:
    """N(0, std^2) samples of the given shape, stored as fp32 or as bf16 bit patterns."""
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.float32 if dtype == F32 else np.uint16)
    nchunk = (n + _CHUNK - 1) // _CHUNK
    kids = ss.spawn(nchunk)

    def work(i: int) -> None:
        lo = i * _CHUNK
        hi = min(n, lo + _CHUNK)
        v = np.random.default_rng(kids[i]).standard_normal(hi - lo, dtype=np.float32)
        v *= np.float32(std)
        out[lo:hi] = v if dtype == F32 else f32_to_bf16_bits(v)

    if nchunk <= 1 or threads <= 1:
        for i in range(nchunk):
            work(i)
    else:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(work, range(nchunk)))
    return out.reshape(shape)


@dataclasses.dataclass
class Workload:
    cfg: MoEConfig
    x: np.ndarray                 # [T, d]  fp32, or uint16 bf16 bit patterns
    logits: np.ndarray            # [T, E]  fp32
    W_gate: Optional[np.ndarray]  # [E_loc, d, f]
    W_up: Optional[np.ndarray]    # [E_loc, d, f]
    W_down: Optional[np.ndarray]  # [E_loc, f, d]

    def x_f32(self) -> np.ndarray:
        return self.x if self.cfg.dtype == F32 else bf16_bits_to_f32(self.x)


def make_workload(cfg: MoEConfig, weights: bool = True, threads: int = 8) -> Workload:
    """Draw order (one SeedSequence child each): x, router, bias permutation, forcing, W_gate, W_up, W_down."""
    if cfg.E % cfg.R != 0:
        raise ValueError("E must be a multiple of R")
    ss_x, ss_router, ss_perm, ss_force, ss_g, ss_u, ss_d = np.random.SeedSequence(cfg.seed).spawn(7)
    x = _fill_normal((cfg.T, cfg.d), 1.0, ss_x, cfg.dtype, threads)

    if cfg.router == "xwr":
        W_r = _fill_normal((cfg.d, cfg.E), 0.02, ss_router, F32, 1)
        xf = x if cfg.dtype == F32 else bf16_bits_to_f32(x)
        logits = (xf.astype(np.float32) @ W_r).astype(np.float32)
    else:
        logits = _fill_normal((cfg.T, cfg.E), 1.0, ss_router, F32, threads)
        if cfg.router == "zipf":
            pi = np.random.default_rng(ss_perm).permutation(cfg.E)
            bias = (-cfg.zipf_s * np.log1p(pi.astype(np.float64))).astype(np.float32)
            logits = (logits + bias[None, :]).astype(np.float32)
        elif cfg.router == "forced":
            g = np.random.default_rng(ss_force)
            forced = g.random(cfg.T) < cfg.force_p
            rank = g.integers(0, cfg.R, size=cfg.T)
            epr = cfg.epr
            rows = np.nonzero(forced)[0]
            for t in rows:
                r = int(rank[t])
                logits[t, r * epr:(r + 1) * epr] += np.float32(16.0)
        elif cfg.router == "zipf_hot":
            bias = (-cfg.zipf_s * np.log1p(np.arange(cfg.E, dtype=np.float64))).astype(np.float32)
            logits = (logits + bias[None, :]).astype(np.float32)
        elif cfg.router == "loadstd":
            p = expert_load_fractions(cfg.E, cfg.load_std, ss_perm)
            # standard normal -> uniform -> Gumbel, per element (keeps the chunked, thread-independent draw above)
            from scipy.special import ndtr
            u = np.clip(ndtr(logits.astype(np.float64)), 1e-12, 1.0 - 1e-12)
            logits = (np.log(p)[None, :] - np.log(-np.log(u))).astype(np.float32)
        elif cfg.router != "normal":
            raise ValueError(f"unknown router kind {cfg.router!r}")
    logits = np.ascontiguousarray(logits, dtype=np.float32)

    Wg = Wu = Wd = None
    if weights:
        El = cfg.E_loc
        Wg = _fill_normal((El, cfg.d, cfg.f), cfg.d ** -0.5, ss_g, cfg.dtype, threads)
        Wu = _fill_normal((El, cfg.d, cfg.f), cfg.d ** -0.5, ss_u, cfg.dtype, threads)
        Wd = _fill_normal((El, cfg.f, cfg.d), cfg.f ** -0.5, ss_d, cfg.dtype, threads)
    return Workload(cfg, x, logits, Wg, Wu, Wd)


def expert_load_fractions(E: int, load_std: float, ss: np.random.SeedSequence) -> np.ndarray:
    """Expected share of the pairs per expert under the ``"loadstd"`` router (sums to 1)."""
    z = np.random.default_rng(ss).standard_normal(E)
    p = np.maximum(1.0 + (load_std / 0.125) * z, 0.05) / E
    return p / p.sum()


def fp8_h_scale(cfg: MoEConfig) -> np.ndarray:
    """Static scale of h for the FP8 form of the GEMMs, one per local expert: an input of the layer (a calibration
    constant).  With x ~ N(0,1) and weights of standard deviation fan_in^-1/2, g and u are about N(0,1) and
    |silu(g) u| stays below ~16 except for rare outliers (which saturate); the values differ between experts so that
    a mix-up of experts shows."""
    le = np.arange(cfg.E_loc)
    return (16.0 / 448.0 * (1.0 + 0.25 * (le % 3))).astype(np.float32)
