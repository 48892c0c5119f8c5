"""The five synthetic ISD-step workloads (shapes and value recipes only).

Each workload stands in for the serving traffic the paper measures (an 8B-class
GQA model, bf16 KV cache, many concurrent requests, contexts up to 32k tokens;
Sec. 4 serving evaluation and App. H serving configuration); none of the
paper's prompts or datasets is used, only their shapes.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Optional, Tuple

BASE_SEED = 20260411


def n_draft_for_stride(S: int) -> int:
    """Number of previously proposed tokens verified in a step of S query rows.

    A steady-state step holds one exact token, n_draft drafted tokens and the
    remaining MASK rows (Alg. 1; App. B "Overhead": 2N-1 = 1 + (N-1) + (N-1)).
    For the even strides of the benchmark configs this gives S/2-1 drafts and
    S/2 MASK rows; S = 1 is a plain autoregressive decode step.
    """
    return max(0, (S - 1) // 2)


@dataclass(frozen=True)
class ISDConfig:
    name: str
    index: int                 # 1-based index in the benchmark list
    B: int                     # concurrent sequences
    S: int                     # query rows per sequence per step
    Hq: int
    Hkv: int
    D: int                     # head dimension
    P: int                     # tokens per KV page
    V: int                     # vocabulary
    dtype: str                 # "f32" | "bf16" (Q / K / V / out)
    ctx_kind: str              # "list" | "uniform" | "loguniform" | "const"
    ctx_lo: int = 0
    ctx_hi: int = 0
    ctx_list: Tuple[int, ...] = ()
    logit_sigma: float = 1.0
    zipf_s: float = 0.0        # >0: add -s*ln(1+i) bias over token ids
    plant_peak: bool = False   # plant p(t*) = pi ~ U(0.5, 1) in every row
    draft_hit: float = 1.0     # probability the draft is the planted / arg-max token
    draft_noise: float = 1.0   # sigma of the noise used for the "noisy argmax" draft
    mode: str = "greedy"       # "greedy" | "stochastic" | "mixed"
    pool_factor: float = 1.0   # page pool size / pages needed (>1 = fragmented)
    n_draft: Optional[int] = None

    @property
    def seed(self) -> int:
        return BASE_SEED * 10 + self.index

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv

    @property
    def drafts(self) -> int:
        return n_draft_for_stride(self.S) if self.n_draft is None else self.n_draft

    def with_(self, **kw) -> "ISDConfig":
        return replace(self, **kw)


CONFIGS = {
    # 1: tiny fp32 step, greedy
    "tiny": ISDConfig("tiny", 1, B=2, S=4, Hq=4, Hkv=2, D=64, P=16, V=1024, dtype="f32",
                      ctx_kind="list", ctx_list=(37, 120), logit_sigma=2.0,
                      draft_noise=1.0, mode="greedy"),
    # 2: small-model step, ~60 % per-token acceptance, greedy and stochastic
    "small": ISDConfig("small", 2, B=16, S=8, Hq=16, Hkv=4, D=128, P=16, V=32768, dtype="bf16",
                       ctx_kind="uniform", ctx_lo=256, ctx_hi=1024, logit_sigma=3.0,
                       plant_peak=True, draft_hit=0.80, mode="stochastic"),
    # 3: 8B-class GQA step, Zipf-skewed logits, ~70 % acceptance, stochastic
    "8b": ISDConfig("8b", 3, B=64, S=8, Hq=32, Hkv=8, D=128, P=16, V=151936, dtype="bf16",
                    ctx_kind="uniform", ctx_lo=1024, ctx_hi=4096, logit_sigma=4.0, zipf_s=1.1,
                    plant_peak=True, draft_hit=0.93, mode="stochastic"),
    # 4: large-concurrency serving step (the benchmark's headline workload)
    "serve256": ISDConfig("serve256", 4, B=256, S=16, Hq=32, Hkv=8, D=128, P=16, V=151936,
                          dtype="bf16", ctx_kind="loguniform", ctx_lo=512, ctx_hi=8192,
                          logit_sigma=4.0, zipf_s=1.1, plant_peak=True, draft_hit=0.93,
                          mode="mixed", pool_factor=1.25),
    # 5: long-context stride sweep (S is overridden per sweep point)
    "long32k": ISDConfig("long32k", 5, B=32, S=8, Hq=64, Hkv=8, D=128, P=16, V=151936,
                         dtype="bf16", ctx_kind="const", ctx_lo=32768, ctx_hi=32768,
                         logit_sigma=4.0, zipf_s=1.1, plant_peak=True, draft_hit=0.93,
                         mode="stochastic"),
}

LONG32K_STRIDES = (1, 4, 8, 16, 32)


def get_config(name: str, **overrides) -> ISDConfig:
    cfg = CONFIGS[name]
    return cfg.with_(**overrides) if overrides else cfg
