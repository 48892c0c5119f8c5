"""Seeded generators for the inputs of the two ISD-step calls.

Everything is drawn with torch (on whatever device is asked for, so the large
workloads can be generated directly in HBM) from a `torch.Generator` seeded with
the config's seed.  The same tensors are handed to the CPU oracle (after a copy
to host memory) and to the HIP path.  No function here evaluates attention, a
softmax-based decision or a sampler: the only statistics computed are those the
*recipe* needs to place a row's probability mass (a log-sum-exp used to plant a
token with a prescribed probability).
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Optional

import numpy as np
import torch

from .configs import ISDConfig

BASE_SEED_LORA = 2026041100


def bf16_bits(t: torch.Tensor) -> np.ndarray:
    """Bit patterns (uint16) of a bfloat16 tensor, on the host."""
    assert t.dtype == torch.bfloat16
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def to_numpy(t: torch.Tensor) -> np.ndarray:
    """Host copy as numpy; bfloat16 becomes its uint16 bit patterns."""
    if t.dtype == torch.bfloat16:
        return bf16_bits(t)
    return t.detach().cpu().contiguous().numpy()


def k_pages_in_operand_order(k_cache: torch.Tensor) -> torch.Tensor:
    """The K pool [num_pages, Hkv, 16, 128] (contiguous) with the 16-byte chunks of every (page, head)
    block permuted from slot-major (entry 16*t + c) to the order the attention kernel's matrix operands
    use (entry 64*(c/4) + 16*(c%4) + t).  A pure permutation of the stored bytes."""
    pages, Hkv, P, D = k_cache.shape
    assert P == 16 and D == 128 and k_cache.is_contiguous()
    v = k_cache.view(pages, Hkv, 16, 4, 4, 8)              # [.., t, c/4, c%4, 8 elements]
    return v.permute(0, 1, 3, 4, 2, 5).contiguous().view(pages, Hkv, P, D)


def _torch_dtype(name: str) -> torch.dtype:
    return {"f32": torch.float32, "bf16": torch.bfloat16}[name]


@dataclass
class AttentionInputs:
    cfg: ISDConfig
    q: torch.Tensor            # [B,S,Hq,D]
    k_cache: torch.Tensor      # [num_pages,Hkv,P,D]
    v_cache: torch.Tensor      # [num_pages,Hkv,P,D]
    block_table: torch.Tensor  # int32 [B,max_pages_per_seq], -1 where unused
    ctx_lens: torch.Tensor     # int32 [B], includes the S rows of this step
    num_pages: int
    max_pages_per_seq: int

    @property
    def kv_tokens(self) -> int:
        return int(self.ctx_lens.sum().item())


@dataclass
class AcceptInputs:
    cfg: ISDConfig
    logits: torch.Tensor        # fp32 [B,S,V]
    draft_tokens: torch.Tensor  # int32 [B,max(S-1,1)]
    n_draft: torch.Tensor       # int32 [B]
    greedy: torch.Tensor        # uint8 [B], 1 = greedy
    rng_seed: int
    rng_offset: int


def draw_ctx_lens(cfg: ISDConfig, gen: torch.Generator) -> torch.Tensor:
    dev = gen.device
    if cfg.ctx_kind == "list":
        assert len(cfg.ctx_list) == cfg.B
        return torch.tensor(cfg.ctx_list, dtype=torch.int32, device=dev)
    if cfg.ctx_kind == "const":
        return torch.full((cfg.B,), cfg.ctx_lo, dtype=torch.int32, device=dev)
    u = torch.rand(cfg.B, generator=gen, device=dev, dtype=torch.float64)
    if cfg.ctx_kind == "uniform":
        c = torch.floor(cfg.ctx_lo + u * (cfg.ctx_hi - cfg.ctx_lo + 1))
    elif cfg.ctx_kind == "loguniform":
        c = torch.floor(torch.exp(math.log(cfg.ctx_lo) + u * (math.log(cfg.ctx_hi) - math.log(cfg.ctx_lo))))
    else:
        raise ValueError(cfg.ctx_kind)
    return c.clamp(max(cfg.ctx_lo, cfg.S), cfg.ctx_hi).to(torch.int32)


def make_attention_inputs(cfg: ISDConfig, device="cpu", seed: Optional[int] = None,
                          poison_unused: bool = False) -> AttentionInputs:
    """Q, paged K/V pools, a random block table and context lengths for `cfg`.

    The pool holds ceil(pool_factor * pages_needed) pages and the pages of all
    sequences are drawn as one random permutation of the whole pool, so tables
    are fragmented.  With `poison_unused`, every pool slot that no sequence owns
    (tail of a last page, spare pages) holds NaN, and unused block-table entries
    are -1: any read outside the valid context shows up in the output.
    """
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(cfg.seed if seed is None else seed)
    dt = _torch_dtype(cfg.dtype)
    B, S, Hq, Hkv, D, P = cfg.B, cfg.S, cfg.Hq, cfg.Hkv, cfg.D, cfg.P

    ctx = draw_ctx_lens(cfg, gen)
    assert int(ctx.min()) >= S, "every sequence must already hold this step's S rows"
    pages_per_seq = (ctx.to(torch.int64) + P - 1) // P
    need = int(pages_per_seq.sum())
    num_pages = max(need, int(math.ceil(cfg.pool_factor * need)))
    if cfg.ctx_kind == "list":
        max_pages = int(pages_per_seq.max())
    else:
        max_pages = (cfg.ctx_hi + P - 1) // P
    perm = torch.randperm(num_pages, generator=gen, device=dev)[:need].to(torch.int32)
    table = torch.full((B, max_pages), -1, dtype=torch.int32, device=dev)
    owner_len = torch.zeros(num_pages, dtype=torch.int32, device=dev)  # valid tokens per page
    off = 0
    pps = pages_per_seq.tolist()
    ctx_l = ctx.tolist()
    for b in range(B):
        n = pps[b]
        ids = perm[off:off + n]
        table[b, :n] = ids
        fill = torch.full((n,), P, dtype=torch.int32, device=dev)
        fill[-1] = ctx_l[b] - (n - 1) * P
        owner_len[ids.long()] = fill
        off += n

    q = torch.randn(B, S, Hq, D, generator=gen, device=dev, dtype=torch.float32).to(dt)

    def pool():
        t = torch.empty(num_pages, Hkv, P, D, dtype=dt, device=dev)
        step = max(1, (1 << 26) // (Hkv * P * D))   # draw in 64M-element slabs
        for s in range(0, num_pages, step):
            e = min(num_pages, s + step)
            t[s:e] = torch.randn(e - s, Hkv, P, D, generator=gen, device=dev,
                                 dtype=torch.float32).to(dt)
        return t

    k_cache, v_cache = pool(), pool()
    if poison_unused:
        slot = torch.arange(P, device=dev, dtype=torch.int32)[None, :]
        unused = slot >= owner_len[:, None]                       # [num_pages,P]
        mask = unused[:, None, :, None].expand(num_pages, Hkv, P, D)
        k_cache[mask] = float("nan")
        v_cache[mask] = float("nan")
    return AttentionInputs(cfg, q, k_cache, v_cache, table, ctx, num_pages, max_pages)


def make_accept_inputs(cfg: ISDConfig, device="cpu", seed: Optional[int] = None,
                       rng_offset: int = 0) -> AcceptInputs:
    """Logits, drafted tokens, per-sequence draft counts and greedy flags.

    logits[b,j,i] = sigma * N(0,1) - zipf_s * ln(1+i).  With `plant_peak`, each
    row's largest entry t* is raised so that its softmax probability is exactly
    pi ~ U(0.5, 1) (l[t*] = LSE(others) + ln(pi / (1 - pi))): a model that is
    confident in one token, which lets the stochastic acceptance rate reach the
    target.  The draft for a row is t* with probability `draft_hit`, otherwise
    the best other token under N(0, draft_noise^2) perturbed logits.
    """
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed((cfg.seed if seed is None else seed) + 7919)
    B, S, V = cfg.B, cfg.S, cfg.V
    ncol = max(S - 1, 1)
    logits = torch.empty(B, S, V, dtype=torch.float32, device=dev)
    drafts = torch.zeros(B, ncol, dtype=torch.int32, device=dev)
    bias = None
    if cfg.zipf_s > 0:
        bias = (-cfg.zipf_s * torch.log1p(torch.arange(V, device=dev, dtype=torch.float64))).float()
    rows_per_slab = max(1, (1 << 25) // V)
    flat = logits.view(B * S, V)
    draft_flat = torch.zeros(B * S, dtype=torch.int64, device=dev)
    for s in range(0, B * S, rows_per_slab):
        e = min(B * S, s + rows_per_slab)
        x = torch.randn(e - s, V, generator=gen, device=dev, dtype=torch.float32) * cfg.logit_sigma
        if bias is not None:
            x += bias
        top = x.argmax(dim=1)
        ar = torch.arange(e - s, device=dev)
        noise = torch.randn(e - s, V, generator=gen, device=dev, dtype=torch.float32) * cfg.draft_noise
        if cfg.plant_peak:
            x[ar, top] = -float("inf")
            lse_others = torch.logsumexp(x.double(), dim=1)
            pi = 0.5 + 0.5 * torch.rand(e - s, generator=gen, device=dev, dtype=torch.float64)
            x[ar, top] = (lse_others + torch.log(pi / (1 - pi))).float()
            pert = x + noise
            pert[ar, top] = -float("inf")
            other = pert.argmax(dim=1)
            hit = torch.rand(e - s, generator=gen, device=dev) < cfg.draft_hit
            draft_flat[s:e] = torch.where(hit, top, other)
        else:
            draft_flat[s:e] = (x + noise).argmax(dim=1)
        flat[s:e] = x
    drafts[:, :S - 1] = draft_flat.view(B, S)[:, :S - 1].to(torch.int32)
    n_draft = torch.full((B,), cfg.drafts, dtype=torch.int32, device=dev)
    if cfg.mode == "greedy":
        greedy = torch.ones(B, dtype=torch.uint8, device=dev)
    elif cfg.mode == "stochastic":
        greedy = torch.zeros(B, dtype=torch.uint8, device=dev)
    else:
        greedy = (torch.rand(B, generator=gen, device=dev) < 0.5).to(torch.uint8)
    rng_seed = (0x9E3779B97F4A7C15 * (cfg.seed if seed is None else seed)) & 0xFFFFFFFFFFFFFFFF
    return AcceptInputs(cfg, logits, drafts, n_draft, greedy, rng_seed, rng_offset)


@dataclass
class LoraInputs:
    """One linear layer with a low-rank adapter and the tokens of one ISD step (bf16 tensors)."""
    x: torch.Tensor          # [B*S, d_in] activations, token b*S+j = stride row j of sequence b
    W: torch.Tensor          # [d_out, d_in] base weight
    A: torch.Tensor          # [r, d_in]  adapter down-projection
    Bm: torch.Tensor         # [d_out, r] adapter up-projection
    n_draft: torch.Tensor    # int32 [B] drafts under introspection per sequence (rows beyond are MASK)
    S: int


def make_lora_inputs(B: int, S: int, d_in: int, d_out: int, r: int, device="cpu", seed: int = 0,
                     n_draft: Optional[int] = None) -> LoraInputs:
    """Unit-variance activations; base weight N(0, 1/d_in) so that outputs are O(1); adapter factors
    N(0, 1/d_in) and N(0, 1/r) so that the residual is of the size of the base output (a trained
    adapter's is smaller: this makes its errors as visible as the base projection's).  n_draft is
    uniform on [0, S-1] per sequence unless given (steady state of a stride: (S-1)//2)."""
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(BASE_SEED_LORA + seed)

    def draw(rows, cols, sigma):
        return (torch.randn(rows, cols, generator=gen, device=dev, dtype=torch.float32) * sigma).to(torch.bfloat16)

    x = draw(B * S, d_in, 1.0)
    W = draw(d_out, d_in, d_in ** -0.5)
    A = draw(r, d_in, d_in ** -0.5)
    Bm = draw(d_out, r, max(r, 1) ** -0.5)
    if n_draft is None:
        nd = torch.randint(0, S, (B,), generator=gen, device=dev, dtype=torch.int32)
    else:
        nd = torch.full((B,), n_draft, dtype=torch.int32, device=dev)
    return LoraInputs(x, W, A, Bm, nd, S)
