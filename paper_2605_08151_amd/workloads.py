"""Seeded synthetic verification batches.

This module only *draws inputs*: shapes, lengths, page tables, random tensors,
draft tokens.  It contains none of the verification step's arithmetic and is
imported neither by the GPU binding nor by the CPU oracle; tests and the
benchmark feed the same tensors to both.  Quantities that depend on the target
model's output (the argmax a greedy drafter copies, the logits a noisy drafter
perturbs) are taken as arguments.

The five named configurations follow the workload shapes of the paper's
experiments (gamma = 4 default, batch 32..256, ShareGPT-like ~4k contexts,
LongBench-like 32k-64k contexts, temperature > 0 runs, and the parallel-mode
mix in which rollback requests carry a single decode row, eq.
parallel_rollback_pad).
"""
from __future__ import annotations

import dataclasses
import math
from typing import Optional, Sequence

import torch


@dataclasses.dataclass(frozen=True)
class VerifyConfig:
    name: str
    seed: int
    B: int
    gamma_choices: Sequence[int]          # gamma_i drawn uniformly from these
    ctx: tuple                            # ("const", c) | ("uniform", lo, hi) | ("lognormal", median, sigma, lo, hi)
    Hq: int
    Hkv: int
    H: int
    V: int
    D: int = 128
    P: int = 16
    temperature: tuple = ("const", 0.0)   # ("const", T) | ("alternate", T_even, T_odd)
    rho: float = 0.7                      # greedy drafter: per-position continue probability
    sigma: float = 0.02                   # std of q, K, V, hidden, W
    sigma_qkv: Optional[float] = None     # override for q, K, V (the "sharp" sets)
    pool_slack: float = 1.25              # physical pages / pages in use


CONFIGS = {
    "tiny": VerifyConfig("tiny", 0, 4, (4,), ("uniform", 128, 512), 8, 1, 1024, 32000, rho=0.7),
    "mid": VerifyConfig("mid", 1, 32, (4,), ("const", 2048), 32, 8, 4096, 151936, rho=0.6),
    "stochastic": VerifyConfig("stochastic", 2, 64, (8,), ("uniform", 1024, 4096), 8, 1, 4096, 151936,
                               temperature=("const", 0.7)),
    "long": VerifyConfig("long", 3, 8, (4,), ("uniform", 32768, 65536), 8, 1, 4096, 151936, rho=0.7),
    "hybrid": VerifyConfig("hybrid", 4, 256, (0, 2, 4, 8), ("lognormal", 4096, 1.0, 256, 32768), 8, 1, 4096,
                           151936, temperature=("alternate", 0.0, 1.0), rho=0.7),
}


def bf16_bits(t: torch.Tensor):
    """bf16 tensor -> numpy uint16 bit patterns (host)."""
    import numpy as np
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def _randn_bf16(shape, std, gen, device):
    # drawn in slabs so the fp32 staging buffer stays small next to a >1 GB bf16 tensor
    out = torch.empty(shape, dtype=torch.bfloat16, device=device)
    flat = out.view(-1)
    step = 1 << 26
    for lo in range(0, flat.numel(), step):
        n = min(step, flat.numel() - lo)
        flat[lo:lo + n] = (torch.randn(n, generator=gen, device=device, dtype=torch.float32) * std).to(torch.bfloat16)
    return out


def draw_lengths(cfg: VerifyConfig, gen_cpu: torch.Generator):
    """gamma_i and committed lengths c_i (host int32 tensors)."""
    B = cfg.B
    choices = torch.tensor(list(cfg.gamma_choices), dtype=torch.int32)
    gammas = choices[torch.randint(0, len(choices), (B,), generator=gen_cpu)]
    kind = cfg.ctx[0]
    if kind == "const":
        ctx = torch.full((B,), int(cfg.ctx[1]), dtype=torch.int32)
    elif kind == "uniform":
        ctx = torch.randint(int(cfg.ctx[1]), int(cfg.ctx[2]) + 1, (B,), generator=gen_cpu).to(torch.int32)
    elif kind == "lognormal":
        _, median, sigma, lo, hi = cfg.ctx
        z = torch.randn(B, generator=gen_cpu, dtype=torch.float64)
        ctx = torch.clamp(torch.floor(median * torch.exp(sigma * z)), lo, hi).to(torch.int32)
    else:
        raise ValueError(kind)
    return gammas.to(torch.int32), ctx


def make_batch(cfg: VerifyConfig, device="cpu", with_lm_head=True, kv_copies: int = 1):
    """Everything the step reads before the LM head: lengths, page table, free list, q, K/V pages,
    hidden rows, W, temperatures and seeds.  `kv_copies` > 1 allocates that many independent K/V pools
    (same page table) so a timing loop can rotate among them."""
    gen_cpu = _gen(cfg.seed, "cpu")
    gen_dev = _gen(cfg.seed + 1000, device)
    gammas, ctx = draw_lengths(cfg, gen_cpu)
    B, P = cfg.B, cfg.P
    n = gammas + 1
    qo_indptr = torch.zeros(B + 1, dtype=torch.int32)
    qo_indptr[1:] = torch.cumsum(n, 0)
    M = int(qo_indptr[-1])
    pages_per_seq = (ctx + n + P - 1) // P
    used = int(pages_per_seq.sum())
    num_pages = max(used + 1, int(math.ceil(used * cfg.pool_slack)))
    max_pages = int(pages_per_seq.max()) + 1           # one spare column, always unmapped
    perm = torch.randperm(num_pages, generator=gen_cpu).to(torch.int32)
    page_table = torch.full((B, max_pages), -1, dtype=torch.int32)
    off = 0
    for i in range(B):
        k = int(pages_per_seq[i])
        page_table[i, :k] = perm[off:off + k]
        off += k
    free_cap = num_pages
    free_list = torch.full((free_cap,), -1, dtype=torch.int32)
    free_count = num_pages - used
    free_list[:free_count] = perm[used:]

    s_qkv = cfg.sigma_qkv if cfg.sigma_qkv is not None else cfg.sigma
    q = _randn_bf16((M, cfg.Hq, cfg.D), s_qkv, gen_dev, device)
    k_caches = [_randn_bf16((num_pages, cfg.Hkv, P, cfg.D), s_qkv, gen_dev, device) for _ in range(kv_copies)]
    v_caches = [_randn_bf16((num_pages, cfg.Hkv, P, cfg.D), s_qkv, gen_dev, device) for _ in range(kv_copies)]

    if cfg.temperature[0] == "const":
        temperature = torch.full((B,), float(cfg.temperature[1]), dtype=torch.float32)
    else:
        temperature = torch.tensor([cfg.temperature[1 + (i & 1)] for i in range(B)], dtype=torch.float32)
    # per-request 64-bit Philox keys: drawn, not computed from the method
    seeds = torch.randint(0, 2 ** 62, (B,), generator=gen_cpu, dtype=torch.int64)

    batch = dict(
        cfg=cfg, B=B, M=M, gamma_max=int(gammas.max()), gammas=gammas, ctx=ctx, num_pages=num_pages,
        max_pages=max_pages, max_kv_len=int((ctx + n).max()),
        qo_indptr=qo_indptr.to(device), seq_lens=ctx.clone().to(device), page_table=page_table.to(device),
        free_list=free_list.to(device), free_count=torch.tensor([free_count], dtype=torch.int32, device=device),
        q=q, k_cache=k_caches[0], v_cache=v_caches[0], k_caches=k_caches, v_caches=v_caches,
        temperature=temperature.to(device), seeds=seeds.to(device),
        scale=1.0 / math.sqrt(cfg.D),
    )
    if with_lm_head:
        s_hw = cfg.sigma
        batch["hidden"] = _randn_bf16((M, cfg.H), s_hw, gen_dev, device)
        batch["W"] = _randn_bf16((cfg.V, cfg.H), s_hw, gen_dev, device)
    return batch


def draft_tokens_greedy(cfg: VerifyConfig, qo_indptr, target_argmax, first_tokens=None):
    """Drafts of a drafter that copies the target's greedy token for a geometric(rho) prefix.

    target_argmax [M] (int, host): the greedy token of every row, supplied by the caller.
    Draft j >= 1 of request i equals target_argmax[row j-1] while j <= k_i, where
    P(k_i >= j) = rho^j; draft k_i + 1 is drawn uniformly from the other V-1 tokens (so the planned
    accepted length is exact) and later drafts uniformly from all V.  Row 0's token is the previous
    bonus token b: any id.  Returns (tokens [M] int32 host, planned_len [B] int32 host)."""
    gen = _gen(cfg.seed + 2000, "cpu")
    qo = qo_indptr.cpu().tolist()
    am = target_argmax.cpu().to(torch.int64)
    B = len(qo) - 1
    M = qo[-1]
    tokens = torch.randint(0, cfg.V, (M,), generator=gen, dtype=torch.int64)
    cont = torch.rand(M, generator=gen) < cfg.rho
    planned = torch.zeros(B, dtype=torch.int32)
    for i in range(B):
        r0, gamma = qo[i], qo[i + 1] - qo[i] - 1
        k = 0
        while k < gamma and bool(cont[r0 + k + 1]):
            k += 1
        planned[i] = k
        for j in range(1, k + 1):
            tokens[r0 + j] = am[r0 + j - 1]
        if k < gamma:
            wrong = int(torch.randint(0, cfg.V - 1, (1,), generator=gen))
            tokens[r0 + k + 1] = wrong + (1 if wrong >= int(am[r0 + k]) else 0)
    return tokens.to(torch.int32), planned


def draft_probs_noisy(cfg: VerifyConfig, qo_indptr, logits, noise_std=1.0, chunk_rows=32):
    """A drafter whose distribution is the target's logits plus N(0, noise_std) noise.

    logits [M,V] fp32 (any device), supplied by the caller.  For draft j >= 1 of request i the drafter's
    distribution is q_j = softmax(logits[row j-1] + eps), eps iid normal, and d_j ~ q_j.
    Returns (draft_probs [M-B, V] fp32 on logits.device, tokens [M] int32 host)."""
    device = logits.device
    gen_dev = _gen(cfg.seed + 3000, device)
    gen_cpu = _gen(cfg.seed + 3001, "cpu")
    qo = qo_indptr.cpu().tolist()
    B = len(qo) - 1
    M, V = logits.shape
    src_rows = []
    for i in range(B):
        src_rows += list(range(qo[i], qo[i + 1] - 1))
    src = torch.tensor(src_rows, dtype=torch.int64, device=device)
    draft_probs = torch.empty((M - B, V), dtype=torch.float32, device=device)
    drawn = torch.empty(M - B, dtype=torch.int64, device=device)
    for lo in range(0, M - B, chunk_rows):
        rows = src[lo:lo + chunk_rows]
        noisy = logits[rows].to(torch.float32)
        noisy = noisy + noise_std * torch.randn(noisy.shape, generator=gen_dev, device=device, dtype=torch.float32)
        qrows = torch.softmax(noisy, dim=-1)
        draft_probs[lo:lo + len(rows)] = qrows
        drawn[lo:lo + len(rows)] = torch.multinomial(qrows, 1, generator=gen_dev).squeeze(1)
    tokens = torch.randint(0, V, (M,), generator=gen_cpu, dtype=torch.int64)
    drawn = drawn.cpu()
    k = 0
    for i in range(B):
        for r in range(qo[i] + 1, qo[i + 1]):
            tokens[r] = drawn[k]
            k += 1
    return draft_probs, tokens.to(torch.int32)
