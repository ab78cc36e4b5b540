"""Seeded synthetic inputs for the batched verification step of speculative decoding.

This module only draws random numbers and lays them out; it holds none of the
method's arithmetic (no attention, no acceptance test, no decomposition).  Both
the CPU oracle's tests and the HIP path's tests/bench take their inputs from
here, so the two sides always see the same bits.

Workload shapes: five configurations of a verification batch in which every
request brings its own number of draft (candidate) tokens, standing in for the
Alpaca / ChatGPT-Prompts / Chatbot-Instruction-Prompts request mixes of the
paper's evaluation (Sec. VI-A), whose length statistics the paper never prints.

Layout produced
  * request table: prefix_len[B], draft_len[B], q_offset[B+1], pt_offset[B+1],
    page_table[...] (int32).  Request i owns ceil((p_i+g_i)/page_size) pages.
  * K/V pools: bf16, logical shape [n_pages][n_kv_heads][page_size][head_dim],
    pages handed out by a random permutation of a pool 1.25x the needed size.
  * Q: bf16 [R][n_q_heads][head_dim], R = sum of draft lengths.
  * logits: target fp32 [R+B][V] (request i owns rows q_offset[i]+i .. +g_i,
    the last one being the bonus row), draft fp32 [R][V].
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Optional

import numpy as np
import torch


@dataclass(frozen=True)
class VerifyConfig:
    name: str
    n_req: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    prefix_lo: int
    prefix_hi: int
    prefix_dist: str          # "uniform" | "loguniform"
    draft_dist: str           # "uniform" | "skewed"
    draft_lo: int = 1
    draft_hi: int = 8
    page_size: int = 16
    vocab: int = 32000
    logit_sigma: float = 3.0
    q_split_width: int = 0    # >0: the batch is decomposed into sub-requests of this many draft rows


CONFIGS = {
    # 0: small enough for the oracle to finish in well under a second
    "tiny": VerifyConfig("tiny", 4, 2, 2, 64, 16, 128, "uniform", "uniform", 1, 5,
                         vocab=1000, logit_sigma=2.0),
    # 1: Llama-7B-shaped attention layer
    "7b": VerifyConfig("7b", 32, 32, 32, 128, 128, 2048, "uniform", "uniform", 1, 8),
    # 2: skewed draft lengths, decomposed into width-4 sub-requests
    "skewed": VerifyConfig("skewed", 64, 32, 32, 128, 256, 2048, "uniform", "skewed",
                           2, 16, q_split_width=4),
    # 3: Llama-13B-shaped (the configuration the bandwidth target is quoted on)
    "13b": VerifyConfig("13b", 128, 40, 40, 128, 256, 4096, "loguniform", "uniform", 1, 8),
    # 4: 70B-shaped grouped-query layer
    "70b_gqa": VerifyConfig("70b_gqa", 256, 64, 8, 128, 512, 8192, "loguniform", "uniform", 1, 8),
}
CONFIG_ORDER = ["tiny", "7b", "skewed", "13b", "70b_gqa"]


@dataclass
class RequestTable:
    prefix_len: np.ndarray    # int32 [B]
    draft_len: np.ndarray     # int32 [B]
    q_offset: np.ndarray      # int32 [B+1]
    pt_offset: np.ndarray     # int32 [B+1]
    page_table: np.ndarray    # int32 [pt_offset[B]]
    page_size: int
    n_pages: int              # pool size in pages

    @property
    def n_req(self) -> int:
        return int(self.prefix_len.shape[0])

    @property
    def n_rows(self) -> int:
        return int(self.q_offset[-1])

    def kv_tokens(self) -> int:
        return int((self.prefix_len.astype(np.int64) + self.draft_len).sum())


@dataclass
class VerifyBatch:
    cfg: VerifyConfig
    table: RequestTable
    q: torch.Tensor           # bf16 [R][Hq][d]
    k_pool: torch.Tensor      # bf16 [n_pages][Hkv][P][d]
    v_pool: torch.Tensor      # bf16 [n_pages][Hkv][P][d]
    extra: dict = field(default_factory=dict)


@dataclass
class AcceptBatch:
    draft_len: np.ndarray       # int32 [B]
    draft_tokens: torch.Tensor  # int32 [R]
    target_logits: torch.Tensor  # fp32 [R+B][V]
    draft_logits: torch.Tensor  # fp32 [R][V]
    u_accept: torch.Tensor      # fp64 [R]   in [0,1)
    u_sample: torch.Tensor      # fp64 [B]   in [0,1)
    vocab: int


def draw_lengths(cfg: VerifyConfig, rng: np.random.Generator):
    """Prefix and draft lengths of one batch (both ends of every range inclusive)."""
    B = cfg.n_req
    if cfg.prefix_dist == "uniform":
        p = rng.integers(cfg.prefix_lo, cfg.prefix_hi + 1, size=B)
    elif cfg.prefix_dist == "loguniform":
        x = rng.uniform(math.log(cfg.prefix_lo), math.log(cfg.prefix_hi), size=B)
        p = np.clip(np.rint(np.exp(x)), cfg.prefix_lo, cfg.prefix_hi).astype(np.int64)
    else:
        raise ValueError(cfg.prefix_dist)
    if cfg.draft_dist == "uniform":
        g = rng.integers(cfg.draft_lo, cfg.draft_hi + 1, size=B)
    elif cfg.draft_dist == "skewed":
        g = np.where(rng.random(B) < 0.7, cfg.draft_lo, cfg.draft_hi)
    else:
        raise ValueError(cfg.draft_dist)
    return p.astype(np.int32), g.astype(np.int32)


def make_table(prefix_len, draft_len, page_size: int, rng: Optional[np.random.Generator],
               pool_slack: float = 1.25, min_pool_pages: int = 0) -> RequestTable:
    """Build offsets and hand out physical pages.

    rng=None assigns pages in order (page i of the pool = i-th page needed);
    otherwise a random permutation of a pool `pool_slack` times the need.
    """
    prefix_len = np.asarray(prefix_len, dtype=np.int32)
    draft_len = np.asarray(draft_len, dtype=np.int32)
    B = prefix_len.shape[0]
    n_tok = prefix_len.astype(np.int64) + draft_len
    n_pg = (n_tok + page_size - 1) // page_size
    q_offset = np.zeros(B + 1, dtype=np.int32)
    q_offset[1:] = np.cumsum(draft_len)
    pt_offset = np.zeros(B + 1, dtype=np.int32)
    pt_offset[1:] = np.cumsum(n_pg)
    need = int(pt_offset[-1])
    pool = max(int(math.ceil(need * pool_slack)), need, min_pool_pages, 1)
    if rng is None:
        page_table = np.arange(need, dtype=np.int32)
    else:
        page_table = rng.permutation(pool)[:need].astype(np.int32)
    return RequestTable(prefix_len, draft_len, q_offset, pt_offset, page_table, page_size, pool)


def _randn_16(shape, gen: torch.Generator, device, dtype=torch.bfloat16) -> torch.Tensor:
    # Drawn in fp32 and rounded to the 16-bit type (round-to-nearest-even) exactly once;
    # everybody downstream reads these bits.  Done in slabs to bound the fp32 temporary.
    out = torch.empty(shape, dtype=dtype, device=device)
    flat = out.view(-1)
    step = 1 << 27
    for s in range(0, flat.numel(), step):
        e = min(flat.numel(), s + step)
        flat[s:e] = torch.randn(e - s, generator=gen, device=device, dtype=torch.float32).to(dtype)
    return out


def make_verify_batch(cfg: VerifyConfig, seed: int, device="cpu", prefix_len=None, draft_len=None,
                      poison_unused: bool = False, shuffle_pages: bool = True, dtype=torch.bfloat16) -> VerifyBatch:
    """One synthetic verification batch (Q, K, V standard normal, rounded once to `dtype`: bf16 or fp16).  `poison_unused` writes NaN into every K/V slot no
    request owns (unused pool pages and the tail of each request's last page)."""
    rng = np.random.default_rng(seed)
    if prefix_len is None or draft_len is None:
        p, g = draw_lengths(cfg, rng)
        prefix_len = p if prefix_len is None else prefix_len
        draft_len = g if draft_len is None else draft_len
    table = make_table(prefix_len, draft_len, cfg.page_size, rng if shuffle_pages else None)
    gen = torch.Generator(device=device)
    gen.manual_seed(1000003 * seed + 17)
    R = table.n_rows
    q = _randn_16((R, cfg.n_q_heads, cfg.head_dim), gen, device, dtype)
    shape = (table.n_pages, cfg.n_kv_heads, cfg.page_size, cfg.head_dim)
    k_pool = _randn_16(shape, gen, device, dtype)
    v_pool = _randn_16(shape, gen, device, dtype)
    if poison_unused:
        owned = torch.zeros((table.n_pages, cfg.page_size), dtype=torch.bool)
        n_tok = table.prefix_len.astype(np.int64) + table.draft_len
        for i in range(table.n_req):
            pages = table.page_table[table.pt_offset[i]:table.pt_offset[i + 1]]
            for c, pg in enumerate(pages):
                used = int(min(cfg.page_size, n_tok[i] - c * cfg.page_size))
                owned[int(pg), :used] = True
        mask = (~owned).to(device)[:, None, :, None].expand(shape)
        k_pool.masked_fill_(mask, float("nan"))
        v_pool.masked_fill_(mask, float("nan"))
    return VerifyBatch(cfg, table, q, k_pool, v_pool)


def make_accept_batch(draft_len, vocab: int, sigma: float, seed: int, device="cpu",
                      rho: Optional[float] = None, draft_token_mode: str = "sample") -> AcceptBatch:
    """Logits, draft tokens and uniforms for the acceptance step.

    rho=None: draft logits independent of the target's (the literal configuration; almost every
    first draft token is rejected).  rho in (0,1): draft = rho*target + sqrt(1-rho^2)*noise, so
    accepted lengths spread over 0..g.  draft_token_mode: "sample" draws each draft token from
    the draft model's own distribution (what a sampling SSM does), "argmax" takes its top token.
    """
    draft_len = np.asarray(draft_len, dtype=np.int32)
    B = draft_len.shape[0]
    R = int(draft_len.sum())
    gen = torch.Generator(device=device)
    gen.manual_seed(7919 * seed + 3)
    target = torch.randn((R + B, vocab), generator=gen, device=device, dtype=torch.float32) * sigma
    noise = torch.randn((R, vocab), generator=gen, device=device, dtype=torch.float32) * sigma
    if rho is None:
        draft = noise
    else:
        # target rows of request i sit at q_offset[i]+i+t; drop each request's bonus row
        keep = np.ones(R + B, dtype=bool)
        ends = np.cumsum(draft_len) + np.arange(B)
        keep[ends] = False
        idx = torch.from_numpy(np.nonzero(keep)[0]).to(device)
        draft = rho * target.index_select(0, idx) + math.sqrt(1.0 - rho * rho) * noise
    if draft_token_mode == "sample":
        probs = torch.softmax(draft.double(), dim=-1)
        tok = torch.multinomial(probs, 1, generator=gen).view(-1).to(torch.int32) if R > 0 else \
            torch.empty(0, dtype=torch.int32, device=device)
    elif draft_token_mode == "argmax":
        tok = draft.argmax(dim=-1).to(torch.int32)
    else:
        raise ValueError(draft_token_mode)
    rng = np.random.default_rng(seed + 104729)
    u_accept = torch.from_numpy(rng.random(R)).to(device)
    u_sample = torch.from_numpy(rng.random(B)).to(device)
    return AcceptBatch(draft_len, tok, target, draft, u_accept, u_sample, vocab)


def random_trees(draft_len, rng, shape: str = "random"):
    """Token trees for the drafts: parents [R] (index of the parent draft token within the request,
    -1 = child of the last prefix token; always smaller than the token's own index) and the
    ancestor-or-self bit masks [R] (uint64) that the attention entry point takes.
    shape: "random" (uniform parent among the earlier tokens or the root), "chain", "star",
    "wide" (a few long branches)."""
    parents, masks = [], []
    for g in np.asarray(draft_len):
        par, msk = [], []
        for t in range(int(g)):
            if shape == "chain":
                q = t - 1
            elif shape == "star":
                q = -1
            elif shape == "wide":
                q = t - 3 if t >= 3 else -1
            else:
                q = int(rng.integers(-1, t))
            par.append(q)
            msk.append((msk[q] if q >= 0 else 0) | (1 << t))
        parents += par
        masks += msk
    return np.asarray(parents, dtype=np.int32), np.asarray(masks, dtype=np.uint64)


def bf16_bits(t: torch.Tensor) -> np.ndarray:
    """The raw 16-bit patterns of a bf16 tensor as a uint16 numpy array (host copy)."""
    assert t.dtype == torch.bfloat16
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def host_elems(t: torch.Tensor) -> np.ndarray:
    """A 16-bit tensor on the host in the form the oracle reads: bf16 as raw uint16 bit patterns, fp16
    as a numpy float16 array (both widen to float64 exactly)."""
    if t.dtype == torch.bfloat16:
        return bf16_bits(t)
    assert t.dtype == torch.float16
    return t.detach().cpu().contiguous().numpy()


def algorithmic_kv_bytes(table: RequestTable, n_kv_heads: int, head_dim: int) -> int:
    """Bytes the step must move at least: every request's K and V once, bf16."""
    return table.kv_tokens() * n_kv_heads * head_dim * 2 * 2
