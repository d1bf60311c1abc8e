"""Seeded synthetic inputs for the selective-reuse prefill path.

This module only *draws inputs*: cached block sequences with their per-block
privacy tag / creator / page id, request streams, and the values of the Q/K/V
tensors.  It holds none of the method's arithmetic (no matching, no counters,
no attention) and is the only module imported both by the CPU oracle's tests
and by the GPU path's callers.

The workloads stand in for the paper's serving traces (Section 7.1: multi-turn
chat, single-request PII prompts, one long uniform system prompt), of which
only the *structure* is taken: many tenants sharing a few long prefixes,
tenant-private content behind them, skewed popularity.  No item of any dataset
is reproduced; token ids are uniform random integers.

Tensor values are a pure function of (seed, stream, element index) built from
integer operations only (a splitmix64-style finaliser followed by a sum of the
eight bytes of the hash, i.e. an Irwin-Hall(8) approximation of N(0,1)), so the
same element evaluates to the same bits on the CPU and on the GPU through
torch, and any subset of pages can be produced without generating the rest.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Optional

import numpy as np
import torch

BLOCK = 16  # tokens per KV block
VOCAB = 32000

STREAM_KPOOL, STREAM_VPOOL, STREAM_Q, STREAM_KNEW, STREAM_VNEW = 0, 1, 2, 3, 4

_M1 = 0xBF58476D1CE4E5B9 - (1 << 64)  # as signed int64
_M2 = 0x94D049BB133111EB - (1 << 64)
_GOLD = 0x9E3779B97F4A7C15 - (1 << 64)
_IH8_MEAN = 8 * 127.5
_IH8_SIGMA = math.sqrt(8 * (256.0 ** 2 - 1.0) / 12.0)


def _lsr(z: torch.Tensor, s: int) -> torch.Tensor:
    return (z >> s) & ((1 << (64 - s)) - 1)


def _hash64(counter: torch.Tensor, seed: int) -> torch.Tensor:
    z = counter * _GOLD + seed
    z = (z ^ _lsr(z, 30)) * _M1
    z = (z ^ _lsr(z, 27)) * _M2
    return z ^ _lsr(z, 31)


def synth_values(seed: int, stream: int, start: int, count: int, sigma: float,
                 device="cpu") -> torch.Tensor:
    """fp32 values for elements [start, start+count) of one stream."""
    seed = (seed * 0x2545F4914F6CDD1D + stream * 0x632BE59BD9B4E019) & ((1 << 63) - 1)
    idx = torch.arange(start, start + count, dtype=torch.int64, device=device)
    h = _hash64(idx, seed)
    acc = torch.zeros_like(h)
    for k in range(8):
        acc += (h >> (8 * k)) & 255
    c = np.float32(sigma / _IH8_SIGMA)
    return (acc.to(torch.float32) - np.float32(_IH8_MEAN)) * float(c)


def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, stream])))


def _zipf_choice(rng, n_ranks: int, a: float, size: int) -> np.ndarray:
    w = 1.0 / np.arange(1, n_ranks + 1, dtype=np.float64) ** a
    cdf = np.cumsum(w / w.sum())
    return np.minimum(np.searchsorted(cdf, rng.random(size)), n_ranks - 1).astype(np.int64)


@dataclass
class AttnShape:
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    dtype: str  # "f32" | "bf16"

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == "f32" else torch.bfloat16

    @property
    def scale(self) -> float:
        return 1.0 / math.sqrt(self.head_dim)


@dataclass
class Workload:
    name: str
    seed: int
    n_tenants: int
    n_pages: int
    # cached side (host)
    seq_tokens: np.ndarray     # int32 [sum len]
    seq_off: np.ndarray        # int64 [n_seq+1], token offsets, multiples of BLOCK
    blk_sensitive: np.ndarray  # uint8 [n_in_blocks]
    blk_owner: np.ndarray      # int32 [n_in_blocks]
    blk_page: np.ndarray       # int32 [n_in_blocks]
    # requests
    req_tokens: np.ndarray     # int32 [sum N_r]
    req_off: np.ndarray        # int32 [R+1]
    req_tenant: np.ndarray     # int32 [R]
    attn: AttnShape
    value_sigma: float         # std of Q/K/V entries
    meta: dict = field(default_factory=dict)

    @property
    def n_req(self) -> int:
        return len(self.req_tenant)

    @property
    def n_in_blocks(self) -> int:
        return len(self.blk_page)

    @property
    def max_blocks(self) -> int:
        n = np.diff(self.req_off)
        return int(n.max() // BLOCK) if len(n) else 0

    @property
    def page_elems(self) -> int:
        return BLOCK * self.attn.n_kv_heads * self.attn.head_dim

    # ---- tensor values (pure functions of the element index) -------------
    def pool_pages(self, which: str, page_lo: int, page_hi: int, device="cpu") -> torch.Tensor:
        """Pages [page_lo, page_hi) of the K or V pool: [n, BLOCK, Hkv, d]."""
        stream = STREAM_KPOOL if which == "k" else STREAM_VPOOL
        pe = self.page_elems
        v = synth_values(self.seed, stream, page_lo * pe, (page_hi - page_lo) * pe,
                         self.value_sigma, device)
        return v.to(self.attn.torch_dtype).view(page_hi - page_lo, BLOCK,
                                                self.attn.n_kv_heads, self.attn.head_dim)

    def fill_pool(self, which: str, out: torch.Tensor, pages=None, chunk_pages: int = 4096):
        """Write pool contents into `out` [n_pages, BLOCK, Hkv, d] (all pages, or the listed ones)."""
        if pages is None:
            for lo in range(0, self.n_pages, chunk_pages):
                hi = min(self.n_pages, lo + chunk_pages)
                out[lo:hi] = self.pool_pages(which, lo, hi, out.device)
        else:
            for p in np.unique(np.asarray(pages, dtype=np.int64)):
                out[int(p)] = self.pool_pages(which, int(p), int(p) + 1, out.device)[0]
        return out

    def token_rows(self, which: str, tok_lo: int, tok_hi: int, device="cpu") -> torch.Tensor:
        """Q / K_new / V_new rows for request-stream token indices [tok_lo, tok_hi).

        The value of a row depends only on the token's index in `req_tokens`, so a
        request's uncached suffix [req_off[r]+L_r, req_off[r+1]) has the same values
        whatever L_r turns out to be."""
        a = self.attn
        stream, heads = {"q": (STREAM_Q, a.n_q_heads), "k": (STREAM_KNEW, a.n_kv_heads),
                         "v": (STREAM_VNEW, a.n_kv_heads)}[which]
        per = heads * a.head_dim
        v = synth_values(self.seed, stream, tok_lo * per, (tok_hi - tok_lo) * per,
                         self.value_sigma, device)
        return v.to(a.torch_dtype).view(tok_hi - tok_lo, heads, a.head_dim)

    def suffix_rows(self, which: str, matched_len: np.ndarray, device="cpu") -> torch.Tensor:
        """Ragged [sum S_r, heads, d] tensor of the uncached suffixes given matched lengths."""
        parts = []
        for r in range(self.n_req):
            lo = int(self.req_off[r]) + int(matched_len[r])
            hi = int(self.req_off[r + 1])
            if hi > lo:
                parts.append(self.token_rows(which, lo, hi, device))
        if not parts:
            a = self.attn
            heads = a.n_q_heads if which == "q" else a.n_kv_heads
            return torch.empty(0, heads, a.head_dim, dtype=a.torch_dtype, device=device)
        return torch.cat(parts, 0)


# ---------------------------------------------------------------------------
# the five configurations
# ---------------------------------------------------------------------------

def _assemble(name, seed, n_tenants, n_pages, prefixes, sens, owner, req_list, req_tenant,
              attn, sigma, rng_pages, meta=None) -> Workload:
    """prefixes: list of int32 arrays (full-block lengths); sens/owner: per input block."""
    lens = np.array([len(p) for p in prefixes], dtype=np.int64)
    assert (lens % BLOCK == 0).all()
    seq_off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    seq_tokens = (np.concatenate(prefixes) if prefixes else np.zeros(0)).astype(np.int32)
    n_blk = int(seq_off[-1] // BLOCK)
    assert n_blk <= n_pages
    blk_page = rng_pages.permutation(n_pages)[:n_blk].astype(np.int32)
    rlens = np.array([len(x) for x in req_list], dtype=np.int64)
    req_off = np.concatenate([[0], np.cumsum(rlens)]).astype(np.int32)
    req_tokens = (np.concatenate(req_list) if req_list else np.zeros(0)).astype(np.int32)
    return Workload(name=name, seed=seed, n_tenants=n_tenants, n_pages=n_pages,
                    seq_tokens=seq_tokens, seq_off=seq_off,
                    blk_sensitive=sens.astype(np.uint8), blk_owner=owner.astype(np.int32),
                    blk_page=blk_page, req_tokens=req_tokens, req_off=req_off,
                    req_tenant=np.asarray(req_tenant, dtype=np.int32), attn=attn,
                    value_sigma=sigma, meta=meta or {})


def _sigma(attn: AttnShape, hard: bool) -> float:
    # literal recipe: entries ~ N(0,1)/sqrt(d); "hard": entries ~ N(0,1) (logit std ~ 1)
    return 1.0 if hard else 1.0 / math.sqrt(attn.head_dim)


def _fixed_prefix_workload(name, seed, n_prefix, prefix_len, n_req, n_tenants, suffix_len,
                           p_sens, n_pages, attn, hard):
    r_tok, r_meta, r_req, r_page = (_rng(seed, s) for s in range(4))
    prefixes = [r_tok.integers(0, VOCAB, prefix_len, dtype=np.int32) for _ in range(n_prefix)]
    n_blk = n_prefix * prefix_len // BLOCK
    sens = r_meta.random(n_blk) < p_sens
    owner = r_meta.integers(0, n_tenants, n_blk)
    which = r_req.integers(0, n_prefix, n_req)
    tenant = r_req.integers(0, n_tenants, n_req)
    reqs = [np.concatenate([prefixes[w], r_req.integers(0, VOCAB, suffix_len, dtype=np.int32)])
            for w in which]
    return _assemble(name, seed, n_tenants, n_pages, prefixes, sens, owner, reqs, tenant,
                     attn, _sigma(attn, hard), r_page, {"prefix_of_req": which})


def config1(hard: bool = False, seed: int = 0x5AFE0001) -> Workload:
    """Tiny: 8 requests, 4 tenants, 4 prefixes x 256 tokens, 30% sensitive, fp32 8/8 heads d=64."""
    return _fixed_prefix_workload("c1_tiny", seed, 4, 256, 8, 4, 64, 0.30, 128,
                                  AttnShape(8, 8, 64, "f32"), hard)


def config2(hard: bool = False, seed: int = 0x5AFE0002) -> Workload:
    """64 requests, 16 tenants, 32 prefixes x 1024 tokens, 20% sensitive, 4096-page pool, bf16 32/8 d=128."""
    return _fixed_prefix_workload("c2_shared_prefix", seed, 32, 1024, 64, 16, 128, 0.20, 4096,
                                  AttnShape(32, 8, 128, "bf16"), hard)


def config3(hard: bool = False, seed: int = 0x5AFE0003, n_prefix: int = 512, n_req: int = 256,
            n_tenants: int = 64, len_lo: int = 256, len_hi: int = 4096) -> Workload:
    """Streaming mix: prefixes with hierarchical sharing, Zipf(1.1) popularity, ragged suffixes."""
    r_tok, r_meta, r_req, r_page = (_rng(seed, s) for s in range(4))
    full = []  # full (unaligned) prefixes
    for i in range(n_prefix):
        n = int(r_tok.integers(len_lo, len_hi + 1))
        if i > 0 and r_tok.random() < 0.5:
            src = full[int(r_tok.integers(0, i))]
            head = int(r_tok.integers(1, min(len(src), n) + 1))  # divergence point, not block aligned
            p = np.concatenate([src[:head], r_tok.integers(0, VOCAB, n - head, dtype=np.int32)])
        else:
            p = r_tok.integers(0, VOCAB, n, dtype=np.int32)
        full.append(p.astype(np.int32))
    cached = [p[: len(p) // BLOCK * BLOCK] for p in full]  # only full blocks are cached
    n_blk = sum(len(p) for p in cached) // BLOCK
    sens = r_meta.random(n_blk) < 0.20
    owner = r_meta.integers(0, n_tenants, n_blk)
    which = _zipf_choice(r_req, n_prefix, 1.1, n_req)
    tenant = r_req.integers(0, n_tenants, n_req)
    reqs = [np.concatenate([full[w], r_req.integers(0, VOCAB, int(r_req.integers(32, 513)),
                                                    dtype=np.int32)]) for w in which]
    n_pages = (n_blk + 1023) // 1024 * 1024
    return _assemble("c3_streaming_mix", seed, n_tenants, n_pages, cached, sens, owner, reqs,
                     tenant, AttnShape(32, 8, 128, "bf16"), _sigma(AttnShape(32, 8, 128, "bf16"), hard),
                     r_page, {"prefix_of_req": which})


def config4(hard: bool = False, seed: int = 0x5AFE0004, literal: bool = False, n_req: int = 32,
            len_lo: int = 16384, len_hi: int = 32768, n_pages: int = 65536) -> Workload:
    """Long context: one long session prefix per request, reused by its creator (intra-tenant
    reuse); `literal=True` draws owners and requesters uniformly instead."""
    n_tenants = 8
    attn = AttnShape(64, 8, 128, "bf16")
    r_tok, r_meta, r_req, r_page = (_rng(seed, s) for s in range(4))
    full = [r_tok.integers(0, VOCAB, int(r_tok.integers(len_lo, len_hi + 1)), dtype=np.int32)
            for _ in range(n_req)]
    cached = [p[: len(p) // BLOCK * BLOCK] for p in full]
    nblk = [len(p) // BLOCK for p in cached]
    creator = r_meta.integers(0, n_tenants, n_req)
    sens = r_meta.random(sum(nblk)) < 0.10
    if literal:
        owner = r_meta.integers(0, n_tenants, sum(nblk))
        tenant = r_req.integers(0, n_tenants, n_req)
    else:
        owner = np.repeat(creator, nblk)
        tenant = creator.copy()
    reqs = [np.concatenate([full[i], r_req.integers(0, VOCAB, 256, dtype=np.int32)])
            for i in range(n_req)]
    return _assemble("c4_long_context" + ("_literal" if literal else ""), seed, n_tenants, n_pages,
                     cached, sens, owner, reqs, tenant, attn, _sigma(attn, hard), r_page)


def config5(p_sensitive: float = 0.25, hard: bool = False, seed: int = 0x5AFE0005,
            n_prefix: int = 2048, n_req: int = 1024, n_tenants: int = 128,
            len_lo: int = 128, len_hi: int = 8192, suf_lo: int = 64, suf_hi: int = 1024) -> Workload:
    """Sensitivity sweep: same tokens / owners / requests for every `p_sensitive`; the sensitive
    sets are nested (block b is sensitive iff u_b < p_sensitive)."""
    attn = AttnShape(32, 8, 128, "bf16")
    r_tok, r_meta, r_req, r_page = (_rng(seed, s) for s in range(4))
    full = [r_tok.integers(0, VOCAB, int(r_tok.integers(len_lo, len_hi + 1)), dtype=np.int32)
            for _ in range(n_prefix)]
    cached = [p[: len(p) // BLOCK * BLOCK] for p in full]
    n_blk = sum(len(p) for p in cached) // BLOCK
    sens = r_meta.random(n_blk) < p_sensitive
    owner = r_meta.integers(0, n_tenants, n_blk)
    which = _zipf_choice(r_req, n_prefix, 1.0, n_req)
    tenant = r_req.integers(0, n_tenants, n_req)
    reqs = [np.concatenate([full[w], r_req.integers(0, VOCAB, int(r_req.integers(suf_lo, suf_hi + 1)),
                                                    dtype=np.int32)]) for w in which]
    n_pages = (n_blk + 1023) // 1024 * 1024
    return _assemble(f"c5_sweep_p{int(round(100 * p_sensitive))}", seed, n_tenants, n_pages, cached,
                     sens, owner, reqs, tenant, attn, _sigma(attn, hard), r_page,
                     {"prefix_of_req": which})


def small_random(seed: int, n_seq: int = 6, max_blocks: int = 8, vocab: int = 3, n_tenants: int = 3,
                 n_req: int = 12, p_sens: float = 0.4, attn: Optional[AttnShape] = None,
                 block_vocab: Optional[int] = None) -> Workload:
    """Tiny collision-heavy case: tokens from a very small vocabulary so that siblings share
    first tokens, sequences are prefixes of one another, and requests branch off mid-node.
    With `block_vocab` set, blocks are drawn from that many distinct 16-token patterns that
    differ from each other only in a few positions (forces long common runs)."""
    attn = attn or AttnShape(4, 2, 64, "f32")
    r_tok, r_meta, r_req, r_page = (_rng(seed, s) for s in range(4))
    if block_vocab:
        base = r_tok.integers(0, vocab, BLOCK, dtype=np.int32)
        pats = np.tile(base, (block_vocab, 1))
        for i in range(1, block_vocab):
            pats[i, r_tok.integers(0, BLOCK)] += 1 + i
        draw = lambda nb: pats[r_tok.integers(0, block_vocab, nb)].reshape(-1)
        rdraw = lambda nb: pats[r_req.integers(0, block_vocab, nb)].reshape(-1)
    else:
        draw = lambda nb: r_tok.integers(0, vocab, nb * BLOCK, dtype=np.int32)
        rdraw = lambda nb: r_req.integers(0, vocab, nb * BLOCK, dtype=np.int32)
    seqs = []
    for i in range(n_seq):
        nb = int(r_tok.integers(1, max_blocks + 1))
        if i > 0 and r_tok.random() < 0.6:
            src = seqs[int(r_tok.integers(0, i))]
            head = int(r_tok.integers(0, len(src) // BLOCK + 1)) * BLOCK
            s = np.concatenate([src[:head], draw(nb)])[: max_blocks * BLOCK]
        else:
            s = draw(nb)
        seqs.append(s.astype(np.int32))
    n_blk = sum(len(s) for s in seqs) // BLOCK
    sens = r_meta.random(n_blk) < p_sens
    owner = r_meta.integers(0, n_tenants, n_blk)
    reqs, tenants = [], []
    for _ in range(n_req):
        src = seqs[int(r_req.integers(0, n_seq))]
        head = int(r_req.integers(0, len(src) + 1))  # any token position
        tail = int(r_req.integers(0, 2 * BLOCK + 1))
        x = np.concatenate([src[:head], rdraw(3)[:tail]])
        if r_req.random() < 0.15:  # occasionally a pure-random or empty request
            x = rdraw(int(r_req.integers(0, 4)))[: int(r_req.integers(0, 49))]
        reqs.append(x.astype(np.int32))
        tenants.append(int(r_req.integers(0, n_tenants)))
    return _assemble(f"small_{seed}", seed, n_tenants, max(n_blk, 1) + 3, seqs, sens, owner, reqs,
                     tenants, attn, 1.0, r_page)


CONFIGS = {"c1": config1, "c2": config2, "c3": config3, "c4": config4, "c5": config5}


@dataclass
class DecodeWorkload:
    """One decode step over a paged cache: per request a context length and the pages that hold it.
    Pool and query values are the same pure functions of the element index as everywhere else."""
    seed: int
    attn: AttnShape
    n_pages: int
    ctx_len: np.ndarray      # int32 [R]: cached tokens the new token attends to (itself included)
    page_table: np.ndarray   # int32 [R, max_blocks], -1 beyond the context
    value_sigma: float

    @property
    def n_req(self) -> int:
        return len(self.ctx_len)

    @property
    def max_blocks(self) -> int:
        return self.page_table.shape[1]

    def pool_pages(self, which: str, page_lo: int, page_hi: int, device="cpu") -> torch.Tensor:
        a = self.attn
        pe = BLOCK * a.n_kv_heads * a.head_dim
        v = synth_values(self.seed, STREAM_KPOOL if which == "k" else STREAM_VPOOL, page_lo * pe,
                         (page_hi - page_lo) * pe, self.value_sigma, device)
        return v.to(a.torch_dtype).view(page_hi - page_lo, BLOCK, a.n_kv_heads, a.head_dim)

    def fill_pool(self, which: str, out: torch.Tensor, pages=None, chunk_pages: int = 4096):
        if pages is None:
            for lo in range(0, self.n_pages, chunk_pages):
                hi = min(self.n_pages, lo + chunk_pages)
                out[lo:hi] = self.pool_pages(which, lo, hi, out.device)
        else:
            for p in np.unique(np.asarray(pages, dtype=np.int64)):
                out[int(p)] = self.pool_pages(which, int(p), int(p) + 1, out.device)[0]
        return out

    def queries(self, device="cpu") -> torch.Tensor:
        a = self.attn
        n = self.n_req * a.n_q_heads * a.head_dim
        return synth_values(self.seed, STREAM_Q, 0, n, self.value_sigma, device).to(a.torch_dtype).view(
            self.n_req, a.n_q_heads, a.head_dim)


def decode_workload(seed: int = 0x5AFE0006, n_req: int = 64, ctx_lo: int = 4096, ctx_hi: int = 16384,
                    attn: Optional[AttnShape] = None, hard: bool = False, ctx=None) -> DecodeWorkload:
    """Decode step of a serving batch: contexts uniform in [ctx_lo, ctx_hi] (or the listed ones), every page
    used once, page ids a seeded permutation of the pool."""
    attn = attn or AttnShape(32, 8, 128, "bf16")
    g = _rng(seed, 0)
    ctx_len = (np.asarray(ctx, dtype=np.int32) if ctx is not None
               else g.integers(ctx_lo, ctx_hi + 1, n_req).astype(np.int32))
    nb = (ctx_len + BLOCK - 1) // BLOCK
    n_pages = int(nb.sum()) + 8
    perm = g.permutation(n_pages).astype(np.int32)
    table = np.full((len(ctx_len), max(int(nb.max()), 1)), -1, np.int32)
    table[np.arange(table.shape[1])[None, :] < nb[:, None]] = perm[: int(nb.sum())]
    return DecodeWorkload(seed, attn, n_pages, ctx_len, table, _sigma(attn, hard))
