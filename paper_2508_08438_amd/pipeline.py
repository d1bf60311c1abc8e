"""Device-resident state of one workload and the sequence of library calls that makes one pass
of the path.  Only buffer management and calls into `binding`; no arithmetic of the method."""
from __future__ import annotations

import numpy as np
import torch

from . import binding as skv
from .inputs import BLOCK, Workload


def _tiled_from_host(chunk: torch.Tensor, n_rows: int, device) -> torch.Tensor:
    """[n_rows, ...] device tensor filled with repetitions of a host chunk: host-to-device copies only."""
    out = torch.empty((n_rows,) + tuple(chunk.shape[1:]), dtype=chunk.dtype, device=device)
    step = chunk.shape[0]
    for lo in range(0, n_rows, step):
        hi = min(n_rows, lo + step)
        out[lo:hi].copy_(chunk[: hi - lo])
    return out


class Session:
    """host_fill=True builds every device buffer from host memory with plain copies, so that no torch device
    kernel runs in the process (for hardware-counter runs, which must see the library's kernels only).  Pools and
    Q/K/V then hold repetitions of one host-generated chunk: same shapes and access pattern, other values.
    kpool / vpool: pools of another session of the same configuration and seed, shared instead of filled again."""

    def __init__(self, w: Workload, device="cuda:0", with_kv=True, gather=True, host_fill=False, kpool=None,
                 vpool=None):
        self.w, self.device, self.do_gather, self.host_fill = w, torch.device(device), gather, host_fill
        dev = self.device
        a = w.attn
        self.desc = skv.attn_desc(a.n_q_heads, a.n_kv_heads, a.head_dim, a.dtype, a.scale)
        self.tree = skv.skv_tree_build(w.seq_tokens, w.seq_off, w.blk_sensitive, w.blk_owner, w.blk_page,
                                       w.n_tenants, w.n_pages, device=dev)
        self.req_off = torch.from_numpy(w.req_off).to(dev)
        self.req_tokens = torch.from_numpy(w.req_tokens).to(dev)
        self.req_tenant = torch.from_numpy(w.req_tenant).to(dev)
        R = w.n_req
        self.max_blocks = max(w.max_blocks, 1)
        self.matched_len = torch.zeros(R, dtype=torch.int32).to(dev)
        self.page_table = torch.full((R, self.max_blocks), -1, dtype=torch.int32).to(dev)
        self.q_off = torch.zeros(R + 1, dtype=torch.int32).to(dev)
        self.ctx_off = torch.zeros(R + 1, dtype=torch.int64).to(dev)
        self.kpool, self.vpool = kpool, vpool
        if with_kv and kpool is None:  # match-only sessions never touch the pools
            shape = (w.n_pages, BLOCK, a.n_kv_heads, a.head_dim)
            if host_fill:
                n = min(w.n_pages, 2048)
                self.kpool = _tiled_from_host(w.pool_pages("k", 0, n), w.n_pages, dev)
                self.vpool = _tiled_from_host(w.pool_pages("v", 0, n), w.n_pages, dev)
            else:
                self.kpool = torch.empty(shape, dtype=a.torch_dtype, device=dev)
                self.vpool = torch.empty(shape, dtype=a.torch_dtype, device=dev)
                w.fill_pool("k", self.kpool)
                w.fill_pool("v", self.vpool)
        self.q = None

    # -- one-off: lay out Q / K_new / V_new for the suffixes this workload's match leaves uncached
    def prepare(self):
        w, dev, a = self.w, self.device, self.w.attn
        skv.skv_counters_reset(self.tree)
        skv.skv_match(self.tree, self.req_off, self.req_tokens, self.req_tenant, self.max_blocks,
                      self.matched_len, self.page_table)
        torch.cuda.synchronize(dev)
        ml = self.matched_len.cpu().numpy()
        self.host_matched_len = ml
        n_ctx = max(int(ml.sum()), BLOCK)
        if self.host_fill:
            total = int((np.diff(w.req_off) - ml).sum())
            n = min(max(total, 1), 4096)
            self.q = _tiled_from_host(w.token_rows("q", 0, n), total, dev)
            self.knew = _tiled_from_host(w.token_rows("k", 0, n), total, dev)
            self.vnew = _tiled_from_host(w.token_rows("v", 0, n), total, dev)
            self.out = torch.empty_like(self.q)
            self.kctx = torch.empty((n_ctx, a.n_kv_heads, a.head_dim), dtype=a.torch_dtype, device=dev)
            self.vctx = torch.empty_like(self.kctx)
        else:
            self.q = w.suffix_rows("q", ml, dev)
            self.knew = w.suffix_rows("k", ml, dev)
            self.vnew = w.suffix_rows("v", ml, dev)
            self.out = torch.zeros_like(self.q)
            self.kctx = torch.zeros((n_ctx, a.n_kv_heads, a.head_dim), dtype=a.torch_dtype, device=dev)
            self.vctx = torch.zeros_like(self.kctx)
        nbytes = skv.skv_prefill_attn_workspace_size(self.desc, w.n_req, self.q.shape[0])
        self.workspace = torch.zeros(nbytes, dtype=torch.uint8).to(dev)
        skv.skv_counters_reset(self.tree)

    # -- the individual stages (each only enqueues on the current stream)
    def match(self):
        skv.skv_counters_reset(self.tree)
        skv.skv_match(self.tree, self.req_off, self.req_tokens, self.req_tenant, self.max_blocks,
                      self.matched_len, self.page_table)
        skv.skv_suffix_offsets(self.req_off, self.matched_len, self.q_off)

    def gather(self):
        skv.skv_gather_kv(self.desc, self.kpool, self.vpool, self.matched_len, self.page_table,
                          self.max_blocks, self.ctx_off, self.kctx, self.vctx)

    def attention(self):
        skv.skv_prefill_attn(self.desc, self.q, self.knew, self.vnew, self.q_off, self.kpool, self.vpool,
                             self.matched_len, self.page_table, self.max_blocks, self.out, self.workspace)

    def step(self):
        if self.q is None:
            self.prepare()
        self.match()
        if self.do_gather:
            self.gather()
        self.attention()
        return {"matched_len": self.matched_len, "page_table": self.page_table, "q_off": self.q_off,
                "ctx_off": self.ctx_off, "out": self.out, "kctx": self.kctx, "vctx": self.vctx}

    # -- the same pass recorded once as a HIP graph and replayed: the calls of match / gather / attention only
    #    enqueue kernels on the stream they are given (no allocation, no memset, no synchronisation)
    def capture_step(self):
        if self.q is None:
            self.prepare()
        self.step()                       # everything loaded and warm before the capture
        torch.cuda.synchronize(self.device)
        self.graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(self.graph):
            self.match()
            if self.do_gather:
                self.gather()
            self.attention()
        return self.graph

    def replay(self):
        self.graph.replay()

    def counters(self):
        n = self.w.n_in_blocks
        hit = torch.zeros(max(n, 1), dtype=torch.int32).to(self.device)
        ucnt = torch.zeros(max(n, 1), dtype=torch.int32).to(self.device)
        skv.skv_counters_read(self.tree, hit, ucnt)
        torch.cuda.synchronize(self.device)
        return hit[:n].cpu().numpy().view(np.uint32), ucnt[:n].cpu().numpy().view(np.uint32)

    def host_pools(self, page_table):
        """CPU copies of the pools holding the pages a page table references (others zero)."""
        w, a = self.w, self.w.attn
        pages = np.unique(page_table[page_table >= 0])
        shape = (w.n_pages, BLOCK, a.n_kv_heads, a.head_dim)
        kpool = torch.zeros(shape, dtype=a.torch_dtype)
        vpool = torch.zeros(shape, dtype=a.torch_dtype)
        w.fill_pool("k", kpool, pages)
        w.fill_pool("v", vpool, pages)
        return kpool, vpool
