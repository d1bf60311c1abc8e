"""Device-resident state of one workload and the sequence of library calls that makes one pass
of the path.  Only buffer management and calls into `binding`; no arithmetic of the method."""
from __future__ import annotations

import numpy as np
import torch

from . import binding as skv
from .inputs import BLOCK, Workload


class Session:
    def __init__(self, w: Workload, device="cuda:0", with_kv=True, gather=True):
        self.w, self.device, self.do_gather = w, torch.device(device), gather
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
        self.matched_len = torch.zeros(R, dtype=torch.int32, device=dev)
        self.page_table = torch.full((R, self.max_blocks), -1, dtype=torch.int32, device=dev)
        self.q_off = torch.zeros(R + 1, dtype=torch.int32, device=dev)
        self.ctx_off = torch.zeros(R + 1, dtype=torch.int64, device=dev)
        self.kpool = self.vpool = None
        if with_kv:  # match-only sessions never touch the pools
            shape = (w.n_pages, BLOCK, a.n_kv_heads, a.head_dim)
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
        self.q = w.suffix_rows("q", ml, dev)
        self.knew = w.suffix_rows("k", ml, dev)
        self.vnew = w.suffix_rows("v", ml, dev)
        self.out = torch.zeros_like(self.q)
        n_ctx = max(int(ml.sum()), BLOCK)
        self.kctx = torch.zeros((n_ctx, a.n_kv_heads, a.head_dim), dtype=a.torch_dtype, device=dev)
        self.vctx = torch.zeros_like(self.kctx)
        nbytes = skv.skv_prefill_attn_workspace_size(self.desc, w.n_req, self.q.shape[0])
        self.workspace = torch.zeros(nbytes, dtype=torch.uint8, device=dev)
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
        hit = torch.zeros(max(n, 1), dtype=torch.int32, device=self.device)
        ucnt = torch.zeros(max(n, 1), dtype=torch.int32, device=self.device)
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
