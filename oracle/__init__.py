"""ctypes access to the CPU oracle (test infrastructure only).

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this module.
It imports nothing from the GPU package and the GPU package never imports it.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "skv_oracle.cpp")
_LIB = os.path.join(_HERE, "libskv_oracle.so")
BLOCK = 16


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["g++", "-O2", "-std=c++17", "-fPIC", "-shared", "-pthread",
                               "-o", _LIB, _SRC])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.okv_tree_new.restype = C.c_void_p
        _lib.okv_tree_new.argtypes = [C.c_int]
        _lib.okv_tree_free.argtypes = [C.c_void_p]
        _lib.okv_tree_insert.argtypes = [C.c_void_p, C.c_int64] + [C.c_void_p] * 5
        _lib.okv_tree_n_blocks.restype = C.c_int64
        _lib.okv_tree_n_blocks.argtypes = [C.c_void_p]
        _lib.okv_tree_n_nodes.restype = C.c_int64
        _lib.okv_tree_n_nodes.argtypes = [C.c_void_p]
        _lib.okv_match.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                   C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int]
        _lib.okv_counters.argtypes = [C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p]
        _lib.okv_sole_tenant.argtypes = [C.c_void_p, C.c_int64, C.c_void_p]
        _lib.okv_counters_reset.argtypes = [C.c_void_p]
        _lib.okv_window_roll.restype = C.c_int64
        _lib.okv_window_roll.argtypes = [C.c_void_p, C.c_int] + [C.c_uint32] * 5
        _lib.okv_block_state.argtypes = [C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p]
        _lib.okv_insert_requests.restype = C.c_int64
        _lib.okv_insert_requests.argtypes = [C.c_void_p, C.c_int32] + [C.c_void_p] * 5 + [C.c_int32, C.c_int64,
                                                                                        C.c_void_p, C.c_void_p, C.c_int32]
        _lib.okv_set_epoch.argtypes = [C.c_void_p, C.c_uint32]
        _lib.okv_block_epochs.argtypes = [C.c_void_p, C.c_int64, C.c_void_p]
        _lib.okv_evict.restype = C.c_int64
        _lib.okv_evict.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p]
        _lib.okv_promote.argtypes = [C.c_void_p, C.c_int64, C.c_void_p]
        _lib.okv_scatter.argtypes = [C.c_int64, C.c_int32, C.c_void_p, C.c_void_p, C.c_int32] + [C.c_void_p] * 4
        _lib.okv_gather.argtypes = [C.c_int64, C.c_int32, C.c_void_p, C.c_void_p, C.c_int32,
                                    C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        _lib.okv_attention.argtypes = [C.c_int, C.c_int, C.c_int, C.c_int, C.c_double, C.c_int32] + \
            [C.c_void_p] * 8 + [C.c_int32, C.c_int64] + [C.c_void_p] * 4 + [C.c_int]
    return _lib


def _p(a):
    if a is None:
        return None
    if isinstance(a, torch.Tensor):
        assert a.device.type == "cpu" and a.is_contiguous()
        return C.c_void_p(a.data_ptr())
    assert a.flags["C_CONTIGUOUS"]
    return C.c_void_p(a.ctypes.data)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


class OracleTree:
    """Pointer-based radix tree over the cached block sequences of a workload."""

    def __init__(self, seq_tokens, seq_off, blk_sensitive, blk_owner, blk_page, compressed=True):
        self._l = lib()
        self._t = C.c_void_p(self._l.okv_tree_new(0 if compressed else 1))
        seq_tokens = _i32(seq_tokens)
        seq_off = np.ascontiguousarray(seq_off, dtype=np.int64)
        sens = np.ascontiguousarray(blk_sensitive, dtype=np.uint8)
        owner, page = _i32(blk_owner), _i32(blk_page)
        self.n_in_blocks = len(page)
        assert len(sens) == len(owner) == len(page) == int(seq_off[-1]) // BLOCK
        rc = self._l.okv_tree_insert(self._t, len(seq_off) - 1, _p(seq_off), _p(seq_tokens),
                                     _p(sens), _p(owner), _p(page))
        if rc:
            raise ValueError("oracle: bad sequence offsets")

    @classmethod
    def from_workload(cls, w, compressed=True):
        return cls(w.seq_tokens, w.seq_off, w.blk_sensitive, w.blk_owner, w.blk_page, compressed)

    def __del__(self):
        if getattr(self, "_t", None):
            self._l.okv_tree_free(self._t)
            self._t = None

    @property
    def n_blocks(self):
        return self._l.okv_tree_n_blocks(self._t)

    @property
    def n_nodes(self):
        return self._l.okv_tree_n_nodes(self._t)

    def match(self, req_off, req_tokens, req_tenant, max_blocks, update=True, want_ids=False):
        req_off, req_tokens, req_tenant = _i32(req_off), _i32(req_tokens), _i32(req_tenant)
        R = len(req_tenant)
        mlen = np.zeros(R, dtype=np.int32)
        pt = np.full((R, max_blocks), -1, dtype=np.int32)
        ids = np.full((R, max_blocks), -1, dtype=np.int64) if want_ids else None
        self._l.okv_match(self._t, R, _p(req_off), _p(req_tokens), _p(req_tenant), max_blocks,
                          _p(mlen), _p(pt), _p(ids), int(update))
        return (mlen, pt, ids) if want_ids else (mlen, pt)

    def counters(self):
        hit = np.zeros(self.n_in_blocks, dtype=np.uint32)
        ucnt = np.zeros(self.n_in_blocks, dtype=np.uint32)
        self._l.okv_counters(self._t, self.n_in_blocks, _p(hit), _p(ucnt))
        return hit, ucnt

    def sole_tenant(self):
        who = np.zeros(self.n_in_blocks, dtype=np.int32)
        self._l.okv_sole_tenant(self._t, self.n_in_blocks, _p(who))
        return who

    def window_roll(self, direction=0, tau=(1, 2), min_hits=1, n_consec=1, u_pre_max=1):
        """Safeguard step at a window boundary; returns the number of blocks demoted."""
        return int(self._l.okv_window_roll(self._t, int(direction), int(tau[0]), int(tau[1]), int(min_hits),
                                           int(n_consec), int(u_pre_max)))

    def insert(self, req_off, req_tokens, req_tenant, matched_len, new_pages, private_copies=False):
        """Append the blocks the tree does not hold yet (private_copies: the blocks the requester cannot see),
        private to the requesting tenant.  Returns (first_inserted, n_inserted) per request; new entries take
        the ids n_in_blocks, n_in_blocks+1, ..."""
        req_off, req_tokens, req_tenant = _i32(req_off), _i32(req_tokens), _i32(req_tenant)
        matched_len, new_pages = _i32(matched_len), _i32(new_pages)
        R = len(req_tenant)
        assert new_pages.shape[0] == R
        first = np.zeros(R, dtype=np.int32)
        n = np.zeros(R, dtype=np.int32)
        self.n_in_blocks = int(self._l.okv_insert_requests(
            self._t, R, _p(req_off), _p(req_tokens), _p(req_tenant), _p(matched_len), _p(new_pages),
            new_pages.shape[1], self.n_in_blocks, _p(first), _p(n), int(private_copies)))
        return first, n

    def set_epoch(self, epoch):
        self._l.okv_set_epoch(self._t, int(epoch))

    def epochs(self):
        e = np.zeros(self.n_in_blocks, dtype=np.uint32)
        self._l.okv_block_epochs(self._t, self.n_in_blocks, _p(e))
        return e

    def evict(self, n_want, protect_ids=()):
        """Evict up to n_want blocks (oldest childless tails first).  Returns (block ids, pages) in order."""
        prot = np.ascontiguousarray(protect_ids, dtype=np.int64)
        n_want = int(min(n_want, self.n_blocks))
        ids = np.zeros(max(n_want, 1), dtype=np.int64)
        pages = np.zeros(max(n_want, 1), dtype=np.int32)
        k = self._l.okv_evict(self._t, n_want, len(prot), _p(prot), _p(ids), _p(pages))
        return ids[:k], pages[:k]

    def promote(self, block_ids):
        ids = np.ascontiguousarray(block_ids, dtype=np.int64)
        self._l.okv_promote(self._t, len(ids), _p(ids))

    def block_state(self):
        """(private_tag, hit_pre, u_pre) per input block id; private_tag 255 = block created no entry."""
        priv = np.zeros(self.n_in_blocks, dtype=np.uint8)
        hp = np.zeros(self.n_in_blocks, dtype=np.uint32)
        up = np.zeros(self.n_in_blocks, dtype=np.uint32)
        self._l.okv_block_state(self._t, self.n_in_blocks, _p(priv), _p(hp), _p(up))
        return priv, hp, up

    def reset_counters(self):
        self._l.okv_counters_reset(self._t)


def gather(kpool: torch.Tensor, vpool: torch.Tensor, matched_len, page_table):
    """Per-request contiguous copies of the matched K / V pages: [sum L_r, Hkv, d] each."""
    matched_len, page_table = _i32(matched_len), _i32(page_table)
    n_tok = int(matched_len.sum())
    kctx = torch.empty((n_tok,) + tuple(kpool.shape[2:]), dtype=kpool.dtype)
    vctx = torch.empty_like(kctx)
    page_bytes = kpool[0].numel() * kpool.element_size()
    lib().okv_gather(page_bytes, len(matched_len), _p(matched_len), _p(page_table),
                     page_table.shape[1] if page_table.ndim == 2 else 0, _p(kpool), _p(vpool),
                     _p(kctx), _p(vctx))
    return kctx, vctx


def scatter(knew: torch.Tensor, vnew: torch.Tensor, q_off, new_pages, kpool: torch.Tensor, vpool: torch.Tensor):
    """Write the full blocks of every request's new K / V rows into the pool pages new_pages[r][j] (in place)."""
    q_off, new_pages = _i32(q_off), _i32(new_pages)
    row_bytes = knew[0].numel() * knew.element_size()
    assert kpool[0].numel() * kpool.element_size() == row_bytes * BLOCK
    lib().okv_scatter(row_bytes, len(q_off) - 1, _p(q_off), _p(new_pages), new_pages.shape[1], _p(knew.contiguous()),
                      _p(vnew.contiguous()), _p(kpool), _p(vpool))


def attention(q, knew, vnew, q_off, kpool, vpool, matched_len, page_table, scale=None, rows=None,
              n_threads=1):
    """fp64 causal GQA attention of the uncached suffixes over paged prefix + own new KV.

    q [sum S, Hq, d]; knew/vnew [sum S, Hkv, d]; kpool/vpool [n_pages, 16, Hkv, d] (fp32 or
    bf16 CPU tensors).  rows=None: returns float64 [sum S, Hq, d]; rows=(req, head, pos) int
    arrays: returns float64 [n_rows, d]."""
    dt = q.dtype
    assert all(t.dtype == dt for t in (knew, vnew, kpool, vpool))
    code = {torch.float32: 0, torch.bfloat16: 1}[dt]
    Hq, d = q.shape[1], q.shape[2]
    Hkv = kpool.shape[2]
    assert kpool.shape[1] == BLOCK and kpool.shape[3] == d and knew.shape[1] == Hkv
    q_off, matched_len, page_table = _i32(q_off), _i32(matched_len), _i32(page_table)
    R = len(matched_len)
    max_blocks = page_table.shape[1]
    assert page_table.shape[0] == R and int(q_off[-1]) == q.shape[0]
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    if rows is None:
        out = np.zeros((q.shape[0], Hq, d), dtype=np.float64)
        n_rows, rr, rh, rp = -1, None, None, None
    else:
        rr, rh, rp = (_i32(x) for x in rows)
        n_rows = len(rr)
        out = np.zeros((n_rows, d), dtype=np.float64)
    rc = lib().okv_attention(code, Hq, Hkv, d, float(scale), R, _p(q_off), _p(q.contiguous()),
                             _p(knew.contiguous()), _p(vnew.contiguous()), _p(kpool), _p(vpool),
                             _p(matched_len), _p(page_table), max_blocks, n_rows, _p(rr), _p(rh),
                             _p(rp), _p(out), int(n_threads))
    if rc:
        raise ValueError("oracle attention: bad shapes")
    return out
