"""Thin ctypes binding of libskv.so: same names as the C ABI, argument marshalling only.

Every step of the path runs in the library's kernels; torch is used for device memory and
streams.  There is no fallback: if the library is not built, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libskv.so")
BLOCK = 16
SKV_F32, SKV_BF16 = 0, 1
SKV_OK, SKV_EINVAL, SKV_ENOMEM, SKV_ERANGE, SKV_EHIP = 0, -1, -2, -3, -4
SKV_LIMIT_BRANCH_POINTS, SKV_LIMIT_COPIES, SKV_LIMIT_WALKS = 1, 2, 4

EXPORTS = ["skv_strerror", "skv_last_hip_error", "skv_tree_build_size", "skv_tree_size_for_capacity", "skv_tree_build", "skv_tree_insert", "skv_set_epoch", "skv_block_epochs_read", "skv_evict", "skv_tree_compact", "skv_mfma_rate",
           "skv_tree_info", "skv_tree_destroy", "skv_match", "skv_match_limits_read", "skv_counters_read",
           "skv_counters_reset", "skv_window_roll", "skv_promote", "skv_block_state_read", "skv_suffix_offsets", "skv_gather_kv",
           "skv_scatter_kv", "skv_stream_copy", "skv_decode_attn_workspace_size", "skv_decode_attn",
           "skv_prefill_attn_workspace_size", "skv_prefill_attn", "skv_prefill_attn_static"]


class SkvError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        msg = lib().skv_strerror(code).decode()
        if code == -4:
            msg += f" (hipError {lib().skv_last_hip_error()})"
        super().__init__(f"{where}: {msg} [{code}]")


class TreeDesc(C.Structure):
    _fields_ = [("block_tokens", C.c_int32), ("n_tenants", C.c_int32), ("n_pages", C.c_int32),
                ("n_seq", C.c_int64), ("seq_off", C.c_void_p), ("tokens", C.c_void_p),
                ("blk_sensitive", C.c_void_p), ("blk_owner", C.c_void_p), ("blk_page", C.c_void_p)]


class AttnDesc(C.Structure):
    _fields_ = [("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("dtype", C.c_int32), ("scale", C.c_float)]


class RdrPolicy(C.Structure):
    _fields_ = [("direction", C.c_int32), ("tau_num", C.c_uint32), ("tau_den", C.c_uint32),
                ("min_hits", C.c_uint32), ("n_consec", C.c_uint32), ("u_pre_max", C.c_uint32)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is not built: run __graft_entry__.build() "
                               "(there is no fallback path)")
        l = C.CDLL(LIB_PATH)
        vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
        l.skv_strerror.restype = C.c_char_p
        l.skv_strerror.argtypes = [C.c_int]
        l.skv_tree_build_size.argtypes = [C.POINTER(TreeDesc), C.POINTER(C.c_size_t)]
        l.skv_tree_build.argtypes = [C.POINTER(TreeDesc), vp, C.c_size_t, vp, C.POINTER(vp)]
        l.skv_tree_info.argtypes = [vp, C.POINTER(i64), C.POINTER(i64), C.POINTER(i64)]
        l.skv_tree_destroy.argtypes = [vp]
        l.skv_tree_destroy.restype = None
        l.skv_match.argtypes = [vp, i32, vp, vp, vp, i32, vp, vp, vp, vp]
        l.skv_counters_read.argtypes = [vp, vp, vp, vp]
        l.skv_counters_reset.argtypes = [vp, vp]
        l.skv_window_roll.argtypes = [vp, C.POINTER(RdrPolicy), vp, vp]
        l.skv_block_state_read.argtypes = [vp, vp, vp, vp, vp]
        l.skv_promote.argtypes = [vp, vp, i32, vp]
        l.skv_decode_attn_workspace_size.argtypes = [C.POINTER(AttnDesc), i32, i32, C.POINTER(C.c_size_t)]
        l.skv_decode_attn.argtypes = [C.POINTER(AttnDesc), i32, vp, vp, vp, i32, vp, vp, i32, vp, vp, C.c_size_t, vp]
        l.skv_set_epoch.argtypes = [vp, C.c_uint32]
        l.skv_block_epochs_read.argtypes = [vp, vp, vp]
        l.skv_evict.argtypes = [vp, C.c_int64, vp, C.c_int64, vp, vp, C.POINTER(C.c_int64), vp]
        l.skv_tree_size_for_capacity.argtypes = [C.c_int64, C.POINTER(C.c_size_t)]
        l.skv_tree_insert.argtypes = [vp, i32, vp, vp, vp, vp, vp, i32, i32, vp, vp, vp, vp]
        l.skv_scatter_kv.argtypes = [C.POINTER(AttnDesc), i32, vp, vp, vp, vp, i32, vp, vp, i32, vp]
        l.skv_suffix_offsets.argtypes = [i32, vp, vp, vp, vp]
        l.skv_gather_kv.argtypes = [C.POINTER(AttnDesc), i32, vp, vp, i32, vp, vp, i32, vp, vp, vp, i64, vp]
        l.skv_prefill_attn_workspace_size.argtypes = [C.POINTER(AttnDesc), i32, i64, C.POINTER(C.c_size_t)]
        l.skv_prefill_attn.argtypes = [C.POINTER(AttnDesc), i32, vp, vp, vp, vp, i64, vp, vp, i32, vp, vp,
                                       i32, vp, vp, C.c_size_t, vp]
        l.skv_prefill_attn_static.argtypes = [C.POINTER(AttnDesc), i32, vp, vp, vp, vp, i64, vp, vp, i32, vp, vp,
                                              i32, vp, vp]
        l.skv_stream_copy.argtypes = [vp, vp, C.c_size_t, vp]
        l.skv_tree_compact.argtypes = [vp, vp, C.POINTER(i64), vp]
        l.skv_mfma_rate.argtypes = [vp, C.c_size_t, i32, i32, vp, C.c_size_t, C.POINTER(C.c_double), vp]
        l.skv_match_limits_read.argtypes = [vp, C.POINTER(C.c_uint32), i32, vp]
        _lib = l
    return _lib


def _check(code, where):
    if code != 0:
        raise SkvError(code, where)


def _dptr(t):
    if t is None:
        return None
    assert isinstance(t, torch.Tensor) and t.is_cuda and t.is_contiguous(), "device tensor expected"
    return C.c_void_p(t.data_ptr())


def _stream(stream):
    s = stream if stream is not None else torch.cuda.current_stream()
    return C.c_void_p(s.cuda_stream)


def attn_desc(n_q_heads, n_kv_heads, head_dim, dtype, scale=None) -> AttnDesc:
    code = {torch.float32: SKV_F32, torch.bfloat16: SKV_BF16, "f32": SKV_F32, "bf16": SKV_BF16}[dtype]
    return AttnDesc(n_q_heads, n_kv_heads, head_dim, code, float(scale if scale is not None else 0.0))


class Tree:
    """Owner of a tree handle and of the torch tensor that backs its device slab."""

    def __init__(self, handle, slab):
        self.handle, self.slab = handle, slab
        self._destroy = lib().skv_tree_destroy   # bound now: module globals may be gone when __del__ runs at exit

    def info(self):
        a, b, c = C.c_int64(), C.c_int64(), C.c_int64()
        _check(lib().skv_tree_info(self.handle, C.byref(a), C.byref(b), C.byref(c)), "skv_tree_info")
        return {"n_nodes": a.value, "n_blocks": b.value, "n_in_blocks": c.value}

    def __del__(self):
        if getattr(self, "handle", None):
            self._destroy(self.handle)
            self.handle = None


def _tree_desc(seq_tokens, seq_off, blk_sensitive, blk_owner, blk_page, n_tenants, n_pages,
               block_tokens=BLOCK):
    keep = [np.ascontiguousarray(seq_off, dtype=np.int64), np.ascontiguousarray(seq_tokens, dtype=np.int32),
            np.ascontiguousarray(blk_sensitive, dtype=np.uint8), np.ascontiguousarray(blk_owner, dtype=np.int32),
            np.ascontiguousarray(blk_page, dtype=np.int32)]
    ptr = [C.c_void_p(a.ctypes.data) if a.size or i == 0 else None for i, a in enumerate(keep)]
    d = TreeDesc(block_tokens, n_tenants, n_pages, len(keep[0]) - 1, *ptr)
    return d, keep


def skv_tree_build_size(seq_tokens, seq_off, blk_sensitive, blk_owner, blk_page, n_tenants, n_pages,
                        block_tokens=BLOCK) -> int:
    d, _keep = _tree_desc(seq_tokens, seq_off, blk_sensitive, blk_owner, blk_page, n_tenants, n_pages,
                          block_tokens)
    n = C.c_size_t()
    _check(lib().skv_tree_build_size(C.byref(d), C.byref(n)), "skv_tree_build_size")
    return n.value


def skv_tree_size_for_capacity(block_capacity: int) -> int:
    n = C.c_size_t()
    _check(lib().skv_tree_size_for_capacity(block_capacity, C.byref(n)), "skv_tree_size_for_capacity")
    return n.value


def skv_tree_build(seq_tokens, seq_off, blk_sensitive, blk_owner, blk_page, n_tenants, n_pages,
                   device="cuda", stream=None, reserve_blocks=0) -> Tree:
    """reserve_blocks: room, beyond the described blocks, for blocks inserted later."""
    d, _keep = _tree_desc(seq_tokens, seq_off, blk_sensitive, blk_owner, blk_page, n_tenants, n_pages)
    n = C.c_size_t()
    _check(lib().skv_tree_build_size(C.byref(d), C.byref(n)), "skv_tree_build_size")
    if reserve_blocks:
        _check(lib().skv_tree_size_for_capacity(len(_keep[4]) + reserve_blocks, C.byref(n)), "skv_tree_size_for_capacity")
    slab = torch.empty(n.value, dtype=torch.uint8, device=device)
    h = C.c_void_p()
    with torch.cuda.device(slab.device):
        _check(lib().skv_tree_build(C.byref(d), _dptr(slab), n.value, _stream(stream), C.byref(h)),
               "skv_tree_build")
    return Tree(h, slab)


def skv_tree_insert(tree: Tree, req_off, req_tokens, req_tenant, matched_len, new_pages, private_copies=False,
                    stream=None, path_end=None):
    """Host arrays in (numpy int32), per-request (first_inserted, n_inserted) out.  path_end: the lookup's path ends
    for this batch (host copy), copies mode only."""
    a = [np.ascontiguousarray(x, dtype=np.int32) for x in (req_off, req_tokens, req_tenant, matched_len, new_pages)]
    n_req = len(a[2])
    assert len(a[0]) == n_req + 1 and len(a[3]) == n_req and a[4].ndim == 2 and a[4].shape[0] == n_req
    first = np.zeros(n_req, dtype=np.int32)
    n = np.zeros(n_req, dtype=np.int32)
    hp = lambda x: C.c_void_p(x.ctypes.data) if x.size else None
    with torch.cuda.device(tree.slab.device):
        pe = None if path_end is None else np.ascontiguousarray(path_end, dtype=np.int32)
        assert pe is None or len(pe) == n_req
        _check(lib().skv_tree_insert(tree.handle, n_req, hp(a[0]), hp(a[1]), hp(a[2]), hp(a[3]), hp(a[4]),
                                     a[4].shape[1], int(private_copies), None if pe is None else C.c_void_p(pe.ctypes.data),
                                     hp(first), hp(n), _stream(stream)),
               "skv_tree_insert")
    return first, n


def skv_set_epoch(tree: Tree, epoch: int):
    _check(lib().skv_set_epoch(tree.handle, epoch), "skv_set_epoch")


def skv_block_epochs_read(tree: Tree, epoch, stream=None):
    assert epoch.dtype == torch.int32 and epoch.numel() >= tree.info()["n_in_blocks"]
    _check(lib().skv_block_epochs_read(tree.handle, _dptr(epoch), _stream(stream)), "skv_block_epochs_read")


def skv_evict(tree: Tree, n_want: int, protect_ids=(), stream=None):
    """Returns (block ids, pages) of the evicted blocks, in eviction order (numpy int32)."""
    prot = np.ascontiguousarray(protect_ids, dtype=np.int32)
    ids = np.zeros(max(n_want, 1), dtype=np.int32)
    pages = np.zeros(max(n_want, 1), dtype=np.int32)
    k = C.c_int64()
    hp = lambda x: C.c_void_p(x.ctypes.data) if x.size else None
    with torch.cuda.device(tree.slab.device):
        _check(lib().skv_evict(tree.handle, n_want, hp(prot), len(prot), hp(ids), hp(pages), C.byref(k),
                               _stream(stream)), "skv_evict")
    return ids[: k.value], pages[: k.value]


MFMA_RATE_OPERAND_BYTES = 512 * 512 * 6 * 32
MFMA_RATE_SINK_BYTES = 512 * 512 * 4


def skv_mfma_rate(operands: torch.Tensor, iters: int, sink: torch.Tensor, stream=None, side_work: bool = False) -> float:
    """Enqueues the matrix-rate kernel; returns the floating-point operations it issues."""
    flops = C.c_double()
    _check(lib().skv_mfma_rate(_dptr(operands), operands.numel() * operands.element_size(), iters, int(side_work),
                               _dptr(sink), sink.numel() * sink.element_size(), C.byref(flops), _stream(stream)),
           "skv_mfma_rate")
    return flops.value


def skv_tree_compact(tree: Tree, stream=None):
    """Returns id_map (numpy int32, old input block id -> new id, -1 if gone)."""
    n = tree.info()["n_in_blocks"]
    id_map = np.full(max(n, 1), -1, dtype=np.int32)
    after = C.c_int64()
    with torch.cuda.device(tree.slab.device):
        _check(lib().skv_tree_compact(tree.handle, C.c_void_p(id_map.ctypes.data), C.byref(after), _stream(stream)),
               "skv_tree_compact")
    return id_map[:n]


def skv_match(tree: Tree, req_off, req_tokens, req_tenant, max_blocks, matched_len, page_table, stream=None,
              path_end=None):
    n_req = req_tenant.numel()
    assert path_end is None or (path_end.dtype == torch.int32 and path_end.numel() >= n_req)
    assert req_off.dtype == req_tokens.dtype == req_tenant.dtype == torch.int32
    assert matched_len.dtype == page_table.dtype == torch.int32
    assert req_off.numel() == n_req + 1 and matched_len.numel() >= n_req
    assert page_table.numel() >= n_req * max_blocks
    _check(lib().skv_match(tree.handle, n_req, _dptr(req_off), _dptr(req_tokens), _dptr(req_tenant),
                           max_blocks, _dptr(matched_len), _dptr(page_table),
                           _dptr(path_end) if path_end is not None else None, _stream(stream)), "skv_match")


def skv_match_limits_read(tree: Tree, clear=True, stream=None) -> int:
    v = C.c_uint32()
    with torch.cuda.device(tree.slab.device):
        _check(lib().skv_match_limits_read(tree.handle, C.byref(v), int(clear), _stream(stream)), "skv_match_limits_read")
    return v.value


def skv_counters_read(tree: Tree, hit, ucnt, stream=None):
    n = tree.info()["n_in_blocks"]
    assert hit.numel() >= n and ucnt.numel() >= n and hit.dtype == ucnt.dtype == torch.int32
    _check(lib().skv_counters_read(tree.handle, _dptr(hit), _dptr(ucnt), _stream(stream)), "skv_counters_read")


def skv_counters_reset(tree: Tree, stream=None):
    _check(lib().skv_counters_reset(tree.handle, _stream(stream)), "skv_counters_reset")


def rdr_policy(direction=0, tau=(1, 2), min_hits=1, n_consec=1, u_pre_max=1) -> RdrPolicy:
    return RdrPolicy(direction, tau[0], tau[1], min_hits, n_consec, u_pre_max)


def skv_window_roll(tree: Tree, policy: RdrPolicy, n_demoted=None, stream=None):
    assert n_demoted is None or (n_demoted.dtype == torch.int32 and n_demoted.numel() >= 1)
    _check(lib().skv_window_roll(tree.handle, C.byref(policy), _dptr(n_demoted), _stream(stream)), "skv_window_roll")


def skv_promote(tree: Tree, block_ids, stream=None):
    assert block_ids.dtype == torch.int32
    _check(lib().skv_promote(tree.handle, _dptr(block_ids), block_ids.numel(), _stream(stream)), "skv_promote")


def skv_scatter_kv(desc: AttnDesc, knew, vnew, q_off, new_pages, kpool, vpool, stream=None):
    n_req = q_off.numel() - 1
    assert new_pages.dtype == torch.int32 and new_pages.dim() == 2 and new_pages.shape[0] == n_req
    _check(lib().skv_scatter_kv(C.byref(desc), n_req, _dptr(knew), _dptr(vnew), _dptr(q_off), _dptr(new_pages),
                                new_pages.shape[1], _dptr(kpool), _dptr(vpool), kpool.shape[0], _stream(stream)),
           "skv_scatter_kv")


def skv_stream_copy(dst, src, stream=None):
    nbytes = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() >= nbytes
    _check(lib().skv_stream_copy(_dptr(dst), _dptr(src), nbytes, _stream(stream)), "skv_stream_copy")


def skv_block_state_read(tree: Tree, private, hit_pre, u_pre, stream=None):
    n = tree.info()["n_in_blocks"]
    assert private is None or (private.dtype == torch.uint8 and private.numel() >= n)
    assert all(x is None or (x.dtype == torch.int32 and x.numel() >= n) for x in (hit_pre, u_pre))
    _check(lib().skv_block_state_read(tree.handle, _dptr(private), _dptr(hit_pre), _dptr(u_pre), _stream(stream)),
           "skv_block_state_read")


def skv_suffix_offsets(req_off, matched_len, q_off, stream=None):
    n_req = matched_len.numel()
    assert q_off.numel() == n_req + 1 and q_off.dtype == torch.int32
    _check(lib().skv_suffix_offsets(n_req, _dptr(req_off), _dptr(matched_len), _dptr(q_off), _stream(stream)),
           "skv_suffix_offsets")


def skv_gather_kv(desc: AttnDesc, kpool, vpool, matched_len, page_table, max_blocks, ctx_off, kctx, vctx,
                  stream=None):
    n_req = matched_len.numel()
    assert ctx_off.dtype == torch.int64 and ctx_off.numel() == n_req + 1
    row = desc.n_kv_heads * desc.head_dim
    cap = kctx.numel() // row
    assert vctx.numel() // row >= cap
    _check(lib().skv_gather_kv(C.byref(desc), n_req, _dptr(kpool), _dptr(vpool), kpool.shape[0],
                               _dptr(matched_len), _dptr(page_table), max_blocks, _dptr(ctx_off),
                               _dptr(kctx), _dptr(vctx), cap, _stream(stream)), "skv_gather_kv")


def skv_prefill_attn_workspace_size(desc: AttnDesc, n_req, total_q_rows) -> int:
    n = C.c_size_t()
    _check(lib().skv_prefill_attn_workspace_size(C.byref(desc), n_req, total_q_rows, C.byref(n)),
           "skv_prefill_attn_workspace_size")
    return n.value


def skv_prefill_attn(desc: AttnDesc, q, knew, vnew, q_off, kpool, vpool, matched_len, page_table, max_blocks,
                     out, workspace, stream=None):
    n_req = matched_len.numel()
    total = q.shape[0]
    assert out.shape == q.shape and knew.shape[0] >= total and vnew.shape[0] >= total
    _check(lib().skv_prefill_attn(C.byref(desc), n_req, _dptr(q), _dptr(knew), _dptr(vnew), _dptr(q_off),
                                  total, _dptr(kpool), _dptr(vpool), kpool.shape[0], _dptr(matched_len),
                                  _dptr(page_table), max_blocks, _dptr(out), _dptr(workspace),
                                  workspace.numel() * workspace.element_size(), _stream(stream)),
           "skv_prefill_attn")


def skv_prefill_attn_static(desc: AttnDesc, q, knew, vnew, q_off, kpool, vpool, matched_len, page_table, max_blocks,
                            out, stream=None):
    n_req = matched_len.numel()
    total = q.shape[0]
    assert out.shape == q.shape and knew.shape[0] >= total and vnew.shape[0] >= total
    _check(lib().skv_prefill_attn_static(C.byref(desc), n_req, _dptr(q), _dptr(knew), _dptr(vnew), _dptr(q_off),
                                         total, _dptr(kpool), _dptr(vpool), kpool.shape[0], _dptr(matched_len),
                                         _dptr(page_table), max_blocks, _dptr(out), _stream(stream)),
           "skv_prefill_attn_static")


def skv_decode_attn_workspace_size(desc: AttnDesc, n_req, max_blocks) -> int:
    n = C.c_size_t()
    _check(lib().skv_decode_attn_workspace_size(C.byref(desc), n_req, max_blocks, C.byref(n)),
           "skv_decode_attn_workspace_size")
    return n.value


def skv_decode_attn(desc: AttnDesc, q, kpool, vpool, ctx_len, page_table, max_blocks, out, workspace, stream=None):
    n_req = ctx_len.numel()
    assert q.shape[0] == n_req and out.shape == q.shape and ctx_len.dtype == page_table.dtype == torch.int32
    _check(lib().skv_decode_attn(C.byref(desc), n_req, _dptr(q), _dptr(kpool), _dptr(vpool), kpool.shape[0],
                                 _dptr(ctx_len), _dptr(page_table), max_blocks, _dptr(out), _dptr(workspace),
                                 workspace.numel(), _stream(stream)), "skv_decode_attn")
