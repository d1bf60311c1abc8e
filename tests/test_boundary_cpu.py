"""The C-ABI library without a GPU: it loads, exports every symbol the header declares, and
rejects malformed arguments before any device work."""
import ctypes as C
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def skv():
    from paper_2508_08438_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2508_08438_amd.build import build_lib
        build_lib()
    binding.lib()
    return binding


def test_library_exports_every_declared_symbol(skv):
    header = open(os.path.join(ROOT, "include", "skv.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(skv_[a-z_0-9]+)\s*\(", header))
    assert declared == set(skv.EXPORTS)
    for name in declared:
        assert hasattr(skv.lib(), name), name


def test_error_strings(skv):
    l = skv.lib()
    assert l.skv_strerror(0) == b"ok"
    for code in (-1, -2, -3, -4, -99):
        assert len(l.skv_strerror(code)) > 0


def _desc_args(n_blocks=4, n_tenants=3, n_pages=8):
    tokens = np.arange(n_blocks * 16, dtype=np.int32)
    return dict(seq_tokens=tokens, seq_off=np.array([0, n_blocks * 16]), blk_sensitive=np.zeros(n_blocks),
                blk_owner=np.zeros(n_blocks), blk_page=np.arange(n_blocks), n_tenants=n_tenants, n_pages=n_pages)


def test_tree_desc_validation(skv):
    ok = skv.skv_tree_build_size(**_desc_args())
    assert ok > 0 and ok % 256 == 0
    assert skv.skv_tree_build_size(**_desc_args(n_blocks=0)) > 0

    def bad(code, **kw):
        a = _desc_args()
        a.update(kw)
        with pytest.raises(skv.SkvError) as e:
            skv.skv_tree_build_size(**a)
        assert e.value.code == code

    bad(-1, block_tokens=32)
    bad(-3, n_tenants=129)
    bad(-3, n_tenants=0)
    bad(-1, n_pages=0)
    bad(-1, seq_off=np.array([0, 60]))          # not a multiple of 16
    bad(-1, seq_off=np.array([0, 64, 32]))      # decreasing
    bad(-1, seq_off=np.array([16, 64]))         # does not start at 0


def test_build_rejects_bad_blocks_before_touching_the_device(skv):
    l = skv.lib()
    out = C.c_void_p()
    fake_slab = C.c_void_p(256 * 1024)  # never dereferenced: validation fails first

    def rc(**kw):
        a = _desc_args()
        a.update(kw)
        d, keep = skv._tree_desc(**a)
        return l.skv_tree_build(C.byref(d), fake_slab, 1 << 20, None, C.byref(out))

    assert rc(blk_owner=np.array([0, 3, 0, 0])) == -1      # owner outside [0, n_tenants)
    assert rc(blk_owner=np.array([0, -1, 0, 0])) == -1
    assert rc(blk_page=np.array([0, 1, 8, 2])) == -1       # page outside [0, n_pages)
    assert rc(blk_page=np.array([0, 1, 1, 2])) == -1       # one page backing two cached blocks
    d, keep = skv._tree_desc(**_desc_args())
    assert l.skv_tree_build(C.byref(d), C.c_void_p(256 * 1024 + 8), 1 << 20, None, C.byref(out)) == -1  # misaligned
    assert l.skv_tree_build(C.byref(d), None, 1 << 20, None, C.byref(out)) == -1
    assert l.skv_tree_build(C.byref(d), fake_slab, 64, None, C.byref(out)) == -2  # slab too small
    assert l.skv_tree_build(None, fake_slab, 64, None, C.byref(out)) == -1


def test_attention_and_gather_argument_checks(skv):
    import torch
    l = skv.lib()
    n = C.c_size_t()
    for bad in (skv.attn_desc(8, 3, 128, "bf16"), skv.attn_desc(8, 2, 64, "bf16"), skv.attn_desc(8, 2, 96, "f32"),
                skv.AttnDesc(8, 2, 128, 7, 1.0)):
        assert l.skv_prefill_attn_workspace_size(C.byref(bad), 4, 100, C.byref(n)) == -1
    good = skv.attn_desc(32, 8, 128, torch.bfloat16)
    assert l.skv_prefill_attn_workspace_size(C.byref(good), 4, 1000, C.byref(n)) == 0 and n.value >= 256
    assert l.skv_prefill_attn_workspace_size(C.byref(good), -1, 1000, C.byref(n)) == -1
    args = [None] * 4 + [100, None, None, 8, None, None, 4, None, None, 0, None]
    assert l.skv_prefill_attn(C.byref(good), 4, *args) == -1          # null tensors
    assert l.skv_prefill_attn(C.byref(good), 0, *args) == 0           # empty batch: nothing to do
    assert l.skv_gather_kv(C.byref(good), 4, None, None, 8, None, None, 4, None, None, None, 0, None) == -1
    assert l.skv_match(None, 1, None, None, None, 1, None, None, None, None) == -1
    assert l.skv_counters_reset(None, None) == -1
    assert l.skv_suffix_offsets(2, None, None, None, None) == -1


def test_no_fallback_when_library_is_missing(skv, monkeypatch):
    monkeypatch.setattr(skv, "_lib", None)
    monkeypatch.setattr(skv, "LIB_PATH", "/nonexistent/libskv.so")
    with pytest.raises(RuntimeError):
        skv.lib()


def test_window_roll_argument_checks(skv):
    l = skv.lib()
    ok = skv.rdr_policy()
    assert l.skv_window_roll(None, C.byref(ok), None, None) == -1
    assert l.skv_block_state_read(None, None, None, None, None) == -1


def test_insert_evict_scatter_decode_argument_checks(skv):
    l = skv.lib()
    n = C.c_size_t()
    k = C.c_int64()
    # tree-side calls need a tree handle
    assert l.skv_tree_insert(None, 1, None, None, None, None, None, 0, 0, None, None, None, None) == -1
    assert l.skv_evict(None, 1, None, 0, None, None, C.byref(k), None) == -1
    assert l.skv_promote(None, None, 0, None) == -1
    assert l.skv_set_epoch(None, 3) == -1
    assert l.skv_block_epochs_read(None, None, None) == -1
    assert l.skv_tree_size_for_capacity(-1, C.byref(n)) == -1
    assert l.skv_tree_size_for_capacity(1 << 40, C.byref(n)) == -3
    assert l.skv_tree_size_for_capacity(1000, C.byref(n)) == 0 and n.value % 256 == 0 and n.value >= 1000 * 200
    small, big = C.c_size_t(), C.c_size_t()
    l.skv_tree_size_for_capacity(10, C.byref(small))
    l.skv_tree_size_for_capacity(11, C.byref(big))
    assert big.value >= small.value
    # scatter: description and pointers
    good = skv.attn_desc(32, 8, 128, "bf16")
    assert l.skv_scatter_kv(None, 1, None, None, None, None, 1, None, None, 4, None) == -1
    assert l.skv_scatter_kv(C.byref(good), 1, None, None, None, None, 1, None, None, 4, None) == -1   # null tensors
    assert l.skv_scatter_kv(C.byref(good), 0, None, None, None, None, 1, None, None, 4, None) == 0    # empty batch
    assert l.skv_scatter_kv(C.byref(skv.AttnDesc(8, 2, 128, 9, 1.0)), 1, None, None, None, None, 1, None, None, 4, None) == -1
    # decode: bf16, d 128, at most 16 query heads per kv head
    for bad in (skv.attn_desc(8, 2, 64, "bf16"), skv.attn_desc(8, 2, 128, "f32"), skv.attn_desc(34, 2, 128, "bf16"),
                skv.attn_desc(8, 3, 128, "bf16")):
        assert l.skv_decode_attn_workspace_size(C.byref(bad), 4, 16, C.byref(n)) == -1
    assert l.skv_decode_attn_workspace_size(C.byref(good), 4, 16, C.byref(n)) == 0 and n.value > 0
    assert l.skv_decode_attn_workspace_size(C.byref(good), -1, 16, C.byref(n)) == -1
    args = [None, None, None, 4, None, None, 16, None, None, 0, None]
    assert l.skv_decode_attn(C.byref(good), 4, *args) == -1          # null tensors
    assert l.skv_decode_attn(C.byref(good), 0, *args) == 0           # empty batch


def test_static_scratch_attention_rejects_oversized_batches_before_touching_the_device(skv):
    l = skv.lib()
    good = skv.attn_desc(32, 8, 128, "bf16")
    n = C.c_size_t()
    rows = 1 << 28
    assert l.skv_prefill_attn_workspace_size(C.byref(good), 4, rows, C.byref(n)) == 0 and n.value > (4 << 20)
    fake = C.c_void_p(1 << 20)   # aligned, never dereferenced: the size check fails first
    args = [fake, fake, fake, fake, rows, fake, fake, 8, fake, fake, 4, fake, None]
    assert l.skv_prefill_attn_static(C.byref(good), 4, *args) == -3
    assert l.skv_prefill_attn_static(C.byref(good), 0, *args) == 0           # empty batch
    args[0] = None
    assert l.skv_prefill_attn_static(C.byref(good), 4, *args) == -1          # null tensor
    assert l.skv_prefill_attn_static(None, 4, *args) == -1


def test_limits_read_and_stream_copy_argument_checks(skv):
    l = skv.lib()
    fake_ptr = C.c_void_p(1 << 20)
    v = C.c_uint32()
    assert l.skv_match_limits_read(None, C.byref(v), 1, None) == -1
    assert l.skv_tree_compact(None, None, None, None) == -1
    assert l.skv_mfma_rate(None, 0, 1, 0, None, 0, None, None) == -1
    assert l.skv_mfma_rate(fake_ptr, 64, 1, 0, fake_ptr, 64, None, None) == -2     # buffers too small
    assert l.skv_mfma_rate(fake_ptr, 1 << 40, 0, 0, fake_ptr, 1 << 40, None, None) == -1   # iters < 1
    assert l.skv_mfma_rate(fake_ptr, 1 << 40, 1, 2, fake_ptr, 1 << 40, None, None) == -1   # side_work is 0 or 1
    fake = C.c_void_p(1 << 20)
    assert l.skv_stream_copy(fake, fake, 0, None) == 0                 # nothing to copy
    assert l.skv_stream_copy(None, fake, 64, None) == -1
    assert l.skv_stream_copy(fake, fake, 24, None) == -1               # not a multiple of 16
    assert l.skv_stream_copy(C.c_void_p((1 << 20) + 4), fake, 64, None) == -1


def test_no_reader_of_an_mfma_result_sits_right_behind_a_branch():
    """Compiles the two MFMA kernels to assembly and scans them (see mfma_hazard_scan): 12 idle states cover the
    8-pass 32x32x16 and the 4-pass 16x16x32 instructions the kernels use."""
    import os, subprocess, tempfile
    from mfma_hazard_scan import scan
    from paper_2508_08438_amd import build
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = [f for f in build.FLAGS if f not in ("-shared", "-fPIC")]
    for src, kernel in (("skv_attn.hip", "attn_bf16_kernel"), ("skv_decode.hip", "decode_attn_kernel")):
        with tempfile.TemporaryDirectory() as tmp:
            out = os.path.join(tmp, "k.s")
            r = subprocess.run([hipcc, *flags, "--cuda-device-only", "-S", "-I", build.INCLUDE, "-I", build.CSRC, "-o", out,
                                os.path.join(build.CSRC, src)], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
            assert r.returncode == 0, r.stdout
            found = scan(open(out).read(), kernel)
        assert not found, (kernel, found)
