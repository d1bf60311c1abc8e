"""End to end on the GPU, step after step, as a serving loop would call the library (Section 4.1 overview):
lookup -> prefill attention over reused pages + new tokens -> the new KV blocks are written to fresh pool pages
and inserted as the requester's private copies -> some blocks are promoted -> window roll (demotions) and eviction
free pages that later steps hand out again.  Later steps reuse pages that earlier steps of the same run wrote on
the device.  Every step is mirrored on the oracle (its own tree, host pools written by its own scatter): lookups,
attention outputs, insert and eviction results must agree at each step, and in the end the pools byte for byte."""
import numpy as np
import pytest
import torch

import oracle
from paper_2508_08438_amd.inputs import BLOCK as B
from test_oracle_insert import make_round

pytestmark = pytest.mark.gpu


def run_stream(seed, dtype, hq, hkv, d, n_steps=5, n_req=8, vocab=3, n_tenants=3, n_pages=1024, tol=2e-2):
    from paper_2508_08438_amd import binding as skv
    dev = "cuda:0"
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    g = np.random.default_rng(seed)
    empty = (np.zeros(0, np.int32), np.array([0]), np.zeros(0, np.uint8), np.zeros(0, np.int32), np.zeros(0, np.int32))
    otree = oracle.OracleTree(*empty)
    dtree = skv.skv_tree_build(*empty, n_tenants, n_pages, device=dev, reserve_blocks=4096)
    desc = skv.attn_desc(hq, hkv, d, dtype)
    kpool_h = torch.zeros((n_pages, B, hkv, d), dtype=tdt)
    vpool_h = torch.zeros_like(kpool_h)
    kpool_d, vpool_d = kpool_h.to(dev), vpool_h.to(dev)
    free = list(range(n_pages))[::-1]
    earlier = []
    pol = dict(direction=0, tau=(1, 2), min_hits=2, n_consec=1, u_pre_max=1)
    n_dem = torch.zeros(1, dtype=torch.int32, device=dev)
    reused_tokens = 0
    for step in range(n_steps):
        otree.set_epoch(step + 1)
        skv.skv_set_epoch(dtree, step + 1)
        reqs, off, toks, tenants = make_round(g, earlier, vocab, n_tenants, n_req, None)
        mb = max(max(len(x) // B for x in reqs), 1)
        # 1. lookup
        off_d, toks_d, ten_d = (torch.from_numpy(a).to(dev) for a in (off, toks if len(toks) else np.zeros(1, np.int32), tenants))
        mlen_d = torch.zeros(n_req, dtype=torch.int32, device=dev)
        pt_d = torch.full((n_req, mb), -1, dtype=torch.int32, device=dev)
        skv.skv_match(dtree, off_d, toks_d, ten_d, mb, mlen_d, pt_d)
        o_mlen, o_pt, o_ids = otree.match(off, toks, tenants, mb, want_ids=True)
        torch.cuda.synchronize()
        mlen = mlen_d.cpu().numpy()
        assert np.array_equal(mlen, o_mlen) and np.array_equal(pt_d.cpu().numpy(), o_pt), (seed, step)
        reused_tokens += int(mlen.sum())
        # 2. prefill attention of the uncached suffixes
        q_off_d = torch.zeros(n_req + 1, dtype=torch.int32, device=dev)
        skv.skv_suffix_offsets(off_d, mlen_d, q_off_d)
        q_off = np.concatenate([[0], np.cumsum(np.diff(off) - mlen)]).astype(np.int32)
        T = int(q_off[-1])
        gen = torch.Generator().manual_seed(seed * 100 + step)
        q = torch.randn((max(T, 1), hq, d), generator=gen).to(tdt)[:T]
        knew = torch.randn((max(T, 1), hkv, d), generator=gen).to(tdt)[:T]
        vnew = torch.randn((max(T, 1), hkv, d), generator=gen).to(tdt)[:T]
        if T:
            out_d = torch.zeros((T, hq, d), dtype=tdt, device=dev)
            ws = torch.zeros(skv.skv_prefill_attn_workspace_size(desc, n_req, T), dtype=torch.uint8, device=dev)
            q_d, knew_d, vnew_d = q.to(dev), knew.to(dev), vnew.to(dev)
            skv.skv_prefill_attn(desc, q_d, knew_d, vnew_d, q_off_d, kpool_d, vpool_d, mlen_d, pt_d, mb, out_d, ws)
            want = oracle.attention(q, knew, vnew, q_off, kpool_h, vpool_h, o_mlen, o_pt, n_threads=8)
            torch.cuda.synchronize()
            assert np.array_equal(q_off_d.cpu().numpy(), q_off)
            err = np.abs(out_d.double().cpu().numpy() - want).max()
            assert err <= tol, (seed, step, err)
        # 3. the new full blocks go to fresh pages and into the index as the requester's own copies
        full = (np.diff(off) - mlen) // B
        new_pages = np.full((n_req, int(full.max()) + 1), -1, np.int32)
        for r in range(n_req):
            for j in range(int(full[r])):
                new_pages[r, j] = free.pop()
        if T:
            skv.skv_scatter_kv(desc, knew_d, vnew_d, q_off_d, torch.from_numpy(new_pages).to(dev), kpool_d, vpool_d)
            oracle.scatter(knew, vnew, q_off, new_pages, kpool_h, vpool_h)
        first, n = skv.skv_tree_insert(dtree, off, toks, tenants, mlen, new_pages, private_copies=True)
        o_first, o_n = otree.insert(off, toks, tenants, mlen, new_pages, private_copies=True)
        assert np.array_equal(first, o_first) and np.array_equal(n, o_n), (seed, step)
        for r in range(n_req):                       # pages of blocks that were not inserted go back
            used = int(first[r]) - int(mlen[r]) // B + int(n[r]) if n[r] else 0
            for j in range(int(full[r])):
                if not (n[r] and (first[r] - mlen[r] // B) <= j < used):
                    free.append(int(new_pages[r, j]))
        # 4. the verifier clears some blocks; the safeguard may take some back; eviction frees pages
        priv = otree.block_state()[0]
        alive = np.flatnonzero(priv != 255)
        pick = alive[g.random(len(alive)) < 0.4].astype(np.int32)
        if len(pick):
            skv.skv_promote(dtree, torch.from_numpy(pick).to(dev))
            otree.promote(pick)
        if step % 2 == 1:
            skv.skv_window_roll(dtree, skv.rdr_policy(**pol), n_dem)
            want_dem = otree.window_roll(**pol)
            assert int(n_dem.item()) == want_dem
            n_want = otree.n_blocks // 5
            ids, pages = skv.skv_evict(dtree, n_want, o_ids[o_ids >= 0].astype(np.int32))
            want_ids, want_pages = otree.evict(n_want, o_ids[o_ids >= 0])
            assert np.array_equal(ids, want_ids) and np.array_equal(pages, want_pages), (seed, step)
            free += [int(p) for p in pages]
        earlier += reqs
    torch.cuda.synchronize()
    bits = torch.int16 if dtype == "bf16" else torch.int32
    assert torch.equal(kpool_d.cpu().view(bits), kpool_h.view(bits)) and torch.equal(vpool_d.cpu().view(bits), vpool_h.view(bits))
    return reused_tokens


def test_serving_stream_bf16():
    total = 0
    for seed in range(6):
        print(f"[stream] bf16 {seed}", flush=True)
        total += run_stream(seed, "bf16", 8, 2, 128)
    assert total > 500          # later steps did reuse what earlier steps cached


def test_serving_stream_fp32():
    total = 0
    for seed in range(4):
        print(f"[stream] fp32 {seed}", flush=True)
        total += run_stream(10 + seed, "f32", 4, 2, 64, tol=1e-4)
    assert total > 300
