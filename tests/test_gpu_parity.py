"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded
inputs.  Integers (matched lengths, page ids, counters, gathered bytes) must be bit-exact;
attention must agree within max-abs 1e-4 (fp32) / 2e-2 (bf16) with the fp64 oracle."""
import numpy as np
import pytest
import torch

import oracle
from paper_2508_08438_amd import inputs
from paper_2508_08438_amd.inputs import BLOCK as B

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}


def _skv():
    from paper_2508_08438_amd import binding
    return binding


def _session(w, **kw):
    from paper_2508_08438_amd.pipeline import Session
    return Session(w, device="cuda:0", **kw)


def check_match(w, label):
    print(f"[match] {label}: R={w.n_req} in_blocks={w.n_in_blocks}", flush=True)
    s = _session(w, with_kv=False)
    s.match()
    torch.cuda.synchronize()
    tree = oracle.OracleTree.from_workload(w)
    mb = max(w.max_blocks, 1)
    mlen, pt = tree.match(w.req_off, w.req_tokens, w.req_tenant, mb)
    hit, ucnt = tree.counters()
    info = s.tree.info()
    assert info["n_blocks"] == tree.n_blocks and info["n_in_blocks"] == w.n_in_blocks
    assert info["n_nodes"] <= tree.n_nodes  # runs that grew past an old leaf are merged here
    assert np.array_equal(s.matched_len.cpu().numpy(), mlen), label
    assert np.array_equal(s.page_table.cpu().numpy(), pt), label
    g_hit, g_ucnt = s.counters()
    assert np.array_equal(g_hit, hit) and np.array_equal(g_ucnt, ucnt), label
    q_off = np.concatenate([[0], np.cumsum(np.diff(w.req_off) - mlen)]).astype(np.int32)
    assert np.array_equal(s.q_off.cpu().numpy(), q_off)
    # a second batch in the same window accumulates; reset starts a new window
    skv = _skv()
    skv.skv_match(s.tree, s.req_off, s.req_tokens, s.req_tenant, s.max_blocks, s.matched_len, s.page_table)
    h2, u2 = s.counters()
    assert np.array_equal(h2, 2 * hit) and np.array_equal(u2, ucnt)
    skv.skv_counters_reset(s.tree)
    h3, u3 = s.counters()
    assert h3.sum() == 0 and u3.sum() == 0
    return s, mlen, pt


def test_match_small_collision_heavy_cases():
    for seed in range(120):
        kw = dict(seed=seed, vocab=2 + seed % 2, n_tenants=1 + seed % 3, p_sens=[0.0, 0.3, 0.6, 1.0][seed % 4],
                  block_vocab=(3 if seed % 5 == 0 else None), n_req=24)
        check_match(inputs.small_random(**kw), f"small{seed}")


def test_match_many_tenants_and_wide_root():
    # 128 tenants (all four bitmap words), hundreds of root children (multi-round probing)
    w = inputs.config5(0.5, n_prefix=600, n_req=300, len_lo=16, len_hi=700, suf_lo=0, suf_hi=40)
    check_match(w, "wide_root")


def test_match_empty_tree_and_empty_batch():
    skv = _skv()
    w = inputs.small_random(seed=1)
    w.seq_tokens, w.seq_off = np.zeros(0, np.int32), np.zeros(1, np.int64)
    w.blk_sensitive, w.blk_owner, w.blk_page = np.zeros(0, np.uint8), np.zeros(0, np.int32), np.zeros(0, np.int32)
    s, mlen, _ = check_match(w, "empty_tree")
    assert mlen.sum() == 0
    z = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    skv.skv_match(s.tree, z, z, z[:0], 4, z, z)  # n_req = 0: no-op
    torch.cuda.synchronize()


def test_match_clamps_requests_longer_than_the_page_table_row():
    """max_blocks smaller than a request's block count: the first max_blocks blocks are considered, as the oracle's
    cap does; lengths, page ids and counters agree."""
    skv = _skv()
    cases = [(inputs.small_random(seed=s, n_req=24, p_sens=0.2), 2) for s in range(20)]
    cases += [(inputs.config2(), 10), (inputs.config4(), 100), (inputs.config3(), 7)]
    for w, cap in cases:
        assert w.max_blocks > cap or w.n_req == 0 or "small" in w.name
        tree = skv.skv_tree_build(w.seq_tokens, w.seq_off, w.blk_sensitive, w.blk_owner, w.blk_page, w.n_tenants,
                                  w.n_pages, device="cuda:0")
        mlen, pt = device_match(skv, tree, w.req_off, w.req_tokens, w.req_tenant, cap)
        otree = oracle.OracleTree.from_workload(w)
        o_mlen, o_pt = otree.match(w.req_off, w.req_tokens, w.req_tenant, cap)
        assert (o_mlen <= cap * B).all() and (o_mlen == cap * B).any(), w.name    # the cap bites
        assert np.array_equal(mlen, o_mlen) and np.array_equal(pt, o_pt), w.name
        compare_state(skv, tree, otree, w.name)


@pytest.mark.parametrize("name", ["c1", "c2", "c3", "c4", "c5"])
def test_match_configs_full_size(name):
    if name == "c5":
        prev = None
        for p in (0.0, 0.25, 0.5, 1.0):
            _, mlen, _ = check_match(inputs.config5(p), f"c5@{p}")
            if prev is not None:
                assert (mlen <= prev).all()
            prev = mlen
    else:
        w = inputs.CONFIGS[name]()
        _, mlen, _ = check_match(w, name)
        if name == "c4":
            assert (mlen == np.diff(w.seq_off)).all()
            check_match(inputs.config4(literal=True), "c4_literal")


def sample_rows(S, n_heads, n, seed=0):
    """(request, head, position) triples over requests with suffix lengths S: always the first/last
    rows and the rows next to tile, page and prefix boundaries, then uniform random ones."""
    g = np.random.default_rng(seed)
    rows = []
    live = [r for r in range(len(S)) if S[r] > 0]
    for r in live[: max(1, n // 64)]:
        for i in {0, 1, 15, 16, 31, 32, 63, 64, 65, 127, 128, S[r] - 2, S[r] - 1}:
            if 0 <= i < S[r]:
                rows.append((r, int(g.integers(0, n_heads)), int(i)))
    while len(rows) < n:
        r = live[int(g.integers(0, len(live)))]
        rows.append((r, int(g.integers(0, n_heads)), int(g.integers(0, S[r]))))
    a = np.array(rows[:n], dtype=np.int32)
    return a[:, 0].copy(), a[:, 1].copy(), a[:, 2].copy()


def oracle_sub_batch(w, reqs, mlen, pt):
    """Oracle inputs for a subset of requests: their Q/K_new/V_new rows and a compact pool holding only
    the pages they reference (pages relabelled in order of first use; the oracle is invariant to that)."""
    reqs = np.asarray(reqs)
    S = (np.diff(w.req_off) - mlen)[reqs]
    q_off = np.concatenate([[0], np.cumsum(S)]).astype(np.int32)
    parts = {x: [] for x in "qkv"}
    for r in reqs:
        lo, hi = int(w.req_off[r]) + int(mlen[r]), int(w.req_off[r + 1])
        for x in "qkv":
            parts[x].append(w.token_rows(x, lo, hi))
    q, kn, vn = (torch.cat(parts[x]) for x in "qkv")
    sub_pt = pt[reqs]
    pages = np.unique(sub_pt[sub_pt >= 0])
    relabel = {int(p): i for i, p in enumerate(pages)}
    cpt = np.vectorize(lambda p: relabel.get(int(p), -1))(sub_pt).astype(np.int32) if sub_pt.size else sub_pt
    a = w.attn
    shape = (max(len(pages), 1), B, a.n_kv_heads, a.head_dim)
    kpool, vpool = torch.zeros(shape, dtype=a.torch_dtype), torch.zeros(shape, dtype=a.torch_dtype)
    for i, pg in enumerate(pages):
        kpool[i] = w.pool_pages("k", int(pg), int(pg) + 1)[0]
        vpool[i] = w.pool_pages("v", int(pg), int(pg) + 1)[0]
    return dict(q=q, knew=kn, vnew=vn, q_off=q_off, kpool=kpool, vpool=vpool, matched_len=mlen[reqs],
                page_table=cpt, scale=a.scale), S


def check_pipeline(w, label, n_sample=None, n_sub_req=None, threads=16):
    print(f"[pipeline] {label}", flush=True)
    s = _session(w)
    res = s.step()
    torch.cuda.synchronize()
    tree = oracle.OracleTree.from_workload(w)
    mlen, pt = tree.match(w.req_off, w.req_tokens, w.req_tenant, max(w.max_blocks, 1))
    assert np.array_equal(res["matched_len"].cpu().numpy(), mlen)
    assert np.array_equal(res["page_table"].cpu().numpy(), pt)
    g_hit, g_ucnt = s.counters()
    hit, ucnt = tree.counters()
    assert np.array_equal(g_hit, hit) and np.array_equal(g_ucnt, ucnt)
    ctx_off = np.concatenate([[0], np.cumsum(mlen.astype(np.int64))])
    assert np.array_equal(res["ctx_off"].cpu().numpy(), ctx_off)
    q_off_all = np.concatenate([[0], np.cumsum(np.diff(w.req_off) - mlen)]).astype(np.int32)
    assert np.array_equal(res["q_off"].cpu().numpy(), q_off_all)
    bits = torch.int32 if w.attn.dtype == "f32" else torch.int16
    # which requests the oracle recomputes: all of them, or a seeded subset that always holds the
    # longest reuse and the longest suffix
    if n_sub_req is None or n_sub_req >= w.n_req:
        reqs = np.arange(w.n_req)
    else:
        g = np.random.default_rng(7)
        S_all = np.diff(w.req_off) - mlen
        reqs = np.unique(np.concatenate([[int(np.argmax(mlen)), int(np.argmax(S_all))],
                                         g.choice(w.n_req, n_sub_req, replace=False)]))
    sub, S = oracle_sub_batch(w, reqs, mlen, pt)
    # gather: byte-exact, request by request
    kc, vc = oracle.gather(sub["kpool"], sub["vpool"], sub["matched_len"], sub["page_table"])
    o = 0
    for r in reqs:
        n = int(mlen[r])
        lo = int(ctx_off[r])
        assert torch.equal(res["kctx"][lo: lo + n].cpu().view(bits), kc[o: o + n].view(bits)), (label, r)
        assert torch.equal(res["vctx"][lo: lo + n].cpu().view(bits), vc[o: o + n].view(bits)), (label, r)
        o += n
    # attention
    if n_sample is None:
        want = oracle.attention(**sub, n_threads=threads)
        got = torch.cat([res["out"][q_off_all[r]: q_off_all[r + 1]] for r in reqs]).double().cpu().numpy()
    else:
        rows = sample_rows(S, w.attn.n_q_heads, n_sample)
        want = oracle.attention(**sub, rows=rows, n_threads=threads)
        idx = torch.from_numpy(q_off_all[reqs[rows[0]]].astype(np.int64) + rows[2]).to(res["out"].device)
        got = res["out"][idx, torch.from_numpy(rows[1].astype(np.int64)).to(idx.device)].double().cpu().numpy()
    err = np.abs(got - want)
    ref = np.abs(want).max()
    print(f"   {len(reqs)} requests checked, max-abs err {err.max():.3e}  (|ref| max {ref:.3e}, rel {err.max() / ref:.3e})",
          flush=True)
    assert err.max() <= TOL[w.attn.dtype], (label, err.max())
    return err.max(), ref


def test_pipeline_config1_fp32_full():
    check_pipeline(inputs.config1(), "c1")
    check_pipeline(inputs.config1(hard=True), "c1_hard")


def test_pipeline_config2_bf16_sampled():
    check_pipeline(inputs.config2(), "c2", n_sample=4096)
    err, ref = check_pipeline(inputs.config2(hard=True), "c2_hard", n_sample=4096)
    assert err / ref < 2e-2  # N(0,1) inputs: the relative error has to be small too


def test_pipeline_config3_streaming_mix():
    check_pipeline(inputs.config3(), "c3", n_sample=4096, n_sub_req=24)
    check_pipeline(inputs.config3(hard=True), "c3_hard", n_sample=2048, n_sub_req=12)


def test_pipeline_config4_long_context():
    check_pipeline(inputs.config4(), "c4", n_sample=4096, n_sub_req=4)
    check_pipeline(inputs.config4(hard=True), "c4_hard", n_sample=4096, n_sub_req=2)


def test_pipeline_config5_sweep_quarter_sensitive():
    check_pipeline(inputs.config5(0.25), "c5@0.25", n_sample=4096, n_sub_req=24)


def test_pipeline_config5_sweep_no_sensitive_blocks():
    # the one setting of the sweep with long reused prefixes (88.7 % of the prompt tokens)
    check_pipeline(inputs.config5(0.0), "c5@0", n_sample=4096, n_sub_req=8)


@pytest.mark.parametrize("p", [0.5, 1.0])
def test_pipeline_config5_sweep_half_and_all_sensitive(p):
    check_pipeline(inputs.config5(p), f"c5@{p}", n_sample=4096, n_sub_req=4)


# ---- attention alone, on shapes the configs do not reach ---------------------------------------
def attn_case(seed, R, Hq, Hkv, d, dtype, max_blocks, S_list, k_list, n_pages=64, sigma=1.0):
    g = np.random.default_rng(seed)
    S = np.asarray(S_list)
    k_blocks = np.asarray(k_list)
    perm = g.permutation(n_pages)
    pt = np.full((R, max_blocks), -1, np.int32)
    used = 0
    for r in range(R):
        pt[r, : k_blocks[r]] = perm[used: used + k_blocks[r]]
        used += k_blocks[r]
    q_off = np.concatenate([[0], np.cumsum(S)]).astype(np.int32)
    T = int(q_off[-1])
    t = lambda *s: torch.from_numpy(g.standard_normal(s).astype(np.float32) * sigma).to(dtype)
    return dict(q=t(T, Hq, d), knew=t(T, Hkv, d), vnew=t(T, Hkv, d), q_off=q_off,
                kpool=t(n_pages, B, Hkv, d), vpool=t(n_pages, B, Hkv, d),
                matched_len=(k_blocks * B).astype(np.int32), page_table=pt)


def run_attn(c, scale=None):
    skv = _skv()
    dev = "cuda:0"
    q = c["q"].to(dev)
    Hq, d = q.shape[1], q.shape[2]
    Hkv = c["kpool"].shape[2]
    desc = skv.attn_desc(Hq, Hkv, d, q.dtype, scale)
    R = len(c["matched_len"])
    ws = torch.zeros(skv.skv_prefill_attn_workspace_size(desc, R, q.shape[0]), dtype=torch.uint8, device=dev)
    out = torch.full_like(q, 7.0)
    pt = torch.from_numpy(c["page_table"]).to(dev)
    skv.skv_prefill_attn(desc, q, c["knew"].to(dev), c["vnew"].to(dev), torch.from_numpy(c["q_off"]).to(dev),
                         c["kpool"].to(dev), c["vpool"].to(dev), torch.from_numpy(c["matched_len"]).to(dev),
                         pt, pt.shape[1], out, ws)
    torch.cuda.synchronize()
    return out.double().cpu().numpy()


ATTN_SHAPES = [
    # Hq, Hkv, d, dtype, S per request, matched blocks per request
    (8, 2, 128, torch.bfloat16, [1, 63, 64, 65, 0, 200], [0, 1, 3, 4, 5, 9]),     # G=4, ragged tails, S=0
    (8, 1, 128, torch.bfloat16, [130, 17], [7, 0]),                               # G=8: two head groups
    (4, 2, 128, torch.bfloat16, [300, 5, 129], [2, 11, 0]),                       # G=2: 2 heads x 2 position tiles
    (3, 3, 128, torch.bfloat16, [257, 1, 64], [0, 5, 8]),                         # G=1: 4 position tiles
    (16, 8, 128, torch.bfloat16, [70, 33], [3, 6]),                               # Hkv=8: per-XCD head placement
    (16, 1, 128, torch.bfloat16, [70, 33, 129], [3, 6, 0]),                       # G=16: four head groups
    (3, 1, 128, torch.bfloat16, [300, 33], [1, 6]),                               # G=3: one head, 8 position tiles of 32
    (12, 2, 128, torch.bfloat16, [140, 20], [5, 2]),                              # G=6: 2 heads x 4 position tiles, 3 groups
    (4, 2, 64, torch.float32, [1, 50, 0, 70], [0, 2, 3, 6]),
    (2, 1, 128, torch.float32, [40, 9], [1, 4]),
]


@pytest.mark.parametrize("case", range(len(ATTN_SHAPES)))
def test_attention_shapes_and_ragged_edges(case):
    Hq, Hkv, d, dtype, S, k = ATTN_SHAPES[case]
    c = attn_case(100 + case, len(S), Hq, Hkv, d, dtype, max(k) + 1, S, k, sigma=1.0)
    print(f"[attn] case {case}: Hq={Hq} Hkv={Hkv} d={d} {dtype} S={S} k={k}", flush=True)
    got = run_attn(c)
    want = oracle.attention(**c, n_threads=8)
    n = want.shape[0]
    err = np.abs(got[:n] - want).max()
    print(f"   max-abs err {err:.3e}", flush=True)
    assert err <= (1e-4 if dtype == torch.float32 else 2e-2)


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_matched_length_inside_a_block_counts_whole_blocks_only(dtype):
    """A matched length that is not a multiple of 16 is rounded down to whole blocks by the gather and by both
    attention kernels alike (Section 4.3.1: reuse is block granular): same result as with the rounded lengths."""
    skv = _skv()
    d = 128 if dtype == torch.bfloat16 else 64
    S, k = [70, 33, 5], [3, 6, 1]
    c = attn_case(41, len(S), 4, 2, d, dtype, max(k) + 1, S, k, sigma=1.0)
    want = oracle.attention(**c, n_threads=8)
    floor_len = c["matched_len"].copy()
    c["matched_len"] = (floor_len + np.asarray([5, 15, 0], np.int32)).astype(np.int32)
    got = run_attn(c)
    err = np.abs(got[: want.shape[0]] - want).max()
    print(f"   {dtype}: max-abs err {err:.3e}", flush=True)
    assert err <= (1e-4 if dtype == torch.float32 else 2e-2)
    dev = "cuda:0"
    kp, vp = c["kpool"].to(dev), c["vpool"].to(dev)
    ml, pt = torch.from_numpy(c["matched_len"]).to(dev), torch.from_numpy(c["page_table"]).to(dev)
    total = int(floor_len.sum())
    desc = skv.attn_desc(4, 2, d, dtype)
    kctx = torch.full((total + 16,) + tuple(kp.shape[2:]), 7.0, dtype=dtype, device=dev)
    vctx = torch.full_like(kctx, 7.0)
    off = torch.zeros(len(S) + 1, dtype=torch.int64, device=dev)
    skv.skv_gather_kv(desc, kp, vp, ml, pt, pt.shape[1], off, kctx, vctx)
    torch.cuda.synchronize()
    assert off.cpu().numpy().tolist() == np.concatenate([[0], np.cumsum(floor_len)]).tolist()
    wk, wv = oracle.gather(c["kpool"], c["vpool"], floor_len, c["page_table"])
    as_bytes = lambda t: t.contiguous().cpu().view(torch.uint8)
    assert torch.equal(as_bytes(kctx[:total]), as_bytes(wk)) and torch.equal(as_bytes(vctx[:total]), as_bytes(wv))
    assert float(kctx[total:].float().min()) == 7.0 and float(kctx[total:].float().max()) == 7.0   # nothing past the end


def test_attention_reference_moves_under_large_scores():
    """Scores with a spread of hundreds of log2 units (entries ~ N(0, 16)) over contexts long enough for the
    pipelined loop (49 and 30 key tiles): the softmax reference has to move again and again, in the steady-state
    loop as well as in the first and last iterations, and the result must still be the oracle's; then a ramp
    (every key scores higher than all keys before it) that trips the reference in every sub-tile."""
    c = attn_case(11, 2, 8, 2, 128, torch.bfloat16, 200, [150, 64], [190, 116], n_pages=320, sigma=4.0)
    got = run_attn(c)
    want = oracle.attention(c["q"], c["knew"], c["vnew"], c["q_off"], c["kpool"], c["vpool"], c["matched_len"],
                            c["page_table"], n_threads=16)
    err = np.abs(got - want)
    print(f"   large scores: max-abs err {err.max():.3e} (|ref| max {np.abs(want).max():.3e})", flush=True)
    assert np.isfinite(got).all() and err.max() <= 2e-2 * max(1.0, np.abs(want).max())
    # ramp: K row j = (j / 4) * u, Q rows = u (unit-ish vector): score of key j grows by ~16 log2 units per 4 keys
    g = np.random.default_rng(3)
    u = g.standard_normal(128).astype(np.float32)
    u *= 8.0 / np.linalg.norm(u)
    c = attn_case(12, 1, 8, 2, 128, torch.bfloat16, 64, [128], [56], n_pages=64, sigma=1.0)
    c["q"][:] = torch.from_numpy(u).to(torch.bfloat16)
    L = int(c["matched_len"][0])
    for j in range(L):
        c["kpool"][c["page_table"][0, j // B], j % B] = torch.from_numpy(u * (j // 4)).to(torch.bfloat16)
    for i in range(128):
        c["knew"][i] = torch.from_numpy(u * ((L + i) // 4)).to(torch.bfloat16)
    got = run_attn(c)
    want = oracle.attention(c["q"], c["knew"], c["vnew"], c["q_off"], c["kpool"], c["vpool"], c["matched_len"],
                            c["page_table"], n_threads=16)
    err = np.abs(got - want)
    print(f"   ramp: max-abs err {err.max():.3e} (|ref| max {np.abs(want).max():.3e})", flush=True)
    assert np.isfinite(got).all() and err.max() <= 2e-2 * max(1.0, np.abs(want).max())


def test_attention_closed_forms_on_gpu():
    """The oracle's closed-form pins, applied to the GPU path directly: V == 1 gives 1; K == 0 with
    V = position gives (L+i)/2 (bf16 holds integers up to 256 exactly)."""
    S, k = [100, 37], [4, 0]
    c = attn_case(5, 2, 8, 2, 128, torch.bfloat16, 5, S, k)
    c["vpool"].fill_(1.0); c["vnew"].fill_(1.0)
    assert np.abs(run_attn(c) - 1.0).max() <= 1e-2
    c["kpool"].zero_(); c["knew"].zero_()
    for r in range(2):
        L = int(c["matched_len"][r])
        for j in range(L):
            c["vpool"][c["page_table"][r, j // B], j % B] = float(j)
        for i in range(S[r]):
            c["vnew"][c["q_off"][r] + i] = float(L + i)
    got = run_attn(c)
    for r in range(2):
        L = int(c["matched_len"][r])
        for i in range(S[r]):
            assert np.abs(got[c["q_off"][r] + i] - (L + i) / 2.0).max() <= 0.5 + 1e-6, (r, i)


def test_error_codes_need_no_launch():
    skv = _skv()
    desc = skv.attn_desc(8, 3, 128, torch.bfloat16)
    with pytest.raises(skv.SkvError):
        skv.skv_prefill_attn_workspace_size(desc, 1, 1)


# ---- safeguard step: window roll + RDR predicate + demotion, several windows in a row ----------------
POLICIES = [dict(direction=0, tau=(1, 2), min_hits=1, n_consec=1, u_pre_max=1),
            dict(direction=0, tau=(2, 3), min_hits=3, n_consec=2, u_pre_max=1),
            dict(direction=1, tau=(1, 3), min_hits=1, n_consec=1, u_pre_max=2)]


def run_windows(w, label, policy, n_windows=4, seed=0):
    skv = _skv()
    print(f"[safeguard] {label} {policy}", flush=True)
    s = _session(w, with_kv=False)
    tree = oracle.OracleTree.from_workload(w)
    pol = skv.rdr_policy(**policy)
    n_dem = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    n = w.n_in_blocks
    priv = torch.zeros(max(n, 1), dtype=torch.uint8, device="cuda:0")
    hp = torch.zeros(max(n, 1), dtype=torch.int32, device="cuda:0")
    up = torch.zeros(max(n, 1), dtype=torch.int32, device="cuda:0")
    g = np.random.default_rng(seed)
    total = 0
    for win in range(n_windows):
        tenants = g.integers(0, w.n_tenants, w.n_req).astype(np.int32)   # a new tenant mix every window
        s.req_tenant.copy_(torch.from_numpy(tenants))
        skv.skv_match(s.tree, s.req_off, s.req_tokens, s.req_tenant, s.max_blocks, s.matched_len, s.page_table)
        mlen, pt = tree.match(w.req_off, w.req_tokens, tenants, s.max_blocks)
        torch.cuda.synchronize()
        assert np.array_equal(s.matched_len.cpu().numpy(), mlen), (label, win)   # demotions change visibility
        assert np.array_equal(s.page_table.cpu().numpy(), pt), (label, win)
        skv.skv_window_roll(s.tree, pol, n_dem)
        want = tree.window_roll(**policy)
        skv.skv_block_state_read(s.tree, priv, hp, up)
        torch.cuda.synchronize()
        o_priv, o_hp, o_up = tree.block_state()
        assert int(n_dem.item()) == want, (label, win)
        assert np.array_equal(priv[:n].cpu().numpy(), o_priv)
        assert np.array_equal(hp[:n].cpu().numpy().view(np.uint32), o_hp)
        assert np.array_equal(up[:n].cpu().numpy().view(np.uint32), o_up)
        h, u = s.counters()
        assert h.sum() == 0 and u.sum() == 0
        total += want
    return total


def test_safeguard_small_cases_all_policies():
    total = 0
    for seed in range(40):
        w = inputs.small_random(seed=seed, n_req=60, p_sens=0.3, n_tenants=3)
        total += run_windows(w, f"small{seed}", POLICIES[seed % 3], seed=seed)
    assert total > 50


def test_safeguard_config3_and_config5():
    assert run_windows(inputs.config3(), "c3", dict(direction=0, tau=(9, 10), min_hits=2, n_consec=1, u_pre_max=1),
                       n_windows=3) > 0
    run_windows(inputs.config5(0.25), "c5@0.25", POLICIES[1], n_windows=3)
    run_windows(inputs.config2(), "c2", POLICIES[2], n_windows=3)


# ---------------------------------------------------------------------------------------------
# insert side: promotion (Section 4.2.3) and the write of new KV blocks into pool pages (Section 4.3.1)

def check_promote(w, label, seed, frac=0.4):
    skv = _skv()
    print(f"[promote] {label}", flush=True)
    s = _session(w, with_kv=False)
    tree = oracle.OracleTree.from_workload(w)
    g = np.random.default_rng(seed)
    n = w.n_in_blocks
    ids = np.flatnonzero(g.random(n) < frac).astype(np.int32)
    ids_dev = np.concatenate([ids, [-1, n, n + 12345], ids[:3]]).astype(np.int32)   # invalid ids and repeats are ignored
    skv.skv_promote(s.tree, torch.from_numpy(ids_dev).to("cuda:0"))
    tree.promote(ids)
    priv = torch.zeros(max(n, 1), dtype=torch.uint8, device="cuda:0")
    hp = torch.zeros(max(n, 1), dtype=torch.int32, device="cuda:0")
    up = torch.zeros(max(n, 1), dtype=torch.int32, device="cuda:0")
    skv.skv_block_state_read(s.tree, priv, hp, up)
    torch.cuda.synchronize()
    assert np.array_equal(priv[:n].cpu().numpy(), tree.block_state()[0]), label
    skv.skv_match(s.tree, s.req_off, s.req_tokens, s.req_tenant, s.max_blocks, s.matched_len, s.page_table)
    mlen, pt = tree.match(w.req_off, w.req_tokens, w.req_tenant, s.max_blocks)
    torch.cuda.synchronize()
    assert np.array_equal(s.matched_len.cpu().numpy(), mlen), label
    assert np.array_equal(s.page_table.cpu().numpy(), pt), label
    hit, ucnt = s.counters()
    o_hit, o_ucnt = tree.counters()
    assert np.array_equal(hit, o_hit) and np.array_equal(ucnt, o_ucnt), label
    return mlen


def test_promote_small_cases_and_config5():
    for seed in range(30):
        check_promote(inputs.small_random(seed=seed, n_req=40, p_sens=0.6, n_tenants=4), f"small{seed}", seed)
    w = inputs.config5(p_sensitive=0.75)
    base, _ = oracle.OracleTree.from_workload(w).match(w.req_off, w.req_tokens, w.req_tenant, max(w.max_blocks, 1),
                                                       update=False)
    after = check_promote(w, "c5@0.75", 1, frac=0.5)
    assert after.sum() > base.sum()                       # promotion does open up reuse at full size
    skv = _skv()
    s = _session(inputs.small_random(seed=1), with_kv=False)
    skv.skv_promote(s.tree, torch.zeros(0, dtype=torch.int32, device="cuda:0"))   # empty list: no launch
    torch.cuda.synchronize()


def scatter_inputs(seed, R, H, d, dtype, max_s=200, p_alloc=0.85):
    g = np.random.default_rng(seed)
    S = g.integers(0, max_s, R)
    S[:3] = [0, 15, 32]
    q_off = np.concatenate([[0], np.cumsum(S)]).astype(np.int32)
    T = int(q_off[-1])
    knew = torch.from_numpy(g.standard_normal((T, H, d))).to(dtype)
    vnew = torch.from_numpy(g.standard_normal((T, H, d))).to(dtype)
    mb = int(max(S) // B) + 1
    n_pages = R * mb + 5
    perm = g.permutation(n_pages)
    new_pages = np.full((R, mb), -1, np.int32)
    alloc = g.random((R, mb)) < p_alloc
    new_pages[alloc] = perm[: int(alloc.sum())]
    kpool = torch.from_numpy(g.standard_normal((n_pages, B, H, d))).to(dtype)
    vpool = torch.from_numpy(g.standard_normal((n_pages, B, H, d))).to(dtype)
    return q_off, knew, vnew, new_pages, kpool, vpool


def run_scatter(label, H, d, dtype, q_off, knew, vnew, new_pages, kpool, vpool):
    skv = _skv()
    print(f"[scatter] {label}", flush=True)
    dev = "cuda:0"
    desc = skv.attn_desc(H, H, d, "f32" if dtype == torch.float32 else "bf16", 1.0)
    kp, vp = kpool.to(dev), vpool.to(dev)
    skv.skv_scatter_kv(desc, knew.to(dev), vnew.to(dev), torch.from_numpy(q_off).to(dev),
                       torch.from_numpy(new_pages).to(dev), kp, vp)
    torch.cuda.synchronize()
    oracle.scatter(knew, vnew, q_off, new_pages, kpool, vpool)          # in place on the host copies
    assert torch.equal(kp.cpu().view(torch.uint8), kpool.view(torch.uint8)), label
    assert torch.equal(vp.cpu().view(torch.uint8), vpool.view(torch.uint8)), label


def test_scatter_small_ragged_cases():
    for seed, (H, d, dtype) in enumerate([(2, 8, torch.float32), (8, 128, torch.bfloat16), (1, 64, torch.bfloat16),
                                          (3, 40, torch.float32), (8, 64, torch.float32)]):
        run_scatter(f"small{seed}", H, d, dtype, *scatter_inputs(seed, 9, H, d, dtype))
    # out-of-range page ids are skipped like negative ones; an empty batch and a zero-column table launch nothing
    q_off, knew, vnew, new_pages, kpool, vpool = scatter_inputs(7, 6, 2, 16, torch.float32)
    bad = new_pages.copy()
    sel = np.flatnonzero(new_pages.ravel() >= 0)[::3]
    bad.ravel()[sel] = kpool.shape[0] + 3
    ref = new_pages.copy()
    ref.ravel()[sel] = -1
    skv = _skv()
    desc = skv.attn_desc(2, 2, 16, "f32", 1.0)
    kp, vp = kpool.cuda(), vpool.cuda()
    skv.skv_scatter_kv(desc, knew.cuda(), vnew.cuda(), torch.from_numpy(q_off).cuda(), torch.from_numpy(bad).cuda(), kp, vp)
    torch.cuda.synchronize()
    oracle.scatter(knew, vnew, q_off, ref, kpool, vpool)
    assert torch.equal(kp.cpu(), kpool) and torch.equal(vp.cpu(), vpool)
    skv.skv_scatter_kv(desc, knew.cuda(), vnew.cuda(), torch.zeros(1, dtype=torch.int32, device="cuda:0"),
                       torch.zeros((0, 4), dtype=torch.int32, device="cuda:0"), kp, vp)
    torch.cuda.synchronize()


def test_scatter_then_gather_round_trip_config2():
    """Full-size insert: every full block of config 2's uncached suffixes goes to a fresh page; the pages,
    gathered back through the same table, are the suffix rows again, and match the oracle's pools."""
    skv = _skv()
    w = inputs.config2()
    s = _session(w)
    s.prepare()
    s.match()
    torch.cuda.synchronize()
    q_off = s.q_off.cpu().numpy()
    R = w.n_req
    full = np.diff(q_off) // B
    mb = int(full.max()) + 1
    n_new = int(full.sum())
    g = np.random.default_rng(0)
    perm = g.permutation(n_new + 7).astype(np.int32)
    new_pages = np.full((R, mb), -1, np.int32)
    mask = np.arange(mb)[None, :] < full[:, None]
    new_pages[mask] = perm[:n_new]
    a = w.attn
    shape = (n_new + 7, B, a.n_kv_heads, a.head_dim)
    kp = torch.zeros(shape, dtype=a.torch_dtype, device="cuda:0")
    vp = torch.zeros(shape, dtype=a.torch_dtype, device="cuda:0")
    np_dev = torch.from_numpy(new_pages).cuda()
    print(f"[scatter] c2 {n_new} pages", flush=True)
    skv.skv_scatter_kv(s.desc, s.knew, s.vnew, s.q_off, np_dev, kp, vp)
    torch.cuda.synchronize()
    knew, vnew = s.knew.cpu(), s.vnew.cpu()                 # rows from the seeded generator
    kpool, vpool = torch.zeros(shape, dtype=a.torch_dtype), torch.zeros(shape, dtype=a.torch_dtype)
    oracle.scatter(knew, vnew, q_off, new_pages, kpool, vpool)
    assert torch.equal(kp.cpu().view(torch.int16), kpool.view(torch.int16))
    assert torch.equal(vp.cpu().view(torch.int16), vpool.view(torch.int16))
    # round trip through the gather
    full_len = torch.from_numpy((full * B).astype(np.int32)).cuda()
    kctx = torch.zeros((n_new * B, a.n_kv_heads, a.head_dim), dtype=a.torch_dtype, device="cuda:0")
    vctx = torch.zeros_like(kctx)
    ctx_off = torch.zeros(R + 1, dtype=torch.int64, device="cuda:0")
    skv.skv_gather_kv(s.desc, kp, vp, full_len, np_dev, mb, ctx_off, kctx, vctx)
    torch.cuda.synchronize()
    co = ctx_off.cpu().numpy()
    for r in range(R):
        n = int(full[r]) * B
        assert torch.equal(kctx[co[r]: co[r] + n], s.knew[q_off[r]: q_off[r] + n])
        assert torch.equal(vctx[co[r]: co[r] + n], s.vnew[q_off[r]: q_off[r] + n])


# ---------------------------------------------------------------------------------------------
# insert after prefill (Section 4.3.1 Insert): a stream of match -> insert rounds on the device tree and on
# the oracle tree, which must stay interchangeable

def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def device_match(skv, tree, off, toks, tenants, mb, want_path_end=False):
    R = len(tenants)
    mlen = torch.zeros(max(R, 1), dtype=torch.int32, device="cuda:0")
    pt = torch.full((max(R, 1), mb), -1, dtype=torch.int32, device="cuda:0")
    pe = torch.full((max(R, 1),), -7, dtype=torch.int32, device="cuda:0") if want_path_end else None
    skv.skv_match(tree, _dev(off), _dev(toks) if len(toks) else torch.zeros(1, dtype=torch.int32, device="cuda:0"),
                  _dev(tenants), mb, mlen, pt, path_end=pe)
    torch.cuda.synchronize()
    if want_path_end:
        return mlen[:R].cpu().numpy(), pt[:R].cpu().numpy(), pe[:R].cpu().numpy()
    return mlen[:R].cpu().numpy(), pt[:R].cpu().numpy()


def compare_state(skv, dtree, otree, label):
    n = otree.n_in_blocks
    info = dtree.info()
    # (node counts are not compared: how a chain is cut into nodes is not unique, only what lookups return is)
    assert info["n_in_blocks"] == n and info["n_blocks"] == otree.n_blocks, label
    hit = torch.zeros(max(n, 1), dtype=torch.int32, device="cuda:0")
    ucnt = torch.zeros_like(hit)
    priv = torch.zeros(max(n, 1), dtype=torch.uint8, device="cuda:0")
    skv.skv_counters_read(dtree, hit, ucnt)
    skv.skv_block_state_read(dtree, priv, torch.zeros_like(hit), torch.zeros_like(hit))
    torch.cuda.synchronize()
    o_hit, o_ucnt = otree.counters()
    assert np.array_equal(hit[:n].cpu().numpy().view(np.uint32), o_hit), label
    assert np.array_equal(ucnt[:n].cpu().numpy().view(np.uint32), o_ucnt), label
    assert np.array_equal(priv[:n].cpu().numpy(), otree.block_state()[0]), label


def run_insert_stream(seed, n_rounds=4, n_req=12):
    from test_oracle_insert import make_round
    skv = _skv()
    block_vocab = 3 if seed % 3 == 0 else None
    w = inputs.small_random(seed=seed, n_req=8, p_sens=0.4, n_tenants=3, block_vocab=block_vocab)
    vocab = int(w.seq_tokens.max()) + 1 if len(w.seq_tokens) else 2
    n_pages = w.n_pages + 4096
    otree = oracle.OracleTree.from_workload(w)
    dtree = skv.skv_tree_build(w.seq_tokens, w.seq_off, w.blk_sensitive, w.blk_owner, w.blk_page, w.n_tenants,
                               n_pages, device="cuda:0", reserve_blocks=1024)
    g = np.random.default_rng(1000 + seed)
    next_page = w.n_pages
    earlier = [w.req_tokens[w.req_off[r]: w.req_off[r + 1]] for r in range(w.n_req)]
    inserted = 0
    for rnd in range(n_rounds):
        reqs, off, toks, tenants = make_round(g, earlier, vocab, w.n_tenants, n_req, block_vocab)
        mb = max(max(len(x) // B for x in reqs), 1)
        mlen, pt = device_match(skv, dtree, off, toks, tenants, mb)
        o_mlen, o_pt = otree.match(off, toks, tenants, mb)
        assert np.array_equal(mlen, o_mlen) and np.array_equal(pt, o_pt), (seed, rnd)
        new_pages = np.full((n_req, mb + 1), -1, np.int32)
        for r, x in enumerate(reqs):
            n_suffix = len(x) // B - mlen[r] // B
            if g.random() < 0.15:
                n_suffix = int(g.integers(0, n_suffix + 1))
            new_pages[r, :n_suffix] = np.arange(next_page, next_page + n_suffix)
            next_page += n_suffix
        first, n = skv.skv_tree_insert(dtree, off, toks, tenants, mlen, new_pages)
        o_first, o_n = otree.insert(off, toks, tenants, mlen, new_pages)
        assert np.array_equal(first, o_first) and np.array_equal(n, o_n), (seed, rnd)
        inserted += int(n.sum())
        if rnd == 1 and n.sum() > 0:    # the verifier clears some of the new blocks
            ids = np.arange(otree.n_in_blocks - int(n.sum()), otree.n_in_blocks)[::2].astype(np.int32)
            skv.skv_promote(dtree, _dev(ids))
            otree.promote(ids)
        earlier += reqs
        # everything seen so far, as every tenant: lengths, page ids, then counters and visibility bits
        for t in range(w.n_tenants):
            sample = [earlier[i] for i in g.choice(len(earlier), min(24, len(earlier)), replace=False)]
            o = np.concatenate([[0], np.cumsum([len(x) for x in sample])]).astype(np.int32)
            tk = np.concatenate(sample + [np.zeros(0, np.int32)]).astype(np.int32)
            ten = np.full(len(sample), t, np.int32)
            mb2 = max(max(len(x) // B for x in sample), 1)
            ml2, pt2 = device_match(skv, dtree, o, tk, ten, mb2)
            o_ml2, o_pt2 = otree.match(o, tk, ten, mb2)
            assert np.array_equal(ml2, o_ml2) and np.array_equal(pt2, o_pt2), (seed, rnd, t)
        compare_state(skv, dtree, otree, (seed, rnd))
    return inserted


def test_insert_stream_small_cases():
    total = 0
    for seed in range(30):
        print(f"[insert] stream {seed}", flush=True)
        total += run_insert_stream(seed)
    assert total > 500


def test_insert_errors_leave_the_tree_unchanged():
    skv = _skv()
    w = inputs.small_random(seed=2, n_req=8, p_sens=0.3, n_tenants=3)
    otree = oracle.OracleTree.from_workload(w)
    dtree = skv.skv_tree_build(w.seq_tokens, w.seq_off, w.blk_sensitive, w.blk_owner, w.blk_page, w.n_tenants,
                               w.n_pages + 64, device="cuda:0")          # no room reserved
    g = np.random.default_rng(0)
    x = g.integers(0, 1000, 40 * B).astype(np.int32)
    off = np.array([0, len(x)], np.int32)
    ten = np.array([1], np.int32)
    pages = (w.n_pages + np.arange(40, dtype=np.int32))[None, :]
    with pytest.raises(skv.SkvError) as e:
        skv.skv_tree_insert(dtree, off, x, ten, np.zeros(1, np.int32), pages)
    assert e.value.code == skv.SKV_ENOMEM
    used = int(w.blk_page[0])
    for bad_pages, bad_ten in ((np.array([[used]], np.int32), ten), (np.array([[w.n_pages + 64]], np.int32), ten),
                               (np.array([[w.n_pages, w.n_pages]], np.int32), ten),
                               (np.array([[w.n_pages]], np.int32), np.array([w.n_tenants], np.int32))):
        with pytest.raises(skv.SkvError) as e:
            skv.skv_tree_insert(dtree, off, x, bad_ten, np.zeros(1, np.int32), bad_pages)
        assert e.value.code == skv.SKV_EINVAL
    # path ends that do not belong to the request: a record although nothing matched, no record although something
    # did, a record number outside the index, and the record of some other block
    mb = max(w.max_blocks, 1)
    r_hit = int(np.argmax(np.diff(w.req_off) // B > 0))
    one_off = np.array([0, w.req_off[r_hit + 1] - w.req_off[r_hit]], np.int32)
    one_tok = w.req_tokens[w.req_off[r_hit]: w.req_off[r_hit + 1]]
    one_ten = w.req_tenant[r_hit: r_hit + 1]
    ml1, _, pe1 = device_match(skv, dtree, one_off, one_tok, one_ten, mb, want_path_end=True)
    otree.match(one_off, one_tok, one_ten, mb)
    if ml1[0] >= B:
        n_rec = dtree.info()["n_blocks"]
        wrong = [np.array([-1], np.int32), np.array([n_rec + 3], np.int32)]
        other = [f for f in range(n_rec) if f != pe1[0]]
        if other:
            wrong.append(np.array([other[-1]], np.int32))
        for bad_pe in wrong:
            with pytest.raises(skv.SkvError) as e:
                skv.skv_tree_insert(dtree, one_off, one_tok, one_ten, ml1, np.array([[w.n_pages]], np.int32),
                                    private_copies=True, path_end=bad_pe)
            assert e.value.code == skv.SKV_EINVAL
    with pytest.raises(skv.SkvError) as e:
        skv.skv_tree_insert(dtree, off, x, ten, np.zeros(1, np.int32), np.array([[w.n_pages]], np.int32),
                            private_copies=True, path_end=np.array([0], np.int32))
    assert e.value.code == skv.SKV_EINVAL
    mlen, pt = device_match(skv, dtree, w.req_off, w.req_tokens, w.req_tenant, mb)
    o_mlen, o_pt = otree.match(w.req_off, w.req_tokens, w.req_tenant, mb)
    assert np.array_equal(mlen, o_mlen) and np.array_equal(pt, o_pt)
    compare_state(skv, dtree, otree, "after errors")


@pytest.mark.parametrize("name", ["c2", "c3"])
def test_insert_configs_full_size(name):
    """Full size: every request of config 2 inserts its uncached suffix; asked again, requests reuse what
    their own tenant inserted, and the oracle tree agrees block for block for the same and for other tenants."""
    import time
    skv = _skv()
    w = inputs.CONFIGS[name]()
    otree = oracle.OracleTree.from_workload(w)
    nb_req = int((np.diff(w.req_off) // B).sum())
    dtree = skv.skv_tree_build(w.seq_tokens, w.seq_off, w.blk_sensitive, w.blk_owner, w.blk_page, w.n_tenants,
                               w.n_pages + nb_req, device="cuda:0", reserve_blocks=nb_req)
    mb = max(w.max_blocks, 1)
    mlen, pt = device_match(skv, dtree, w.req_off, w.req_tokens, w.req_tenant, mb)
    o_mlen, o_pt = otree.match(w.req_off, w.req_tokens, w.req_tenant, mb)
    assert np.array_equal(mlen, o_mlen) and np.array_equal(pt, o_pt)
    full = np.diff(w.req_off) // B - mlen // B
    new_pages = np.full((w.n_req, int(full.max())), -1, np.int32)
    new_pages[np.arange(new_pages.shape[1])[None, :] < full[:, None]] = w.n_pages + np.arange(int(full.sum()), dtype=np.int32)
    t0 = time.perf_counter()
    first, n = skv.skv_tree_insert(dtree, w.req_off, w.req_tokens, w.req_tenant, mlen, new_pages)
    dt = time.perf_counter() - t0
    print(f"[insert] {name}: {int(n.sum())} of {int(full.sum())} suffix blocks new, {dt * 1e3:.2f} ms "
          f"({w.n_req / dt:.0f} requests/s)", flush=True)
    o_first, o_n = otree.insert(w.req_off, w.req_tokens, w.req_tenant, mlen, new_pages)
    assert np.array_equal(first, o_first) and np.array_equal(n, o_n)
    assert n.sum() > 0           # requests of one group share their prompt: only the first of them inserts it
    for shift in (0, 1):
        ten = ((w.req_tenant + shift) % w.n_tenants).astype(np.int32)
        ml2, pt2 = device_match(skv, dtree, w.req_off, w.req_tokens, ten, mb)
        o_ml2, o_pt2 = otree.match(w.req_off, w.req_tokens, ten, mb)
        assert np.array_equal(ml2, o_ml2) and np.array_equal(pt2, o_pt2)
        if shift == 0:
            assert np.all(ml2 >= mlen)   # (many requests stop at other tenants' private blocks, before and after)
            print(f"   reuse before {int(mlen.sum())} tokens, after {int(ml2.sum())}", flush=True)
    compare_state(skv, dtree, otree, name)


# ---------------------------------------------------------------------------------------------
# eviction (Section 4.3.1 Evict, Section 4.3.2 progressive eviction): epochs stamped by the match kernel,
# then the same victims in the same order as the oracle, and identical lookups afterwards

def device_epochs(skv, dtree):
    n = dtree.info()["n_in_blocks"]
    e = torch.zeros(max(n, 1), dtype=torch.int32, device="cuda:0")
    skv.skv_block_epochs_read(dtree, e)
    torch.cuda.synchronize()
    return e[:n].cpu().numpy().view(np.uint32)


def run_evict_stream(seed, n_rounds=5, n_req=10):
    from test_oracle_insert import make_round
    skv = _skv()
    block_vocab = 3 if seed % 3 == 0 else None
    w = inputs.small_random(seed=seed, n_req=8, p_sens=0.4, n_tenants=3, block_vocab=block_vocab)
    vocab = int(w.seq_tokens.max()) + 1 if len(w.seq_tokens) else 2
    otree = oracle.OracleTree.from_workload(w)
    dtree = skv.skv_tree_build(w.seq_tokens, w.seq_off, w.blk_sensitive, w.blk_owner, w.blk_page, w.n_tenants,
                               w.n_pages + 4096, device="cuda:0", reserve_blocks=1024)
    g = np.random.default_rng(2000 + seed)
    free_pages = list(range(w.n_pages, w.n_pages + 4096))[::-1]
    earlier = [w.req_tokens[w.req_off[r]: w.req_off[r + 1]] for r in range(w.n_req)]
    evicted = 0
    for rnd in range(n_rounds):
        otree.set_epoch(rnd + 1)
        skv.skv_set_epoch(dtree, rnd + 1)
        reqs, off, toks, tenants = make_round(g, earlier, vocab, w.n_tenants, n_req, block_vocab)
        mb = max(max(len(x) // B for x in reqs), 1)
        mlen, pt = device_match(skv, dtree, off, toks, tenants, mb)
        o_mlen, o_pt, o_ids = otree.match(off, toks, tenants, mb, want_ids=True)
        assert np.array_equal(mlen, o_mlen) and np.array_equal(pt, o_pt), (seed, rnd)
        new_pages = np.full((n_req, mb + 1), -1, np.int32)
        for r, x in enumerate(reqs):
            for j in range(len(x) // B - mlen[r] // B):
                new_pages[r, j] = free_pages.pop()
        first, n = skv.skv_tree_insert(dtree, off, toks, tenants, mlen, new_pages)
        o_first, o_n = otree.insert(off, toks, tenants, mlen, new_pages)
        assert np.array_equal(first, o_first) and np.array_equal(n, o_n), (seed, rnd)
        assert np.array_equal(device_epochs(skv, dtree), otree.epochs()), (seed, rnd)
        protect = o_ids[o_ids >= 0][:: int(g.integers(1, 4))].astype(np.int32)
        n_want = int(g.integers(0, max(otree.n_blocks // 3, 1) + 1))
        ids, pages = skv.skv_evict(dtree, n_want, protect)
        want_ids, want_pages = otree.evict(n_want, protect)
        assert np.array_equal(ids, want_ids) and np.array_equal(pages, want_pages), (seed, rnd)
        evicted += len(ids)
        free_pages += [int(p) for p in pages]              # evicted pages are handed out again
        earlier += reqs
        for t in range(w.n_tenants):
            sample = [earlier[i] for i in g.choice(len(earlier), min(24, len(earlier)), replace=False)]
            o = np.concatenate([[0], np.cumsum([len(x) for x in sample])]).astype(np.int32)
            tk = np.concatenate(sample + [np.zeros(0, np.int32)]).astype(np.int32)
            ten = np.full(len(sample), t, np.int32)
            mb2 = max(max(len(x) // B for x in sample), 1)
            ml2, pt2 = device_match(skv, dtree, o, tk, ten, mb2)
            o_ml2, o_pt2 = otree.match(o, tk, ten, mb2)
            assert np.array_equal(ml2, o_ml2) and np.array_equal(pt2, o_pt2), (seed, rnd, t)
        compare_state(skv, dtree, otree, (seed, rnd))
        assert np.array_equal(device_epochs(skv, dtree), otree.epochs()), (seed, rnd)
    return evicted


def test_evict_stream_small_cases():
    total = 0
    for seed in range(30):
        print(f"[evict] stream {seed}", flush=True)
        total += run_evict_stream(seed)
    assert total > 500


def test_evict_config3_then_reinsert():
    """Full size: half of config 3's requests touch the tree at epoch 1, then 1500 blocks are evicted with the
    touched blocks protected; victims, pages and all later lookups agree with the oracle; the evicted pages are
    then handed to an insert, which must accept them."""
    skv = _skv()
    w = inputs.config3()
    otree = oracle.OracleTree.from_workload(w)
    dtree = skv.skv_tree_build(w.seq_tokens, w.seq_off, w.blk_sensitive, w.blk_owner, w.blk_page, w.n_tenants,
                               w.n_pages, device="cuda:0", reserve_blocks=4096)
    mb = max(w.max_blocks, 1)
    half = w.n_req // 2
    off, ten = w.req_off[: half + 1], w.req_tenant[:half]
    toks = w.req_tokens[: off[-1]]
    otree.set_epoch(1)
    skv.skv_set_epoch(dtree, 1)
    mlen, pt = device_match(skv, dtree, off, toks, ten, mb)
    o_mlen, o_pt, o_ids = otree.match(off, toks, ten, mb, want_ids=True)
    assert np.array_equal(mlen, o_mlen) and np.array_equal(pt, o_pt)
    assert np.array_equal(device_epochs(skv, dtree), otree.epochs())
    protect = np.unique(o_ids[o_ids >= 0]).astype(np.int32)
    print(f"[evict] c3: {otree.n_blocks} blocks, {len(protect)} protected", flush=True)
    ids, pages = skv.skv_evict(dtree, 1500, protect)
    want_ids, want_pages = otree.evict(1500, protect)
    assert len(ids) == 1500 and np.array_equal(ids, want_ids) and np.array_equal(pages, want_pages)
    ml2, pt2 = device_match(skv, dtree, w.req_off, w.req_tokens, w.req_tenant, mb)
    o_ml2, o_pt2 = otree.match(w.req_off, w.req_tokens, w.req_tenant, mb)
    assert np.array_equal(ml2, o_ml2) and np.array_equal(pt2, o_pt2)
    # the second half's suffixes go into the freed pages
    off2 = (w.req_off[half:] - w.req_off[half]).astype(np.int32)
    toks2, ten2 = w.req_tokens[w.req_off[half]:], w.req_tenant[half:]
    ml3 = ml2[half:]
    need = np.minimum(np.diff(off2) // B - ml3 // B, 8)      # up to 8 new blocks per request
    new_pages = np.full((len(ten2), 8), -1, np.int32)
    pool = [int(p) for p in pages]
    for r in range(len(ten2)):
        for j in range(int(need[r])):
            if pool:
                new_pages[r, j] = pool.pop()
    first, n = skv.skv_tree_insert(dtree, off2, toks2, ten2, ml3, new_pages)
    o_first, o_n = otree.insert(off2, toks2, ten2, ml3, new_pages)
    assert np.array_equal(first, o_first) and np.array_equal(n, o_n)
    ml4, pt4 = device_match(skv, dtree, w.req_off, w.req_tokens, w.req_tenant, mb)
    o_ml4, o_pt4 = otree.match(w.req_off, w.req_tokens, w.req_tenant, mb)
    assert np.array_equal(ml4, o_ml4) and np.array_equal(pt4, o_pt4)
    compare_state(skv, dtree, otree, "c3")


# ---------------------------------------------------------------------------------------------
# reclaiming record space (Section 4.3.2 progressive eviction): a tree with little spare room lives through many
# times its capacity in evictions and insertions; when the slab is full it is compacted and the insert repeated.
# The oracle never renumbers, so device block ids are translated through the maps the compactions returned.

def run_compact_stream(seed, n_rounds, copies, reserve=96, n_req=10):
    from test_oracle_insert import make_round
    skv = _skv()
    block_vocab = 3 if seed % 3 == 0 else None
    w = inputs.small_random(seed=seed, n_req=8, p_sens=0.4, n_tenants=3, block_vocab=block_vocab)
    vocab = int(w.seq_tokens.max()) + 1 if len(w.seq_tokens) else 2
    n_pages = w.n_pages + 1024
    otree = oracle.OracleTree.from_workload(w)
    dtree = skv.skv_tree_build(w.seq_tokens, w.seq_off, w.blk_sensitive, w.blk_owner, w.blk_page, w.n_tenants,
                               n_pages, device="cuda:0", reserve_blocks=reserve)
    cap = w.n_in_blocks + reserve              # what the slab was sized for (it may hold a little more)
    keep = max(cap - 64, 8)                    # live blocks after each round's eviction
    g = np.random.default_rng(4000 + seed)
    free_pages = list(range(w.n_pages, n_pages))[::-1]
    earlier = [w.req_tokens[w.req_off[r]: w.req_off[r + 1]] for r in range(w.n_req)]
    d2o = np.arange(w.n_in_blocks, dtype=np.int64)          # device block id -> oracle block id
    tot = dict(inserted=0, evicted=0, compactions=0, forced=0, demoted=0)
    roll_policy = dict(direction=0, tau=(1, 2), min_hits=1, n_consec=1, u_pre_max=1)

    def o2d():
        inv = np.full(otree.n_in_blocks, -1, np.int64)
        inv[d2o] = np.arange(len(d2o))
        return inv

    def compact():
        nonlocal d2o
        id_map = skv.skv_tree_compact(dtree)
        assert len(id_map) == len(d2o)
        live = id_map >= 0
        assert np.array_equal(id_map[live], np.arange(live.sum()))          # dense, old order kept
        d2o = d2o[live]
        info = dtree.info()
        assert info["n_in_blocks"] == len(d2o) == info["n_blocks"] == otree.n_blocks
        tot["compactions"] += 1

    def state_agrees(tag):
        info = dtree.info()
        assert info["n_in_blocks"] == len(d2o) and info["n_blocks"] == otree.n_blocks, tag
        n = len(d2o)
        hit = torch.zeros(max(n, 1), dtype=torch.int32, device="cuda:0")
        ucnt, hit_pre, u_pre = torch.zeros_like(hit), torch.zeros_like(hit), torch.zeros_like(hit)
        priv = torch.zeros(max(n, 1), dtype=torch.uint8, device="cuda:0")
        skv.skv_counters_read(dtree, hit, ucnt)
        skv.skv_block_state_read(dtree, priv, hit_pre, u_pre)
        ep = device_epochs(skv, dtree)
        o_hit, o_ucnt = otree.counters()
        o_state = otree.block_state()
        o_ep = otree.epochs()
        alive = np.flatnonzero(priv[:n].cpu().numpy() != 255)
        o_alive = np.flatnonzero(o_state[0] != 255)
        assert np.array_equal(d2o[alive], o_alive), tag                      # the same blocks exist
        sel = d2o[alive]
        assert np.array_equal(hit[:n].cpu().numpy().view(np.uint32)[alive], o_hit[sel]), tag
        assert np.array_equal(ucnt[:n].cpu().numpy().view(np.uint32)[alive], o_ucnt[sel]), tag
        assert np.array_equal(priv[:n].cpu().numpy()[alive], o_state[0][sel]), tag
        assert np.array_equal(hit_pre[:n].cpu().numpy().view(np.uint32)[alive], o_state[1][sel]), tag
        assert np.array_equal(u_pre[:n].cpu().numpy().view(np.uint32)[alive], o_state[2][sel]), tag
        assert np.array_equal(ep[alive], o_ep[sel]), tag

    def lookups_agree(tag):
        for t in range(w.n_tenants):
            sample = [earlier[i] for i in g.choice(len(earlier), min(24, len(earlier)), replace=False)]
            o = np.concatenate([[0], np.cumsum([len(x) for x in sample])]).astype(np.int32)
            tk = np.concatenate(sample + [np.zeros(0, np.int32)]).astype(np.int32)
            ten = np.full(len(sample), t, np.int32)
            mb2 = max(max(len(x) // B for x in sample), 1)
            ml2, pt2 = device_match(skv, dtree, o, tk, ten, mb2)
            o_ml2, o_pt2 = otree.match(o, tk, ten, mb2)
            assert np.array_equal(ml2, o_ml2) and np.array_equal(pt2, o_pt2), (seed, tag, t)

    for rnd in range(n_rounds):
        otree.set_epoch(rnd + 1)
        skv.skv_set_epoch(dtree, rnd + 1)
        reqs, off, toks, tenants = make_round(g, earlier, vocab, w.n_tenants, n_req, block_vocab)
        mb = max(max(len(x) // B for x in reqs), 1)
        mlen, pt, pe = device_match(skv, dtree, off, toks, tenants, mb, want_path_end=True)
        o_mlen, o_pt, o_ids = otree.match(off, toks, tenants, mb, want_ids=True)
        assert np.array_equal(mlen, o_mlen) and np.array_equal(pt, o_pt), (seed, rnd)
        new_pages = np.full((n_req, mb + 1), -1, np.int32)
        for r, x in enumerate(reqs):
            for j in range(len(x) // B - mlen[r] // B):
                new_pages[r, j] = free_pages.pop()
        use_path_ends = copies and seed % 2 == 0         # path ends name records: a compaction invalidates them
        if g.random() < 0.1:
            compact()                                   # also when nothing forces it
            lookups_agree((rnd, "compacted early"))
            use_path_ends = False
        try:
            first, n = skv.skv_tree_insert(dtree, off, toks, tenants, mlen, new_pages, private_copies=copies,
                                           path_end=pe if use_path_ends else None)
        except skv.SkvError as e:
            assert e.code == -2, e                      # the slab is full of records that evictions left behind
            lookups_agree((rnd, "refused"))             # the refused insert changed nothing
            compact()
            tot["forced"] += 1
            first, n = skv.skv_tree_insert(dtree, off, toks, tenants, mlen, new_pages, private_copies=copies)
        o_before = otree.n_in_blocks
        o_first, o_n = otree.insert(off, toks, tenants, mlen, new_pages, private_copies=copies)
        assert np.array_equal(first, o_first) and np.array_equal(n, o_n), (seed, rnd)
        # both sides number the new blocks upwards from their own count, in request order
        d2o = np.concatenate([d2o, o_before + np.arange(int(n.sum()), dtype=np.int64)])
        assert otree.n_in_blocks == o_before + int(n.sum())
        tot["inserted"] += int(n.sum())
        if rnd % 3 == 0:                                 # the verifier clears a random part of what is cached
            alive = np.flatnonzero(otree.block_state()[0] != 255)
            pick = alive[g.random(len(alive)) < 0.3]
            if len(pick):
                assert (o2d()[pick] >= 0).all()
                skv.skv_promote(dtree, _dev(o2d()[pick].astype(np.int32)))
                otree.promote(pick.astype(np.int32))
        earlier = (earlier + reqs)[-200:]
        lookups_agree(rnd)
        if rnd % 5 == 4:                                 # a safeguard window ends: some public blocks turn private
            n_dem = torch.zeros(1, dtype=torch.int32, device="cuda:0")
            skv.skv_window_roll(dtree, skv.rdr_policy(**roll_policy), n_dem)
            want = otree.window_roll(**roll_policy)
            assert int(n_dem.item()) == want, (seed, rnd)
            tot["demoted"] += want
            lookups_agree((rnd, "window"))
        protect = o_ids[o_ids >= 0][::3].astype(np.int32)
        n_want = max(otree.n_blocks - keep, 0)
        ids, pages = skv.skv_evict(dtree, n_want, o2d()[protect].astype(np.int32))
        want_ids, want_pages = otree.evict(n_want, protect)
        assert np.array_equal(d2o[ids], want_ids) and np.array_equal(pages, want_pages), (seed, rnd)
        tot["evicted"] += len(ids)
        free_pages += [int(p) for p in pages]
        lookups_agree((rnd, "evicted"))
        state_agrees((seed, rnd))
    compact()
    lookups_agree("end")
    state_agrees((seed, "end"))
    tot["cap"] = cap
    return tot


@pytest.mark.parametrize("copies", [False, True])
def test_compaction_keeps_a_small_slab_going(copies):
    """Many times the slab's capacity goes through it; every forced compaction is followed by an insert that
    succeeds, and lookups, evictions, counters, visibility bits and epochs stay those of the oracle throughout."""
    demoted = 0
    for seed in range(6):
        print(f"[compact] copies={copies} stream {seed}", flush=True)
        tot = run_compact_stream(seed, n_rounds=60, copies=copies)
        print(f"[compact]   {tot}", flush=True)
        assert tot["evicted"] > 3 * tot["cap"] and tot["forced"] >= 3, tot
        demoted += tot["demoted"]
    assert demoted > 0


# ---------------------------------------------------------------------------------------------
# per-tenant copies of the same content (Section 4.1): insert below the requester's own path, branching lookup

def run_copy_stream(seed, n_rounds=5, n_req=10):
    from test_oracle_insert import make_round
    skv = _skv()
    block_vocab = 3 if seed % 3 == 0 else None
    w = inputs.small_random(seed=seed, n_req=8, p_sens=0.4, n_tenants=3, block_vocab=block_vocab)
    vocab = int(w.seq_tokens.max()) + 1 if len(w.seq_tokens) else 2
    otree = oracle.OracleTree.from_workload(w)
    dtree = skv.skv_tree_build(w.seq_tokens, w.seq_off, w.blk_sensitive, w.blk_owner, w.blk_page, w.n_tenants,
                               w.n_pages + 8192, device="cuda:0", reserve_blocks=2048)
    g = np.random.default_rng(3000 + seed)
    free_pages = list(range(w.n_pages, w.n_pages + 8192))[::-1]
    earlier = [w.req_tokens[w.req_off[r]: w.req_off[r + 1]] for r in range(w.n_req)]
    inserted = evicted = 0

    def lookups_agree(tag):
        for t in range(w.n_tenants):
            sample = [earlier[i] for i in g.choice(len(earlier), min(24, len(earlier)), replace=False)]
            o = np.concatenate([[0], np.cumsum([len(x) for x in sample])]).astype(np.int32)
            tk = np.concatenate(sample + [np.zeros(0, np.int32)]).astype(np.int32)
            ten = np.full(len(sample), t, np.int32)
            mb2 = max(max(len(x) // B for x in sample), 1)
            ml2, pt2 = device_match(skv, dtree, o, tk, ten, mb2)
            o_ml2, o_pt2 = otree.match(o, tk, ten, mb2)
            assert np.array_equal(ml2, o_ml2) and np.array_equal(pt2, o_pt2), (seed, tag, t)

    for rnd in range(n_rounds):
        otree.set_epoch(rnd + 1)
        skv.skv_set_epoch(dtree, rnd + 1)
        reqs, off, toks, tenants = make_round(g, earlier, vocab, w.n_tenants, n_req, block_vocab)
        mb = max(max(len(x) // B for x in reqs), 1)
        # even seeds hand the lookup's path ends to the insert (no search on the host), odd seeds let it search
        mlen, pt, pe = device_match(skv, dtree, off, toks, tenants, mb, want_path_end=True)
        o_mlen, o_pt, o_ids = otree.match(off, toks, tenants, mb, want_ids=True)
        assert np.array_equal(mlen, o_mlen) and np.array_equal(pt, o_pt), (seed, rnd)
        assert np.array_equal(pe >= 0, mlen > 0), (seed, rnd)
        new_pages = np.full((n_req, mb + 1), -1, np.int32)
        for r, x in enumerate(reqs):
            for j in range(len(x) // B - mlen[r] // B):
                new_pages[r, j] = free_pages.pop()
        first, n = skv.skv_tree_insert(dtree, off, toks, tenants, mlen, new_pages, private_copies=True,
                                       path_end=pe if seed % 2 == 0 else None)
        o_first, o_n = otree.insert(off, toks, tenants, mlen, new_pages, private_copies=True)
        assert np.array_equal(first, o_first) and np.array_equal(n, o_n), (seed, rnd)
        inserted += int(n.sum())
        # the verifier clears a random third of what is cached: public copies appear next to private ones
        priv = otree.block_state()[0]
        alive = np.flatnonzero(priv != 255)
        pick = alive[g.random(len(alive)) < 0.3].astype(np.int32)
        if len(pick):
            skv.skv_promote(dtree, _dev(pick))
            otree.promote(pick)
        earlier += reqs
        lookups_agree(rnd)
        if rnd % 2 == 1:
            protect = o_ids[o_ids >= 0][::3].astype(np.int32)
            n_want = int(g.integers(0, otree.n_blocks // 4 + 1))
            ids, pages = skv.skv_evict(dtree, n_want, protect)
            want_ids, want_pages = otree.evict(n_want, protect)
            assert np.array_equal(ids, want_ids) and np.array_equal(pages, want_pages), (seed, rnd)
            evicted += len(ids)
            free_pages += [int(p) for p in pages]
            lookups_agree((rnd, "evicted"))
        compare_state(skv, dtree, otree, (seed, rnd))
        assert np.array_equal(device_epochs(skv, dtree), otree.epochs()), (seed, rnd)
    return inserted, evicted


def test_private_copy_streams():
    tot = np.zeros(2, np.int64)
    for seed in range(30):
        print(f"[copies] stream {seed}", flush=True)
        tot += np.array(run_copy_stream(seed))
    assert tot[0] > 1000 and tot[1] > 200


def test_private_copy_lookup_backtracks():
    # the hand-made case of the oracle's pins, through the C ABI: tenant 1's own copy of X leads further than the
    # older, public copy of X
    skv = _skv()
    blocks = lambda *ids: np.concatenate([np.full(B, i, np.int32) for i in ids])
    X, Y, Z = 1, 2, 3
    seq = blocks(X, Y)
    args = (seq, np.array([0, 2 * B]), np.ones(2, np.uint8), np.zeros(2, np.int32), np.array([10, 11], np.int32))
    otree = oracle.OracleTree(*args)
    dtree = skv.skv_tree_build(*args, 3, 64, device="cuda:0", reserve_blocks=64)
    req, off, t1 = blocks(X, Z), np.array([0, 2 * B], np.int32), np.array([1], np.int32)
    mlen, _ = device_match(skv, dtree, off, req, t1, 2)
    assert mlen[0] == 0
    first, n = skv.skv_tree_insert(dtree, off, req, t1, mlen, np.array([[20, 21]], np.int32), private_copies=True)
    otree.insert(off, req, t1, mlen, np.array([[20, 21]], np.int32), private_copies=True)
    assert (first[0], n[0]) == (0, 2)
    skv.skv_promote(dtree, _dev(np.array([0], np.int32)))
    otree.promote([0])
    for q, ten in ((req, 1), (blocks(X, Y), 1), (req, 2), (blocks(X, Y), 0)):
        ml, pt = device_match(skv, dtree, off, q, np.array([ten], np.int32), 2)
        o_ml, o_pt = otree.match(off, q, np.array([ten], np.int32), 2)
        assert np.array_equal(ml, o_ml) and np.array_equal(pt, o_pt), (ten,)
    ml, pt = device_match(skv, dtree, off, req, t1, 2)
    otree.match(off, req, t1, 2)
    assert ml[0] == 2 * B and list(pt[0]) == [20, 21]
    compare_state(skv, dtree, otree, "backtrack")


def test_path_ends_continue_through_blocks_added_in_the_same_batch():
    """The insert is given the lookup's path ends.  Requests of one batch: A adds six blocks below a shared public
    prefix; B (same tenant) repeats A and goes on; C (same tenant) leaves A's new blocks after two of them; D (other
    tenant) has A's content and must get its own copy; E (same tenant as A) repeats B entirely.  First new block,
    counts and every later lookup must be the oracle's, which searches the updated tree for every request."""
    skv = _skv()
    g = np.random.default_rng(77)
    blk = lambda n: g.integers(0, 30000, n * B).astype(np.int32)
    prefix, a_new, b_more, c_other = blk(3), blk(6), blk(2), blk(3)
    seq_off = np.array([0, len(prefix)], np.int32)
    n_pages = 3 + 64
    otree = oracle.OracleTree(prefix, seq_off, np.zeros(3, np.uint8), np.zeros(3, np.int32), np.arange(3, dtype=np.int32))
    dtree = skv.skv_tree_build(prefix, seq_off, np.zeros(3, np.uint8), np.zeros(3, np.int32), np.arange(3, dtype=np.int32),
                               3, n_pages, device="cuda:0", reserve_blocks=64)
    reqs = [np.concatenate([prefix, a_new]), np.concatenate([prefix, a_new, b_more]),
            np.concatenate([prefix, a_new[: 2 * B], c_other]), np.concatenate([prefix, a_new]),
            np.concatenate([prefix, a_new, b_more])]
    tenants = np.array([1, 1, 1, 2, 1], np.int32)
    off = np.concatenate([[0], np.cumsum([len(x) for x in reqs])]).astype(np.int32)
    toks = np.concatenate(reqs).astype(np.int32)
    mb = max(len(x) // B for x in reqs)
    mlen, pt, pe = device_match(skv, dtree, off, toks, tenants, mb, want_path_end=True)
    o_mlen, o_pt = otree.match(off, toks, tenants, mb)
    assert np.array_equal(mlen, o_mlen) and np.array_equal(pt, o_pt) and (mlen == 3 * B).all()
    new_pages = np.full((len(reqs), mb), -1, np.int32)
    nxt = 3
    for r, x in enumerate(reqs):
        k = len(x) // B - 3
        new_pages[r, :k] = np.arange(nxt, nxt + k)
        nxt += k
    first, n = skv.skv_tree_insert(dtree, off, toks, tenants, mlen, new_pages, private_copies=True, path_end=pe)
    o_first, o_n = otree.insert(off, toks, tenants, mlen, new_pages, private_copies=True)
    assert np.array_equal(first, o_first) and np.array_equal(n, o_n), (first, o_first, n, o_n)
    assert list(first) == [3, 9, 5, 3, 11] and list(n) == [6, 2, 3, 6, 0]
    for t in range(3):
        ten = np.full(len(reqs), t, np.int32)
        ml2, pt2 = device_match(skv, dtree, off, toks, ten, mb)
        o_ml2, o_pt2 = otree.match(off, toks, ten, mb)
        assert np.array_equal(ml2, o_ml2) and np.array_equal(pt2, o_pt2), t
    compare_state(skv, dtree, otree, "same batch")


def test_branching_lookup_reports_its_limits():
    """More visible copies at one position than the lookup ranks, and more branch points / walks than it explores:
    the limits word says so; inside the limits it stays zero and results equal the oracle's."""
    skv = _skv()
    blocks = lambda *ids: np.concatenate([np.full(B, i, np.int32) for i in ids])
    T = 100
    # (a) 70 tenants each cache their own copy of the same two blocks below an empty tree; all copies are promoted
    args = (np.zeros(0, np.int32), np.zeros(1, np.int64), np.zeros(0, np.uint8), np.zeros(0, np.int32), np.zeros(0, np.int32))
    off = np.array([0, 2 * B], np.int32)
    for n_copies, want_flag in ((64, 0), (70, skv.SKV_LIMIT_COPIES)):
        otree = oracle.OracleTree(*args)
        dtree = skv.skv_tree_build(*args, T, 4096, device="cuda:0", reserve_blocks=1024)
        assert skv.skv_match_limits_read(dtree) == 0
        for c in range(n_copies):
            ten = np.array([c], np.int32)
            mlen, _ = device_match(skv, dtree, off, blocks(7, 8), ten, 2)
            assert mlen[0] == 0        # the copies of the others are private
            pages = np.array([[2 * c, 2 * c + 1]], np.int32)
            skv.skv_tree_insert(dtree, off, blocks(7, 8), ten, mlen, pages, private_copies=True)
            otree.insert(off, blocks(7, 8), ten, mlen, pages, private_copies=True)
        assert skv.skv_match_limits_read(dtree) == 0       # each tenant saw one visible copy at most
        ids = np.arange(otree.n_in_blocks, dtype=np.int32)
        skv.skv_promote(dtree, _dev(ids))
        otree.promote(ids)
        ml, pt = device_match(skv, dtree, off, blocks(7, 8), np.array([99], np.int32), 2)
        o_ml, o_pt = otree.match(off, blocks(7, 8), np.array([99], np.int32), 2)
        assert np.array_equal(ml, o_ml) and np.array_equal(pt, o_pt), n_copies    # equally long paths: the oldest copy
        assert skv.skv_match_limits_read(dtree) == want_flag, n_copies
        assert skv.skv_match_limits_read(dtree) == 0                                  # reading cleared it
    # (b) a ladder: every round one more position of the same 14-block sequence gets a second visible copy
    otree = oracle.OracleTree(*args)
    dtree = skv.skv_tree_build(*args, T, 4096, device="cuda:0", reserve_blocks=1024)
    seq = blocks(*range(20, 34))
    off = np.array([0, 14 * B], np.int32)
    page = 0
    hit_limit_at = None
    pos_of_id, promoted = {}, set()
    for rnd in range(14):
        ten = np.array([rnd], np.int32)
        mlen, _ = device_match(skv, dtree, off, seq, ten, 14)
        flags = skv.skv_match_limits_read(dtree)
        o_mlen, _ = otree.match(off, seq, ten, 14)
        if flags == 0:
            assert np.array_equal(mlen, o_mlen), rnd
        elif hit_limit_at is None:
            hit_limit_at = rnd
        # insert with the oracle's matched length, so that both sides build the same tree whatever the device found
        n_new = 14 - int(o_mlen[0]) // B
        pages = np.full((1, 14), -1, np.int32)
        pages[0, :n_new] = np.arange(page, page + n_new)
        page += n_new
        first, n = skv.skv_tree_insert(dtree, off, seq, ten, o_mlen, pages, private_copies=True)
        o_first, o_n = otree.insert(off, seq, ten, o_mlen, pages, private_copies=True)
        assert np.array_equal(first, o_first) and np.array_equal(n, o_n), rnd
        base_id = otree.n_in_blocks - int(n[0])
        for k in range(int(n[0])):
            pos_of_id[base_id + k] = int(first[0]) + k     # first_inserted: index of the request's first new block
        # the verifier clears every copy's blocks up to position rnd + 1: one more position with several visible copies
        ids = np.array([i for i, pos in pos_of_id.items() if pos <= rnd + 1 and i not in promoted], np.int32)
        if len(ids):
            skv.skv_promote(dtree, _dev(ids))
            otree.promote(ids)
            promoted.update(int(i) for i in ids)
        skv.skv_match_limits_read(dtree)
    print(f"[limits] ladder: first limit reported in round {hit_limit_at}", flush=True)
    assert hit_limit_at is not None and hit_limit_at >= 8


def test_private_copies_config3_full_size():
    """Full size: every request of config 3 adds its own copy of what it could not see; asked again, each request
    now reuses its whole prompt; other tenants gain nothing from the private copies; all of it agrees with the
    oracle, counters included."""
    skv = _skv()
    w = inputs.config3()
    otree = oracle.OracleTree.from_workload(w)
    nb_req = int((np.diff(w.req_off) // B).sum())
    dtree = skv.skv_tree_build(w.seq_tokens, w.seq_off, w.blk_sensitive, w.blk_owner, w.blk_page, w.n_tenants,
                               w.n_pages + nb_req, device="cuda:0", reserve_blocks=nb_req)
    mb = max(w.max_blocks, 1)
    mlen, pt, pe = device_match(skv, dtree, w.req_off, w.req_tokens, w.req_tenant, mb, want_path_end=True)
    o_mlen, _ = otree.match(w.req_off, w.req_tokens, w.req_tenant, mb)
    assert np.array_equal(mlen, o_mlen)
    full = np.diff(w.req_off) // B - mlen // B
    new_pages = np.full((w.n_req, int(full.max())), -1, np.int32)
    new_pages[np.arange(new_pages.shape[1])[None, :] < full[:, None]] = w.n_pages + np.arange(int(full.sum()), dtype=np.int32)
    # the lookup's path ends go to the insert: 256 requests of 64 tenants, many of them continuing what an earlier
    # request of the same tenant added in this very batch
    first, n = skv.skv_tree_insert(dtree, w.req_off, w.req_tokens, w.req_tenant, mlen, new_pages, private_copies=True,
                                   path_end=pe)
    o_first, o_n = otree.insert(w.req_off, w.req_tokens, w.req_tenant, mlen, new_pages, private_copies=True)
    assert np.array_equal(first, o_first) and np.array_equal(n, o_n)
    print(f"[copies] c3: {int(n.sum())} of {int(full.sum())} suffix blocks inserted", flush=True)
    for shift in (0, 1):
        ten = ((w.req_tenant + shift) % w.n_tenants).astype(np.int32)
        ml2, pt2 = device_match(skv, dtree, w.req_off, w.req_tokens, ten, mb)
        o_ml2, o_pt2 = otree.match(w.req_off, w.req_tokens, ten, mb)
        assert np.array_equal(ml2, o_ml2) and np.array_equal(pt2, o_pt2)
        if shift == 0:
            assert np.array_equal(ml2 // B, np.diff(w.req_off) // B)      # the stream now feeds itself completely
            print(f"   reuse before {int(mlen.sum())} tokens, after {int(ml2.sum())}", flush=True)
    compare_state(skv, dtree, otree, "c3 copies")
