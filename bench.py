#!/usr/bin/env python3
"""Benchmark of the selective-reuse prefill path on one MI355X.

One step = one pass of the whole path over one batch of synthetic requests already resident in
HBM: counter reset + visible prefix match + suffix offsets, page gather of the reused KV, and
causal GQA prefill attention of the uncached suffixes.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c2|c3|c4|c5|c1]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_FP32_TFLOPS = 157.3    # vector fp32 (the fp32 correctness configuration)
PEAK_HBM_GBS = 8000.0


def attention_flops(w, mlen):
    import numpy as np
    S = (np.diff(w.req_off) - mlen).astype(np.float64)
    L = mlen.astype(np.float64)
    return 4.0 * w.attn.head_dim * w.attn.n_q_heads * float((S * L + S * (S + 1) / 2).sum())


def measured_traffic(workload_key, kernel):
    """HBM bytes per launch from the committed rocprofv3 counter runs (profiles/hbm_traffic.json), or None
    if there is no measurement for this workload or the kernel source changed since it was taken."""
    import hashlib
    try:
        rec = json.load(open(os.path.join(ROOT, "profiles", "hbm_traffic.json")))
        src = os.path.join(ROOT, "paper_2508_08438_amd", "csrc", "skv_attn.hip")
        if hashlib.sha256(open(src, "rb").read()).hexdigest() != rec["attn_source_sha256"]:
            return None
        t = rec["per_launch"][workload_key][kernel]
        return t["read_bytes"] + t["write_bytes"]
    except (OSError, KeyError, ValueError):
        return None


def cpu_baseline(w, sess, mlen, pt, rows_target, flops_total, max_req=8):
    """Time the oracle, as it stands, on the host cores: match over the whole batch, gather and fp64
    attention on a bounded seeded sample (a few requests; a sample of their output rows), scaled to the
    batch by algorithmic bytes / flops."""
    import numpy as np
    import torch
    import oracle
    from paper_2508_08438_amd.inputs import BLOCK
    threads = min(16, os.cpu_count() or 1)
    t0 = time.perf_counter()
    tree = oracle.OracleTree.from_workload(w)
    t_build = time.perf_counter() - t0
    t0 = time.perf_counter()
    o_mlen, o_pt = tree.match(w.req_off, w.req_tokens, w.req_tenant, max(w.max_blocks, 1))
    t_match = time.perf_counter() - t0
    exact = bool(np.array_equal(o_mlen, mlen) and np.array_equal(o_pt, pt))
    # sub-batch: a seeded choice of requests, their rows, and a compact pool of the pages they use
    g = np.random.default_rng(1234)
    S_all = np.diff(w.req_off) - o_mlen
    live = np.flatnonzero(S_all > 0)
    reqs = np.sort(g.choice(live, min(max_req, len(live)), replace=False))
    S = S_all[reqs]
    q_off = np.concatenate([[0], np.cumsum(S)]).astype(np.int32)
    parts = {x: [] for x in "qkv"}
    for r in reqs:
        lo, hi = int(w.req_off[r]) + int(o_mlen[r]), int(w.req_off[r + 1])
        for x in "qkv":
            parts[x].append(w.token_rows(x, lo, hi))
    q, kn, vn = (torch.cat(parts[x]) for x in "qkv")
    sub_pt = o_pt[reqs]
    pages = np.unique(sub_pt[sub_pt >= 0])
    relabel = {int(p): i for i, p in enumerate(pages)}
    cpt = np.array([[relabel.get(int(p), -1) for p in row] for row in sub_pt], dtype=np.int32).reshape(sub_pt.shape)
    a = w.attn
    shape = (max(len(pages), 1), BLOCK, a.n_kv_heads, a.head_dim)
    kpool, vpool = torch.zeros(shape, dtype=a.torch_dtype), torch.zeros(shape, dtype=a.torch_dtype)
    for i, pg in enumerate(pages):
        kpool[i] = w.pool_pages("k", int(pg), int(pg) + 1)[0]
        vpool[i] = w.pool_pages("v", int(pg), int(pg) + 1)[0]
    t0 = time.perf_counter()
    oracle.gather(kpool, vpool, o_mlen[reqs], cpt)
    t_gather = time.perf_counter() - t0
    t_gather_full = t_gather * float(o_mlen.sum()) / max(float(o_mlen[reqs].sum()), 1.0)
    rr = g.integers(0, len(reqs), rows_target).astype(np.int32)
    rp = (g.random(rows_target) * S[rr]).astype(np.int32)
    rh = g.integers(0, a.n_q_heads, rows_target).astype(np.int32)
    t0 = time.perf_counter()
    want = oracle.attention(q, kn, vn, q_off, kpool, vpool, o_mlen[reqs], cpt, scale=a.scale,
                            rows=(rr, rh, rp), n_threads=threads)
    t_attn = time.perf_counter() - t0
    sample_flops = 4.0 * a.head_dim * float((o_mlen[reqs][rr] + rp + 1).sum())
    t_attn_full = t_attn * flops_total / sample_flops
    tokens = float(len(w.req_tokens))
    q_off_all = np.concatenate([[0], np.cumsum(S_all)]).astype(np.int64)
    idx = torch.from_numpy(q_off_all[reqs[rr]] + rp).to(sess.out.device)
    got = sess.out[idx, torch.from_numpy(rh.astype(np.int64)).to(idx.device)].double().cpu().numpy()
    err = float(np.abs(got - want).max())
    return {"value": tokens / (t_match + t_gather_full + t_attn_full), "unit": "tokens/s", "cores": threads,
            "kind": "oracle",
            "sample": f"match over all {w.n_req} requests ({t_match * 1e3:.2f} ms, 1 thread); gather of {len(reqs)} requests "
                      f"({t_gather * 1e3:.2f} ms, 1 thread) and fp64 attention on {rows_target} seeded (request, head, row) "
                      f"samples of those requests ({t_attn:.2f} s on {threads} threads), scaled to the batch by reused "
                      f"bytes / algorithmic flops",
            "lookups_per_s": w.n_req / t_match, "tree_build_s": t_build}, err, exact


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c2", choices=["c1", "c2", "c3", "c4", "c5"])
    ap.add_argument("--hard", action="store_true", help="N(0,1) tensor entries instead of N(0,1)/sqrt(d)")
    ap.add_argument("--calib-mib", type=int, default=0,
                    help="also run one plain streaming kernel (out = 2 * in over this many MiB of fp32) outside the "
                         "timed region, as the known-size reference for HBM traffic counters")
    ap.add_argument("--p-sensitive", type=float, default=None,
                    help="config 5 only: fraction of cached blocks marked sensitive (0, 0.25, 0.5 or 1; nested sets)")
    ap.add_argument("--cold", action="store_true",
                    help="also time each stage after flushing L2 / Infinity Cache (512 MiB written between stages)")
    ap.add_argument("--no-decode", action="store_true", help="skip the decode-step attention measurement")
    ap.add_argument("--no-graph", action="store_true", help="skip the HIP-graph replay of the same pass")
    ap.add_argument("--cpu-rows", type=int, default=262144, help="oracle attention rows to time (0 = skip)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: the path is measured on ONE GPU; --gpus N with N > 1 is not supported "
                 "(no collectives or sharding are part of it)")

    import numpy as np
    import torch
    from paper_2508_08438_amd import inputs
    from paper_2508_08438_amd.pipeline import Session

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.p_sensitive is not None:
        assert args.workload == "c5", "--p-sensitive belongs to config 5"
        w = inputs.config5(p_sensitive=args.p_sensitive, hard=args.hard)
    else:
        w = inputs.CONFIGS[args.workload](hard=args.hard)
    sess = Session(w, device="cuda:0")
    sess.prepare()
    mlen = sess.host_matched_len.copy()

    for _ in range(args.warmup):
        sess.step()
    torch.cuda.synchronize()
    if args.calib_mib > 0:
        src = torch.ones(args.calib_mib * (1 << 18), dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        torch.mul(src, 2.0, out=dst)
        torch.cuda.synchronize()
        del src, dst
    K = args.steps
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(K)]
    t0 = time.perf_counter()
    for k in range(K):  # events sit on the stream the kernels are launched on (torch's current stream)
        ev[k][0].record()
        sess.match()
        ev[k][1].record()
        sess.gather()
        ev[k][2].record()
        sess.attention()
        ev[k][3].record()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms = np.array([[e[i].elapsed_time(e[i + 1]) for i in range(3)] for e in ev])
    t_match, t_gather, t_attn = (float(x) * 1e-3 for x in ms.mean(0))
    step_ms = ms.sum(1)

    # the same pass recorded once as a HIP graph and replayed K times (no per-stage events, one launch per step)
    graph_ms = None
    if not args.no_graph:
        sess.capture_step()
        sess.replay()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(K):
            sess.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - t1) / K * 1e3

    from paper_2508_08438_amd import binding as skv
    # the counters after one step of this batch: what the safeguard would read (reuse statistics of the workload)
    hit, ucnt = sess.counters()
    used = hit > 0
    rdr = ucnt[used] / hit[used]
    reuse_stats = {"sum_hit": int(hit.sum()), "blocks_hit": int(used.sum()),
                   "rdr_histogram_10_bins_0_to_1": np.histogram(rdr, bins=10, range=(0.0, 1.0))[0].tolist()}

    stage_ms_cold = None
    if args.cold:
        flush = torch.zeros(512 << 18, dtype=torch.float32, device=sess.device)   # 512 MiB
        ce = [torch.cuda.Event(enable_timing=True) for _ in range(6)]
        acc = np.zeros(3)
        for _ in range(5):
            for i, stage in enumerate((sess.match, sess.gather, sess.attention)):
                flush.add_(1.0)
                ce[2 * i].record()
                stage()
                ce[2 * i + 1].record()
            torch.cuda.synchronize()
            acc += np.array([ce[2 * i].elapsed_time(ce[2 * i + 1]) for i in range(3)])
        stage_ms_cold = dict(zip(("match", "gather", "attention"), (acc / 5).tolist()))
        del flush

    # a sixteen times longer request stream in one launch (the batch repeated with re-drawn tenants): steady-state
    # lookups/s, where the single batch mostly measures launch latency
    rep = 16
    g16 = np.random.default_rng(16)
    lens = np.diff(w.req_off)
    off16 = np.concatenate([[0], np.cumsum(np.tile(lens, rep))]).astype(np.int64)
    x16 = None
    if off16[-1] < 2 ** 31 and w.n_req * rep * sess.max_blocks < 2 ** 30:
        ten16 = g16.integers(0, w.n_tenants, w.n_req * rep).astype(np.int32)
        d_off16 = torch.from_numpy(off16.astype(np.int32)).to(sess.device)
        d_tok16 = sess.req_tokens.repeat(rep)
        d_ten16 = torch.from_numpy(ten16).to(sess.device)
        d_len16 = torch.zeros(w.n_req * rep, dtype=torch.int32, device=sess.device)
        d_pt16 = torch.empty((w.n_req * rep, sess.max_blocks), dtype=torch.int32, device=sess.device)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        skv.skv_match(sess.tree, d_off16, d_tok16, d_ten16, sess.max_blocks, d_len16, d_pt16)
        e0.record()
        for _ in range(10):
            skv.skv_match(sess.tree, d_off16, d_tok16, d_ten16, sess.max_blocks, d_len16, d_pt16)
        e1.record()
        torch.cuda.synchronize()
        x16 = {"requests": w.n_req * rep, "ms": e0.elapsed_time(e1) / 10,
               "lookups_per_s": w.n_req * rep / (e0.elapsed_time(e1) * 1e-3 / 10)}
        del d_pt16, d_tok16

    # safeguard step (window roll + RDR scan), outside the timed region: a streaming pass over the block records
    pol = skv.rdr_policy(direction=0, tau=(1, 2), min_hits=2, n_consec=2)
    sg = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    skv.skv_window_roll(sess.tree, pol)
    sg[0].record()
    for _ in range(10):
        skv.skv_window_roll(sess.tree, pol)
    sg[1].record()
    torch.cuda.synchronize()
    t_roll = sg[0].elapsed_time(sg[1]) * 1e-3 / 10
    n_tree_blocks = sess.tree.info()["n_blocks"]

    # the lookup call alone (skv_match: walk + counter atomics), back to back; the step's "match" stage above also
    # holds the counter reset and the suffix-offset scan
    sg[0].record()
    for _ in range(50):
        skv.skv_match(sess.tree, sess.req_off, sess.req_tokens, sess.req_tenant, sess.max_blocks, sess.matched_len,
                      sess.page_table)
    sg[1].record()
    torch.cuda.synchronize()
    t_match_only = sg[0].elapsed_time(sg[1]) * 1e-3 / 50

    # insert side, outside the timed region: the suffixes' full blocks written to fresh pages (read + write, K and V)
    q_off_h = sess.q_off.cpu().numpy()
    full = np.diff(q_off_h) // 16
    n_new = int(full.sum())
    t_scatter = None
    if n_new:
        mb = int(full.max())
        table = np.full((w.n_req, mb), -1, np.int32)
        table[np.arange(mb)[None, :] < full[:, None]] = np.random.default_rng(0).permutation(n_new).astype(np.int32)
        table = torch.from_numpy(table).to(sess.device)
        shape = (n_new, 16, w.attn.n_kv_heads, w.attn.head_dim)
        kp2 = torch.empty(shape, dtype=w.attn.torch_dtype, device=sess.device)
        vp2 = torch.empty_like(kp2)
        skv.skv_scatter_kv(sess.desc, sess.knew, sess.vnew, sess.q_off, table, kp2, vp2)
        sg[0].record()
        for _ in range(10):
            skv.skv_scatter_kv(sess.desc, sess.knew, sess.vnew, sess.q_off, table, kp2, vp2)
        sg[1].record()
        torch.cuda.synchronize()
        t_scatter = sg[0].elapsed_time(sg[1]) * 1e-3 / 10
        del kp2, vp2

    # decode step, outside the timed region and on its own workload: 64 requests, contexts 4096..16384 tokens
    decode = None
    if not args.no_decode and w.attn.dtype == "bf16":
        dw = inputs.decode_workload()
        da = dw.attn
        dshape = (dw.n_pages, 16, da.n_kv_heads, da.head_dim)
        dk = torch.empty(dshape, dtype=da.torch_dtype, device=sess.device)
        dv = torch.empty(dshape, dtype=da.torch_dtype, device=sess.device)
        dw.fill_pool("k", dk)
        dw.fill_pool("v", dv)
        dq = dw.queries(sess.device)
        dout = torch.zeros_like(dq)
        ddesc = skv.attn_desc(da.n_q_heads, da.n_kv_heads, da.head_dim, da.dtype, da.scale)
        dws = torch.zeros(skv.skv_decode_attn_workspace_size(ddesc, dw.n_req, dw.max_blocks), dtype=torch.uint8,
                          device=sess.device)
        dctx = torch.from_numpy(dw.ctx_len).to(sess.device)
        dpt = torch.from_numpy(dw.page_table).to(sess.device)
        for _ in range(3):
            skv.skv_decode_attn(ddesc, dq, dk, dv, dctx, dpt, dw.max_blocks, dout, dws)
        sg[0].record()
        for _ in range(20):
            skv.skv_decode_attn(ddesc, dq, dk, dv, dctx, dpt, dw.max_blocks, dout, dws)
        sg[1].record()
        torch.cuda.synchronize()
        t_dec = sg[0].elapsed_time(sg[1]) * 1e-3 / 20
        dbytes = float(dw.ctx_len.sum()) * 2 * da.n_kv_heads * da.head_dim * 2    # every cached K and V byte once
        decode = {"requests": dw.n_req, "cached_tokens": int(dw.ctx_len.sum()), "ms": t_dec * 1e3,
                  "tokens_per_s": dw.n_req / t_dec, "gbs": dbytes / t_dec / 1e9, "frac_of_hbm_peak": dbytes / t_dec / 8e12}
        del dk, dv

    tokens = float(len(w.req_tokens))
    pt = sess.page_table.cpu().numpy()
    flops = attention_flops(w, mlen)
    a = w.attn
    esz = 4 if a.dtype == "f32" else 2
    gather_bytes = 2.0 * float(mlen.sum()) * 2 * a.n_kv_heads * a.head_dim * esz  # read + write, K and V
    peak = PEAK_BF16_TFLOPS if a.dtype == "bf16" else PEAK_FP32_TFLOPS
    achieved = flops / t_attn / 1e12
    out = {
        "metric": "selective-reuse prefill tokens/s + prefix-match lookups/s on 1 MI355X",
        "value": tokens * K / elapsed, "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": args.warmup,
        "ms_per_step": elapsed / K * 1e3, "ms_per_step_median": float(np.median(step_ms)),
        "ms_per_step_min": float(step_ms.min()), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": a.dtype, "data": "synthetic",
        "config": {"workload": f"{w.name}{'_hard' if args.hard else ''}: {w.n_req} requests, {w.n_tenants} tenants, "
                               f"{int(tokens)} prompt tokens, {int(mlen.sum())} reused, "
                               f"GQA {a.n_q_heads}/{a.n_kv_heads} d={a.head_dim} {a.dtype}",
                   "requests": w.n_req, "prompt_tokens": int(tokens), "reused_tokens": int(mlen.sum()),
                   "reuse_rate": float(mlen.sum()) / tokens},
        "graph_replay": None if graph_ms is None else {"ms_per_step": graph_ms, "tokens_per_s": tokens / (graph_ms * 1e-3)},
        "lookups_per_s": w.n_req / t_match,
        "lookups_per_s_match_call_only": w.n_req / t_match_only,
        "lookups_x16_stream": x16,
        "reuse_stats": reuse_stats,
        "stage_ms_cold_cache": stage_ms_cold,
        "computed_tokens_per_s": (tokens - float(mlen.sum())) / t_attn,
        "stage_ms": {"match": t_match * 1e3, "gather": t_gather * 1e3, "attention": t_attn * 1e3},
        "gather_gbs": gather_bytes / t_gather / 1e9 if mlen.sum() else 0.0,
        "safeguard": {"blocks": n_tree_blocks, "ms": t_roll * 1e3, "gbs": n_tree_blocks * 68.0 / t_roll / 1e9,
                      "bytes_per_block": 68},
        "insert": None if t_scatter is None else {
            "pages": n_new, "ms": t_scatter * 1e3,
            "gbs": 2.0 * n_new * 16 * 2 * w.attn.n_kv_heads * w.attn.head_dim * (4 if w.attn.dtype == "f32" else 2)
            / t_scatter / 1e9},
        "decode": decode,
        "roofline": {"bound": "mfma" if a.dtype == "bf16" else "alu", "kernel": "attn_bf16_kernel"
                     if a.dtype == "bf16" else "attn_f32_kernel", "achieved": achieved, "peak": peak,
                     "unit": "TFLOP/s", "frac": achieved / peak,
                     "traffic": None if args.hard else measured_traffic(args.workload, "attn_bf16_kernel"),
                     "traffic_unit": "HBM bytes per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE, scaled)",
                     "flops_per_launch": flops, "avg_launch_ms": t_attn * 1e3},
    }
    if args.cpu_rows > 0:
        cb, err, exact = cpu_baseline(w, sess, mlen, pt, args.cpu_rows, flops)
        out["cpu_baseline"] = cb
        out["parity"] = {"match_exact": exact, "attention_max_abs_err": err}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
