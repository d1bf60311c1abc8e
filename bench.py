#!/usr/bin/env python3
"""Benchmark of the selective-reuse prefill path on one MI355X.

One step = one pass of the whole path over one batch of synthetic requests already resident in
HBM: counter reset + visible prefix match + suffix offsets, page gather of the reused KV, and
causal GQA prefill attention of the uncached suffixes.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c5|c4|c3|c2|c1] [--quick]

The default workload is the largest configuration, config 5 (1024 requests, 128 tenants) at 25 %
sensitive blocks; the other configurations, the config 5 sweep and the literal variant of config 4
are timed briefly in the same run and reported under "other_configs" (skipped with --quick).
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
MATCH_BYTES_PER_BLOCK = 150.0   # algorithmic bytes of the lookup per matched block ...
MATCH_BYTES_PER_HOP = 100.0     # ... and per node visited


def log(msg):
    print(f"[bench {time.strftime('%H:%M:%S')}] {msg}", file=sys.stderr, flush=True)


def attention_flops(w, mlen):
    import numpy as np
    S = (np.diff(w.req_off) - mlen).astype(np.float64)
    L = mlen.astype(np.float64)
    return 4.0 * w.attn.head_dim * w.attn.n_q_heads * float((S * L + S * (S + 1) / 2).sum())


def attention_min_bytes(w, mlen):
    """Every K/V row once, Q in, O out."""
    import numpy as np
    a = w.attn
    esz = 4 if a.dtype == "f32" else 2
    S = (np.diff(w.req_off) - mlen).astype(np.float64)
    L = mlen.astype(np.float64)
    return float((2 * a.n_kv_heads * a.head_dim * esz * (L + S) + 2 * S * a.n_q_heads * a.head_dim * esz).sum())


def measured_traffic(workload_key):
    """HBM bytes per launch of the library's kernels from the committed rocprofv3 counter runs
    (profiles/hbm_traffic.json), or None if there is none for this workload or a kernel source changed since."""
    import hashlib
    try:
        rec = json.load(open(os.path.join(ROOT, "profiles", "hbm_traffic.json")))
        h = hashlib.sha256()
        for f in rec["sources"]:
            h.update(open(os.path.join(ROOT, "paper_2508_08438_amd", "csrc", f), "rb").read())
        if h.hexdigest() != rec["sources_sha256"]:
            return None
        return rec["per_launch"][workload_key]
    except (OSError, KeyError, ValueError):
        return None


def node_hops(w, mlen):
    """Node visits charged to a batch of lookups.  The number of compressed nodes on a request's path is a property
    of the index, not of the request; every lookup visits at least the root's child table, so one hop per request is
    charged (a lower bound of the algorithmic bytes, hence of the fraction reported)."""
    return float(len(mlen))


def time_stages(sess, steps, torch, np):
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(steps)]
    t0 = time.perf_counter()
    for k in range(steps):  # events sit on the stream the kernels are launched on (torch's current stream)
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
    return elapsed, ms


def match_only_ms(sess, skv, torch, reps=30):
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    skv.skv_match(sess.tree, sess.req_off, sess.req_tokens, sess.req_tenant, sess.max_blocks, sess.matched_len,
                  sess.page_table)
    e0.record()
    for _ in range(reps):
        skv.skv_match(sess.tree, sess.req_off, sess.req_tokens, sess.req_tenant, sess.max_blocks, sess.matched_len,
                      sess.page_table)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps


def summarize(w, mlen, ms, np, match_ms=None):
    """Per-stage figures of one configuration from its stage times (ms per step, [steps, 3])."""
    a = w.attn
    esz = 4 if a.dtype == "f32" else 2
    t_match, t_gather, t_attn = (float(x) * 1e-3 for x in ms.mean(0))
    tokens = float(len(w.req_tokens))
    flops = attention_flops(w, mlen)
    gather_bytes = 2.0 * float(mlen.sum()) * 2 * a.n_kv_heads * a.head_dim * esz  # read + write, K and V
    peak = PEAK_BF16_TFLOPS if a.dtype == "bf16" else PEAK_FP32_TFLOPS
    out = {"requests": w.n_req, "prompt_tokens": int(tokens), "reused_tokens": int(mlen.sum()),
           "reuse_rate": float(mlen.sum()) / tokens,
           "stage_ms": {"match": t_match * 1e3, "gather": t_gather * 1e3, "attention": t_attn * 1e3},
           "prompt_tokens_per_s": tokens / (t_match + t_gather + t_attn),
           "lookups_per_s": w.n_req / t_match,
           "attention_tflops": flops / t_attn / 1e12, "attention_frac_of_peak": flops / t_attn / 1e12 / peak,
           "gather_gbs": gather_bytes / t_gather / 1e9 if mlen.sum() else 0.0,
           "gather_frac_of_hbm_peak": gather_bytes / t_gather / 1e9 / PEAK_HBM_GBS if mlen.sum() else 0.0}
    if match_ms is not None:
        mbytes = MATCH_BYTES_PER_BLOCK * float(mlen.sum()) / 16 + MATCH_BYTES_PER_HOP * node_hops(w, mlen)
        out["match_roofline"] = {"bound": "hbm", "kernel": "skv_match_kernel", "algorithmic_bytes": mbytes,
                                 "ms": match_ms, "achieved": mbytes / (match_ms * 1e-3) / 1e9, "peak": PEAK_HBM_GBS,
                                 "unit": "GB/s", "frac": mbytes / (match_ms * 1e-3) / 1e9 / PEAK_HBM_GBS}
        cb = mbytes + gather_bytes
        out["match_plus_gather_frac_of_hbm_peak"] = cb / (match_ms * 1e-3 + t_gather) / 1e9 / PEAK_HBM_GBS
    return out


def cpu_baseline(w, sess, mlen, pt, rows_target, flops_total, max_req):
    """Time the oracle, as it stands, on the host cores: match over the whole batch, gather and fp64
    attention on a bounded seeded sample (a few requests; a sample of their output rows), scaled to the
    batch by algorithmic bytes / flops."""
    import numpy as np
    import torch
    import oracle
    from paper_2508_08438_amd.inputs import BLOCK
    threads = min(16, os.cpu_count() or 1)
    log("oracle: building the index")
    t0 = time.perf_counter()
    tree = oracle.OracleTree.from_workload(w)
    t_build = time.perf_counter() - t0
    t0 = time.perf_counter()
    o_mlen, o_pt = tree.match(w.req_off, w.req_tokens, w.req_tenant, max(w.max_blocks, 1))
    t_match = time.perf_counter() - t0
    log(f"oracle: match over {w.n_req} requests took {t_match * 1e3:.2f} ms")
    exact = bool(np.array_equal(o_mlen, mlen) and np.array_equal(o_pt, pt))
    # sub-batch: a seeded choice of requests, their rows, and a compact pool of the pages they use
    g = np.random.default_rng(1234)
    S_all = np.diff(w.req_off) - o_mlen
    live = np.flatnonzero(S_all > 0)
    reqs = np.sort(g.choice(live, min(max_req, len(live)), replace=False))
    S = S_all[reqs]
    q_off = np.concatenate([[0], np.cumsum(S)]).astype(np.int32)
    parts = {x: [] for x in "qkv"}
    for n, r in enumerate(reqs):
        lo, hi = int(w.req_off[r]) + int(o_mlen[r]), int(w.req_off[r + 1])
        for x in "qkv":
            parts[x].append(w.token_rows(x, lo, hi))
        log(f"oracle: inputs of sampled request {n + 1}/{len(reqs)} drawn")
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
    log(f"oracle: fp64 attention on {rows_target} sampled rows, {threads} threads")
    t_attn, parts_out, chunk = 0.0, [], 8192
    for lo in range(0, rows_target, chunk):   # in chunks, so that a line appears every second or so
        hi = min(rows_target, lo + chunk)
        t0 = time.perf_counter()
        parts_out.append(oracle.attention(q, kn, vn, q_off, kpool, vpool, o_mlen[reqs], cpt, scale=a.scale,
                                          rows=(rr[lo:hi], rh[lo:hi], rp[lo:hi]), n_threads=threads))
        t_attn += time.perf_counter() - t0
        log(f"oracle: {hi}/{rows_target} rows, {t_attn:.2f} s so far")
    want = np.concatenate(parts_out)
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


def cold_stage_ms(sess, torch, np, reps=5):
    """Stage times with L2 and Infinity Cache flushed before every stage (512 MiB written in between)."""
    flush = torch.zeros(512 << 18, dtype=torch.float32, device=sess.device)   # 512 MiB
    ce = [torch.cuda.Event(enable_timing=True) for _ in range(6)]
    acc = np.zeros(3)
    for _ in range(reps):
        for i, stage in enumerate((sess.match, sess.gather, sess.attention)):
            flush.add_(1.0)
            ce[2 * i].record()
            stage()
            ce[2 * i + 1].record()
        torch.cuda.synchronize()
        acc += np.array([ce[2 * i].elapsed_time(ce[2 * i + 1]) for i in range(3)])
    del flush
    return dict(zip(("match", "gather", "attention"), (acc / reps).tolist()))


def brief_run(w, torch, np, skv, Session, steps=5, kpool=None, vpool=None):
    """A short timing of one more configuration: stage times and the figures derived from them."""
    sess = Session(w, device="cuda:0", kpool=kpool, vpool=vpool)
    sess.prepare()
    mlen = sess.host_matched_len.copy()
    for _ in range(2):
        sess.step()
    torch.cuda.synchronize()
    _, ms = time_stages(sess, steps, torch, np)
    m_ms = match_only_ms(sess, skv, torch, reps=10)
    out = summarize(w, mlen, ms, np, match_ms=m_ms)
    out["workload"] = w.name
    out["steps"] = steps
    hit, ucnt = sess.counters()
    out["sum_hit"] = int(hit.sum())
    out["blocks_hit"] = int((hit > 0).sum())
    return out, sess


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c5", choices=["c1", "c2", "c3", "c4", "c5"])
    ap.add_argument("--hard", action="store_true", help="N(0,1) tensor entries instead of N(0,1)/sqrt(d)")
    ap.add_argument("--literal", action="store_true", help="config 4 only: uniform owners and requesters")
    ap.add_argument("--calib-mib", type=int, default=0,
                    help="also run the library's plain streaming copy over this many MiB, outside the timed region, as "
                         "the known-size reference for HBM traffic counters")
    ap.add_argument("--p-sensitive", type=float, default=None,
                    help="config 5 only: fraction of cached blocks marked sensitive (0, 0.25, 0.5 or 1; nested sets)")
    ap.add_argument("--cold", action="store_true",
                    help="also time each stage after flushing L2 / Infinity Cache (512 MiB written between stages)")
    ap.add_argument("--quick", action="store_true",
                    help="main workload only: no other configurations, decode step, insert side or graph replay")
    ap.add_argument("--host-fill", action="store_true",
                    help="build every device buffer from host memory with plain copies (no torch device kernel runs in the "
                         "process; tensor values repeat one host-generated chunk): for hardware-counter runs.  Implies "
                         "--quick and no oracle leg")
    ap.add_argument("--cpu-rows", type=int, default=None,
                    help="oracle attention rows to time (0 = skip; default 32768 for c1/c2, 65536 for c3-c5, computed in chunks of "
                         "8192 with a progress line each)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: the path is measured on ONE GPU; --gpus N with N > 1 is not supported "
                 "(no collectives or sharding are part of it)")
    if args.host_fill:
        args.quick = True
        args.cpu_rows = 0
    if args.cpu_rows is None:
        args.cpu_rows = 32768 if args.workload in ("c1", "c2") else 65536

    import numpy as np
    import torch
    from paper_2508_08438_amd import binding as skv
    from paper_2508_08438_amd import inputs
    from paper_2508_08438_amd.pipeline import Session

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.p_sensitive is not None:
        assert args.workload == "c5", "--p-sensitive belongs to config 5"
        w = inputs.config5(p_sensitive=args.p_sensitive, hard=args.hard)
    elif args.literal:
        assert args.workload == "c4", "--literal belongs to config 4"
        w = inputs.config4(hard=args.hard, literal=True)
    else:
        w = inputs.CONFIGS[args.workload](hard=args.hard)
    log(f"workload {w.name}: building device state")
    sess = Session(w, device="cuda:0", host_fill=args.host_fill)
    sess.prepare()
    mlen = sess.host_matched_len.copy()

    log(f"{args.warmup} warm-up steps, {args.steps} timed steps")
    for _ in range(args.warmup):
        sess.step()
    torch.cuda.synchronize()
    K = args.steps
    elapsed, ms = time_stages(sess, K, torch, np)
    step_ms = ms.sum(1)
    t_attn = float(ms.mean(0)[2]) * 1e-3
    m_ms = match_only_ms(sess, skv, torch)
    main_fig = summarize(w, mlen, ms, np, match_ms=m_ms)

    # the box's own copy rate, and the known-size reference of the HBM counters
    copy_gbs = None
    n_copy = (args.calib_mib if args.calib_mib > 0 else 1024) << 20
    src = torch.empty(n_copy, dtype=torch.uint8, device=sess.device)
    dst = torch.empty_like(src)
    ce = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    skv.skv_stream_copy(dst, src)
    ce[0].record()
    for _ in range(5):
        skv.skv_stream_copy(dst, src)
    ce[1].record()
    torch.cuda.synchronize()
    copy_gbs = 2.0 * n_copy / (ce[0].elapsed_time(ce[1]) * 1e-3 / 5) / 1e9
    del src, dst

    # what the matrix cores sustain on operands distributed like this workload's tensors, and on constants: the
    # clock under matrix load depends on the values, so the first is the ceiling the attention kernel can be held to
    mfma_rate = None
    if w.attn.dtype == "bf16":
        n_val = skv.MFMA_RATE_OPERAND_BYTES // 2
        chunk = np.random.default_rng(7).standard_normal(1 << 20).astype(np.float32)
        if not args.hard:
            chunk /= np.sqrt(w.attn.head_dim)
        h_ops = torch.from_numpy(chunk).to(torch.bfloat16).repeat((n_val >> 20) + 1)[:n_val]
        sink = torch.empty(skv.MFMA_RATE_SINK_BYTES // 4, dtype=torch.float32).to(sess.device)
        mfma_rate = {"kernel": "mfma_rate_kernel", "unit": "TFLOP/s", "instruction": "v_mfma_f32_32x32x16_bf16"}
        d_ops = h_ops.to(sess.device)
        for label, ops, side in (("workload_like_values", d_ops, False),
                                 ("workload_like_values_with_softmax_side_work", d_ops, True),
                                 ("constant_values", torch.ones(n_val, dtype=torch.bfloat16).to(sess.device), False)):
            skv.skv_mfma_rate(ops, 40000, sink, side_work=side)            # the clock settles under load first
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
            ev[0].record()
            for i in range(3):
                fl = skv.skv_mfma_rate(ops, 40000, sink, side_work=side)
                ev[i + 1].record()
            torch.cuda.synchronize()
            ts = [ev[i].elapsed_time(ev[i + 1]) * 1e-3 for i in range(3)]
            mfma_rate[label] = fl / float(np.median(ts)) / 1e12
        del h_ops, sink, ops, d_ops

    tokens = float(len(w.req_tokens))
    a = w.attn
    flops = main_fig["attention_tflops"] * 1e12 * t_attn
    peak = PEAK_BF16_TFLOPS if a.dtype == "bf16" else PEAK_FP32_TFLOPS
    traffic_rec = None if (args.hard or args.literal) else measured_traffic(w.name)
    attn_kernel = "attn_bf16_kernel" if a.dtype == "bf16" else "attn_f32_kernel"
    traffic = None
    if traffic_rec and attn_kernel in traffic_rec:
        t = traffic_rec[attn_kernel]
        traffic = t["read_bytes"] + t["write_bytes"]
    out = {
        "metric": "selective-reuse prefill tokens/s + prefix-match lookups/s on 1 MI355X",
        "value": tokens * K / elapsed, "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": args.warmup,
        "ms_per_step": elapsed / K * 1e3, "ms_per_step_median": float(np.median(step_ms)),
        "ms_per_step_min": float(step_ms.min()), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": a.dtype, "data": "synthetic" + (" (host-filled, repeated chunk)" if args.host_fill else ""),
        "config": {"workload": f"{w.name}{'_hard' if args.hard else ''}: {w.n_req} requests, {w.n_tenants} tenants, "
                               f"{int(tokens)} prompt tokens, {int(mlen.sum())} reused, "
                               f"GQA {a.n_q_heads}/{a.n_kv_heads} d={a.head_dim} {a.dtype}",
                   "requests": w.n_req, "prompt_tokens": int(tokens), "reused_tokens": int(mlen.sum()),
                   "reuse_rate": float(mlen.sum()) / tokens},
        "lookups_per_s": main_fig["lookups_per_s"],
        "lookups_per_s_match_call_only": w.n_req / (m_ms * 1e-3),
        "computed_tokens_per_s": (tokens - float(mlen.sum())) / t_attn,
        "stage_ms": main_fig["stage_ms"],
        "gather_gbs": main_fig["gather_gbs"],
        "stream_copy_gbs": copy_gbs,
        "match_roofline": main_fig["match_roofline"],
        "match_plus_gather_frac_of_hbm_peak": main_fig["match_plus_gather_frac_of_hbm_peak"],
        "roofline": {"bound": "mfma" if a.dtype == "bf16" else "alu", "kernel": attn_kernel,
                     "achieved": main_fig["attention_tflops"], "peak": peak, "unit": "TFLOP/s",
                     "frac": main_fig["attention_frac_of_peak"], "traffic": traffic,
                     "traffic_unit": "HBM bytes per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE, scaled)",
                     "min_bytes_per_launch": attention_min_bytes(w, mlen),
                     "flops_per_launch": flops, "avg_launch_ms": t_attn * 1e3},
        "hbm_traffic_per_launch": traffic_rec,
    }
    if mfma_rate:
        out["mfma_sustained"] = mfma_rate
        out["roofline"]["frac_of_sustained_mfma_rate_on_workload_like_values"] = (
            main_fig["attention_tflops"] / mfma_rate["workload_like_values"])
        out["roofline"]["frac_of_sustained_rate_with_softmax_side_work"] = (
            main_fig["attention_tflops"] / mfma_rate["workload_like_values_with_softmax_side_work"])

    # the counters after one step of this batch: what the safeguard would read (reuse statistics of the workload)
    hit, ucnt = sess.counters()
    used = hit > 0
    rdr = ucnt[used] / hit[used]
    out["reuse_stats"] = {"sum_hit": int(hit.sum()), "blocks_hit": int(used.sum()),
                          "rdr_histogram_10_bins_0_to_1": np.histogram(rdr, bins=10, range=(0.0, 1.0))[0].tolist()}

    if args.cold:
        out["stage_ms_cold_cache"] = cold_stage_ms(sess, torch, np)

    sg = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    if not args.host_fill:
        # a sixteen times longer request stream in one launch (the batch repeated with re-drawn tenants): steady-state
        # lookups/s, where the single batch mostly measures launch latency
        rep = 16
        g16 = np.random.default_rng(16)
        lens = np.diff(w.req_off)
        off16 = np.concatenate([[0], np.cumsum(np.tile(lens, rep))]).astype(np.int64)
        if off16[-1] < 2 ** 31 and w.n_req * rep * sess.max_blocks < 2 ** 30:
            ten16 = g16.integers(0, w.n_tenants, w.n_req * rep).astype(np.int32)
            d_off16 = torch.from_numpy(off16.astype(np.int32)).to(sess.device)
            d_tok16 = sess.req_tokens.repeat(rep)
            d_ten16 = torch.from_numpy(ten16).to(sess.device)
            d_len16 = torch.zeros(w.n_req * rep, dtype=torch.int32, device=sess.device)
            d_pt16 = torch.empty((w.n_req * rep, sess.max_blocks), dtype=torch.int32, device=sess.device)
            skv.skv_match(sess.tree, d_off16, d_tok16, d_ten16, sess.max_blocks, d_len16, d_pt16)
            sg[0].record()
            for _ in range(10):
                skv.skv_match(sess.tree, d_off16, d_tok16, d_ten16, sess.max_blocks, d_len16, d_pt16)
            sg[1].record()
            torch.cuda.synchronize()
            ml16 = d_len16.cpu().numpy()
            t16 = sg[0].elapsed_time(sg[1]) * 1e-3 / 10
            b16 = MATCH_BYTES_PER_BLOCK * float(ml16.sum()) / 16 + MATCH_BYTES_PER_HOP * float(len(ml16))
            out["lookups_x16_stream"] = {"requests": w.n_req * rep, "ms": t16 * 1e3, "lookups_per_s": w.n_req * rep / t16,
                                         "algorithmic_gbs": b16 / t16 / 1e9, "frac_of_hbm_peak": b16 / t16 / 1e9 / PEAK_HBM_GBS}
            del d_pt16, d_tok16

        # safeguard step (window roll + RDR scan), outside the timed region: a streaming pass over the block records
        pol = skv.rdr_policy(direction=0, tau=(1, 2), min_hits=2, n_consec=2)
        skv.skv_window_roll(sess.tree, pol)
        sg[0].record()
        for _ in range(10):
            skv.skv_window_roll(sess.tree, pol)
        sg[1].record()
        torch.cuda.synchronize()
        t_roll = sg[0].elapsed_time(sg[1]) * 1e-3 / 10
        n_tree_blocks = sess.tree.info()["n_blocks"]
        out["safeguard"] = {"blocks": n_tree_blocks, "ms": t_roll * 1e3, "gbs": n_tree_blocks * 68.0 / t_roll / 1e9,
                            "bytes_per_block": 68}

    if not args.quick:
        # the same pass recorded once as a HIP graph and replayed (no per-stage events, one launch per step)
        sess.capture_step()
        sess.replay()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        n_rep = max(3, K // 4)
        for _ in range(n_rep):
            sess.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - t1) / n_rep * 1e3
        out["graph_replay"] = {"ms_per_step": graph_ms, "tokens_per_s": tokens / (graph_ms * 1e-3)}

        # insert side, outside the timed region: the suffixes' full blocks written to fresh pages (read + write, K, V)
        q_off_h = sess.q_off.cpu().numpy()
        full = np.diff(q_off_h) // 16
        n_new = int(full.sum())
        if n_new and 2 * n_new * 16 * a.n_kv_heads * a.head_dim * 2 < 40e9:
            mb = int(full.max())
            table = np.full((w.n_req, mb), -1, np.int32)
            table[np.arange(mb)[None, :] < full[:, None]] = np.random.default_rng(0).permutation(n_new).astype(np.int32)
            table = torch.from_numpy(table).to(sess.device)
            shape = (n_new, 16, a.n_kv_heads, a.head_dim)
            kp2 = torch.empty(shape, dtype=a.torch_dtype, device=sess.device)
            vp2 = torch.empty_like(kp2)
            skv.skv_scatter_kv(sess.desc, sess.knew, sess.vnew, sess.q_off, table, kp2, vp2)
            sg[0].record()
            for _ in range(5):
                skv.skv_scatter_kv(sess.desc, sess.knew, sess.vnew, sess.q_off, table, kp2, vp2)
            sg[1].record()
            torch.cuda.synchronize()
            t_scatter = sg[0].elapsed_time(sg[1]) * 1e-3 / 5
            out["insert"] = {"pages": n_new, "ms": t_scatter * 1e3,
                             "gbs": 2.0 * n_new * 16 * 2 * a.n_kv_heads * a.head_dim * (4 if a.dtype == "f32" else 2)
                             / t_scatter / 1e9}
            del kp2, vp2

    pt = sess.page_table.cpu().numpy()
    if args.cpu_rows > 0:
        cb, err, exact = cpu_baseline(w, sess, mlen, pt, args.cpu_rows, flops,
                                      max_req=8 if args.workload in ("c1", "c2") else 4)
        out["cpu_baseline"] = cb
        out["parity"] = {"match_exact": exact, "attention_max_abs_err": err}

    if not args.quick:
        # decode step on its own workload: 64 requests, contexts 4096..16384 tokens
        if a.dtype == "bf16":
            log("decode step")
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
            out["decode"] = {"requests": dw.n_req, "cached_tokens": int(dw.ctx_len.sum()), "ms": t_dec * 1e3,
                             "tokens_per_s": dw.n_req / t_dec, "gbs": dbytes / t_dec / 1e9,
                             "frac_of_hbm_peak": dbytes / t_dec / 8e12}
            del dk, dv

        # the other configurations, briefly: stage times, roofline fractions, reuse
        others = {}
        kpool, vpool = sess.kpool, sess.vpool
        main_is_c5 = args.workload == "c5" and not args.hard
        del sess.q, sess.knew, sess.vnew, sess.out, sess.kctx, sess.vctx
        if not main_is_c5:
            del sess, kpool, vpool
            kpool = vpool = None
        torch.cuda.empty_cache()
        plan = []
        for p in (0.0, 0.25, 0.5, 1.0):
            if not (main_is_c5 and w.name == f"c5_sweep_p{int(round(100 * p))}"):
                plan.append((f"c5_p{int(100 * p)}", lambda p=p: inputs.config5(p_sensitive=p), True))
        plan += [("c4", lambda: inputs.config4(), False), ("c4_literal", lambda: inputs.config4(literal=True), False),
                 ("c3", lambda: inputs.config3(), False), ("c2", lambda: inputs.config2(), False)]
        for key, make, share in plan:
            if key == args.workload and not args.hard and not args.literal:
                continue
            log(f"other configuration {key}")
            w2 = make()
            use_pools = share and main_is_c5
            fig, s2 = brief_run(w2, torch, np, skv, Session, steps=5 if key.startswith("c5") else 10,
                                kpool=kpool if use_pools else None, vpool=vpool if use_pools else None)
            if key == "c4":   # a request's whole K/V fits the 256 MB Infinity Cache: warm and cold both
                fig["stage_ms_cold_cache"] = cold_stage_ms(s2, torch, np)
            others[key] = fig
            del s2
            torch.cuda.empty_cache()
        out["other_configs"] = others
    print(json.dumps(out))


if __name__ == "__main__":
    main()
