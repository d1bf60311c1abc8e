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


def cpu_baseline(w, sess, mlen, pt, rows_target, flops_total):
    """Time the oracle, as it stands, on the host cores: match + gather over the whole batch,
    attention on a seeded sample of output rows (scaled to the batch by algorithmic flops)."""
    import numpy as np
    import oracle
    threads = min(16, os.cpu_count() or 1)
    t0 = time.perf_counter()
    tree = oracle.OracleTree.from_workload(w)
    t_build = time.perf_counter() - t0
    t0 = time.perf_counter()
    o_mlen, o_pt = tree.match(w.req_off, w.req_tokens, w.req_tenant, max(w.max_blocks, 1))
    t_match = time.perf_counter() - t0
    kpool, vpool = sess.host_pools(o_pt)
    t0 = time.perf_counter()
    oracle.gather(kpool, vpool, o_mlen, o_pt)
    t_gather = time.perf_counter() - t0
    S = np.diff(w.req_off) - o_mlen
    g = np.random.default_rng(1234)
    live = np.flatnonzero(S > 0)
    rr = live[g.integers(0, len(live), rows_target)].astype(np.int32)
    rp = (g.random(rows_target) * S[rr]).astype(np.int32)
    rh = g.integers(0, w.attn.n_q_heads, rows_target).astype(np.int32)
    q_off = np.concatenate([[0], np.cumsum(S)]).astype(np.int32)
    q, kn, vn = (w.suffix_rows(x, o_mlen) for x in "qkv")
    t0 = time.perf_counter()
    want = oracle.attention(q, kn, vn, q_off, kpool, vpool, o_mlen, o_pt, scale=w.attn.scale,
                            rows=(rr, rh, rp), n_threads=threads)
    t_attn = time.perf_counter() - t0
    sample_flops = 4.0 * w.attn.head_dim * float((o_mlen[rr] + rp + 1).sum())
    t_attn_full = t_attn * flops_total / sample_flops
    tokens = float(len(w.req_tokens))
    got = sess.out.double().cpu().numpy()[q_off[rr] + rp, rh]
    err = float(np.abs(got - want).max())
    exact = bool(np.array_equal(o_mlen, mlen) and np.array_equal(o_pt, pt))
    return {"value": tokens / (t_match + t_gather + t_attn_full), "unit": "tokens/s", "cores": threads,
            "kind": "oracle",
            "sample": f"match+gather over all {w.n_req} requests ({t_match * 1e3:.2f} ms + {t_gather * 1e3:.2f} ms, "
                      f"1 thread), fp64 attention on {rows_target} seeded (request, head, row) samples "
                      f"({t_attn:.2f} s on {threads} threads) scaled to the batch by algorithmic flops",
            "lookups_per_s": w.n_req / t_match, "tree_build_s": t_build}, err, exact


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c2", choices=["c1", "c2", "c3", "c4", "c5"])
    ap.add_argument("--hard", action="store_true", help="N(0,1) tensor entries instead of N(0,1)/sqrt(d)")
    ap.add_argument("--cpu-rows", type=int, default=786432, help="oracle attention rows to time (0 = skip)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build measures the path on ONE GPU; --gpus N with N > 1 is not supported "
                 "(no collectives or sharding are part of it)")

    import numpy as np
    import torch
    from paper_2508_08438_amd import inputs
    from paper_2508_08438_amd.pipeline import Session

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    w = inputs.CONFIGS[args.workload](hard=args.hard)
    sess = Session(w, device="cuda:0")
    sess.prepare()
    mlen = sess.host_matched_len.copy()

    for _ in range(args.warmup):
        sess.step()
    torch.cuda.synchronize()
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
        "ms_per_step": elapsed / K * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": a.dtype, "data": "synthetic",
        "config": {"workload": f"{w.name}{'_hard' if args.hard else ''}: {w.n_req} requests, {w.n_tenants} tenants, "
                               f"{int(tokens)} prompt tokens, {int(mlen.sum())} reused, "
                               f"GQA {a.n_q_heads}/{a.n_kv_heads} d={a.head_dim} {a.dtype}",
                   "requests": w.n_req, "prompt_tokens": int(tokens), "reused_tokens": int(mlen.sum()),
                   "reuse_rate": float(mlen.sum()) / tokens},
        "lookups_per_s": w.n_req / t_match,
        "computed_tokens_per_s": (tokens - float(mlen.sum())) / t_attn,
        "stage_ms": {"match": t_match * 1e3, "gather": t_gather * 1e3, "attention": t_attn * 1e3},
        "gather_gbs": gather_bytes / t_gather / 1e9 if mlen.sum() else 0.0,
        "roofline": {"bound": "mfma" if a.dtype == "bf16" else "alu", "kernel": "attn_bf16_kernel"
                     if a.dtype == "bf16" else "attn_f32_kernel", "achieved": achieved, "peak": peak,
                     "unit": "TFLOP/s", "frac": achieved / peak, "traffic": None,
                     "flops_per_launch": flops, "avg_launch_ms": t_attn * 1e3},
    }
    if args.cpu_rows > 0:
        cb, err, exact = cpu_baseline(w, sess, mlen, pt, args.cpu_rows, flops)
        out["cpu_baseline"] = cb
        out["parity"] = {"match_exact": exact, "attention_max_abs_err": err}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
