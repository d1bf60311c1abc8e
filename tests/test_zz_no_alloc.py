"""skv_prefill_attn_static, the entry point that allocates nothing (work list and zero page in a device array
built into the library), against skv_prefill_attn with a caller workspace: two calls in a row on the shared
scratch, the second on a smaller batch, each bit-identical to the workspace variant and in tolerance against
the fp64 oracle.  Collected last (file name) so that a failure here hides no other test."""
import numpy as np
import pytest
import torch

import oracle
from paper_2508_08438_amd.inputs import BLOCK as B

pytestmark = pytest.mark.gpu


def _case(seed, Hq, Hkv, S_list, k_list, n_pages=96):
    g = np.random.default_rng(seed)
    R = len(S_list)
    S, k = np.asarray(S_list), np.asarray(k_list)
    mb = int(k.max()) + 1
    perm = g.permutation(n_pages)
    pt = np.full((R, mb), -1, np.int32)
    used = 0
    for r in range(R):
        pt[r, : k[r]] = perm[used: used + k[r]]
        used += k[r]
    q_off = np.concatenate([[0], np.cumsum(S)]).astype(np.int32)
    T = int(q_off[-1])
    t = lambda *s: torch.from_numpy(g.standard_normal(s).astype(np.float32)).to(torch.bfloat16)
    return dict(q=t(T, Hq, 128), knew=t(T, Hkv, 128), vnew=t(T, Hkv, 128), q_off=q_off,
                kpool=t(n_pages, B, Hkv, 128), vpool=t(n_pages, B, Hkv, 128),
                matched_len=(k * B).astype(np.int32), page_table=pt)


def _run(c, static):
    from paper_2508_08438_amd import binding as skv
    dev = "cuda:0"
    d = {k: (torch.from_numpy(v) if isinstance(v, np.ndarray) else v).to(dev) for k, v in c.items()}
    q = d["q"]
    desc = skv.attn_desc(q.shape[1], d["kpool"].shape[2], 128, torch.bfloat16)
    out = torch.full_like(q, 7.0)
    R = len(c["matched_len"])
    args = (desc, q, d["knew"], d["vnew"], d["q_off"], d["kpool"], d["vpool"], d["matched_len"], d["page_table"],
            d["page_table"].shape[1], out)
    if static:
        skv.skv_prefill_attn_static(*args)
    else:
        ws = torch.zeros(skv.skv_prefill_attn_workspace_size(desc, R, q.shape[0]), dtype=torch.uint8, device=dev)
        skv.skv_prefill_attn(*args, ws)
    torch.cuda.synchronize()
    return out


def test_static_scratch_entry_point_two_calls_second_smaller():
    big = _case(11, 8, 2, [300, 65, 1, 0, 130, 64], [5, 0, 9, 3, 2, 7])
    small = _case(12, 8, 2, [70, 33], [1, 4])
    for label, c in (("first call", big), ("second, smaller call", small)):
        print(f"[static scratch] {label}: S={np.diff(c['q_off']).tolist()}", flush=True)
        got = _run(c, static=True)
        ref = _run(c, static=False)
        assert torch.equal(got, ref), label       # same kernels, same work list: identical bits
        want = oracle.attention(**c, n_threads=8)
        err = np.abs(got.double().cpu().numpy()[: want.shape[0]] - want).max()
        print(f"   max-abs err vs oracle {err:.3e}", flush=True)
        assert err <= 2e-2, (label, err)
