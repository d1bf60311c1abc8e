"""Pins for the oracle's insert-side steps: promotion (Section 4.2.3) and the write of newly computed KV
blocks into pool pages (Section 4.3.1, Insert).

Promotion is pinned by what it must mean, not by its code: after promoting every sensitive block the
visible match equals the plain longest prefix match of a tenant-blind radix cache (brute force over the
stored sequences), and promoting a subset only ever lengthens matches.  The scatter is pinned by plain
numpy slicing and by being the inverse of the gather."""
import numpy as np
import torch

import oracle
from oracle import OracleTree
from paper_2508_08438_amd import inputs

B = 16


def blind_longest_prefix(w, r):
    """Longest common block prefix of request r with any stored sequence, ignoring visibility."""
    q = w.req_tokens[w.req_off[r]: w.req_off[r + 1]]
    best = 0
    for s in range(len(w.seq_off) - 1):
        t = w.seq_tokens[w.seq_off[s]: w.seq_off[s + 1]]
        n = 0
        while (n + 1) * B <= min(len(q), len(t)) and np.array_equal(q[n * B:(n + 1) * B], t[n * B:(n + 1) * B]):
            n += 1
        best = max(best, n)
    return best * B


def test_promote_all_gives_tenant_blind_match():
    for seed in range(30):
        w = inputs.small_random(seed=seed, n_req=40, p_sens=0.5, n_tenants=4)
        tree = OracleTree.from_workload(w)
        before, _ = tree.match(w.req_off, w.req_tokens, w.req_tenant, max(w.max_blocks, 1), update=False)
        tree.promote(np.arange(w.n_in_blocks))
        after, _ = tree.match(w.req_off, w.req_tokens, w.req_tenant, max(w.max_blocks, 1), update=False)
        want = np.array([blind_longest_prefix(w, r) for r in range(w.n_req)])
        assert np.array_equal(after, want), seed
        assert np.all(after >= before)
        priv, _, _ = tree.block_state()
        assert not np.any(priv == 1)


def test_promote_subset_is_monotone_and_only_touches_listed_blocks():
    hits = 0
    for seed in range(30):
        w = inputs.small_random(seed=seed, n_req=40, p_sens=0.6, n_tenants=4)
        tree = OracleTree.from_workload(w)
        p0, _, _ = tree.block_state()
        m0, _ = tree.match(w.req_off, w.req_tokens, w.req_tenant, max(w.max_blocks, 1), update=False)
        g = np.random.default_rng(seed)
        ids = np.flatnonzero(g.random(w.n_in_blocks) < 0.4)
        tree.promote(ids)
        p1, _, _ = tree.block_state()
        m1, _ = tree.match(w.req_off, w.req_tokens, w.req_tenant, max(w.max_blocks, 1), update=False)
        listed = np.zeros(w.n_in_blocks, bool)
        listed[ids] = True
        assert np.array_equal(p1[~listed], p0[~listed])            # nothing else changes
        assert np.all(p1[listed & (p0 != 255)] == 0)               # listed entries become shareable
        assert np.array_equal(p1 == 255, p0 == 255)                # blocks that created no entry stay that way
        assert np.all(m1 >= m0)
        hits += int((m1 > m0).sum())
    assert hits > 20                                               # the cases do exercise the change


def test_promote_ignores_empty_list():
    w = inputs.small_random(seed=3, n_req=10, p_sens=0.5)
    tree = OracleTree.from_workload(w)
    p0, _, _ = tree.block_state()
    tree.promote(np.zeros(0, np.int64))
    assert np.array_equal(tree.block_state()[0], p0)


def scatter_case(seed, R=7, H=2, d=8, n_pages=128, dtype=torch.float32):
    g = np.random.default_rng(seed)
    S = g.integers(0, 200, R)
    S[0] = 0
    S[1] = 15
    S[2] = 32
    q_off = np.concatenate([[0], np.cumsum(S)]).astype(np.int32)
    T = int(q_off[-1])
    knew = torch.from_numpy(g.standard_normal((T, H, d))).to(dtype)
    vnew = torch.from_numpy(g.standard_normal((T, H, d))).to(dtype)
    mb = int(max(S) // B) + 1                                       # one column more than any request fills
    perm = g.permutation(n_pages)
    new_pages = np.full((R, mb), -1, np.int32)
    k = 0
    for r in range(R):
        for j in range(mb):
            if g.random() < 0.85:                                   # some slots stay unallocated
                new_pages[r, j] = perm[k]
                k += 1
    kpool = torch.from_numpy(g.standard_normal((n_pages, B, H, d))).to(dtype)
    vpool = torch.from_numpy(g.standard_normal((n_pages, B, H, d))).to(dtype)
    return q_off, knew, vnew, new_pages, kpool, vpool


def test_scatter_matches_plain_slicing_and_leaves_other_pages_alone():
    for seed in range(10):
        for dtype in (torch.float32, torch.bfloat16):
            q_off, knew, vnew, new_pages, kpool, vpool = scatter_case(seed, dtype=dtype)
            k0, v0 = kpool.clone(), vpool.clone()
            oracle.scatter(knew, vnew, q_off, new_pages, kpool, vpool)
            touched = set()
            for r in range(len(q_off) - 1):
                for j in range((q_off[r + 1] - q_off[r]) // B):
                    p = new_pages[r, j]
                    if p < 0:
                        continue
                    lo = q_off[r] + j * B
                    assert torch.equal(kpool[p], knew[lo:lo + B]) and torch.equal(vpool[p], vnew[lo:lo + B])
                    touched.add(int(p))
            rest = [p for p in range(kpool.shape[0]) if p not in touched]
            assert torch.equal(kpool[rest], k0[rest]) and torch.equal(vpool[rest], v0[rest])
            assert len(touched) > 3


def test_gather_of_scattered_pages_returns_the_rows():
    q_off, knew, vnew, new_pages, kpool, vpool = scatter_case(11)
    # give every full block a page so that the round trip covers all of them
    R, mb = new_pages.shape
    new_pages = np.arange(R * mb, dtype=np.int32).reshape(R, mb)
    kpool = torch.zeros(R * mb, B, 2, 8)
    vpool = torch.zeros(R * mb, B, 2, 8)
    oracle.scatter(knew, vnew, q_off, new_pages, kpool, vpool)
    full = ((np.diff(q_off) // B) * B).astype(np.int32)
    kctx, vctx = oracle.gather(kpool, vpool, full, new_pages)
    ctx_off = np.concatenate([[0], np.cumsum(full)])
    for r in range(R):
        assert torch.equal(kctx[ctx_off[r]: ctx_off[r + 1]], knew[q_off[r]: q_off[r] + full[r]])
        assert torch.equal(vctx[ctx_off[r]: ctx_off[r + 1]], vnew[q_off[r]: q_off[r] + full[r]])
