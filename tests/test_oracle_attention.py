"""Pins for the oracle's fp64 attention and page gather (CPU only).

Closed forms, degenerate cases, a library cross-check with an explicit mask, and the
identity that KV reuse only avoids recomputation (Section 2.1): attention of the uncached
suffix over reused prefix KV equals the corresponding rows of full causal attention.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2508_08438_amd import inputs

B = 16


def make_case(seed, R=3, Hq=4, Hkv=2, d=8, n_pages=40, max_blocks=6, dtype=torch.float32, sigma=1.0):
    g = np.random.default_rng(seed)
    k_blocks = g.integers(0, max_blocks + 1, R)
    S = g.integers(0, 40, R)
    S[0] = max(S[0], 20)
    perm = g.permutation(n_pages)
    pt = np.full((R, max_blocks), -1, np.int32)
    used = 0
    for r in range(R):
        pt[r, : k_blocks[r]] = perm[used: used + k_blocks[r]]
        used += k_blocks[r]
    q_off = np.concatenate([[0], np.cumsum(S)]).astype(np.int32)
    T = int(q_off[-1])
    t = lambda *s: torch.from_numpy(g.standard_normal(s) * sigma).to(dtype)
    return dict(q=t(T, Hq, d), knew=t(T, Hkv, d), vnew=t(T, Hkv, d), q_off=q_off,
                kpool=t(n_pages, B, Hkv, d), vpool=t(n_pages, B, Hkv, d),
                matched_len=(k_blocks * B).astype(np.int32), page_table=pt)


def assemble_kv(c, r, hk):
    """Prefix K/V of request r for kv head hk, gathered by hand through the page table."""
    k = c["matched_len"][r] // B
    pages = c["page_table"][r, :k]
    lo, hi = c["q_off"][r], c["q_off"][r + 1]
    K = torch.cat([c["kpool"][pages][:, :, hk].reshape(-1, c["kpool"].shape[-1]), c["knew"][lo:hi, hk]])
    V = torch.cat([c["vpool"][pages][:, :, hk].reshape(-1, c["vpool"].shape[-1]), c["vnew"][lo:hi, hk]])
    return K.double(), V.double()


def test_pa1_constant_values_give_constant_output():
    c = make_case(1)
    c["vpool"].fill_(1.0); c["vnew"].fill_(1.0)
    out = oracle.attention(**c)
    assert np.allclose(out, 1.0, atol=1e-14)


def test_pa2_zero_keys_average_the_positions():
    """K == 0 makes the softmax uniform; with V[j] = absolute position j the output row i is the
    mean of 0..L+i = (L+i)/2.  Pins the prefix/new boundary and the causal off-by-one."""
    c = make_case(2)
    c["kpool"].zero_(); c["knew"].zero_()
    for r in range(len(c["matched_len"])):
        L = int(c["matched_len"][r])
        for j in range(L):
            c["vpool"][c["page_table"][r, j // B], j % B] = float(j)
        for i in range(c["q_off"][r + 1] - c["q_off"][r]):
            c["vnew"][c["q_off"][r] + i] = float(L + i)
    out = oracle.attention(**c)
    for r in range(len(c["matched_len"])):
        L = int(c["matched_len"][r])
        for i in range(c["q_off"][r + 1] - c["q_off"][r]):
            assert np.allclose(out[c["q_off"][r] + i], (L + i) / 2.0, atol=1e-12)


def test_pa3_degenerate_cases():
    # no prefix, one query: the output is that token's own value row
    c = make_case(3, R=1, max_blocks=2)
    c["matched_len"][:] = 0; c["page_table"][:] = -1
    out = oracle.attention(**c)
    G = c["q"].shape[1] // c["knew"].shape[1]
    for h in range(c["q"].shape[1]):
        assert np.allclose(out[0, h], c["vnew"][0, h // G].double().numpy(), atol=1e-14)
    # one dominant logit: the output tends to that key's value row
    c = make_case(4, R=1, Hq=2, Hkv=2)
    c["matched_len"][:] = 2 * B
    c["page_table"][0, :2] = [7, 3]
    j_star = 21  # second page, slot 5
    qv = c["q"][-1, 0]
    c["kpool"][3, 5, 0] = 100.0 * qv / qv.norm()
    out = oracle.attention(**c)
    assert np.allclose(out[-1, 0], c["vpool"][3, 5, 0].double().numpy(), atol=1e-9)
    assert j_star // B == 1 and j_star % B == 5
    # an empty suffix writes nothing and is legal
    c = make_case(5, R=2)
    c["q_off"] = np.array([0, 0, c["q_off"][2] - c["q_off"][1]], np.int32)
    n = int(c["q_off"][-1])
    c["q"], c["knew"], c["vnew"] = c["q"][:n], c["knew"][:n], c["vnew"][:n]
    assert oracle.attention(**c).shape[0] == n


@pytest.mark.parametrize("dtype,Hq,Hkv,d", [(torch.float32, 4, 2, 8), (torch.bfloat16, 8, 2, 16),
                                            (torch.float32, 3, 3, 5)])
def test_pa4_library_attention_with_explicit_mask(dtype, Hq, Hkv, d):
    c = make_case(6, Hq=Hq, Hkv=Hkv, d=d, dtype=dtype)
    out = oracle.attention(**c, n_threads=3)
    G = Hq // Hkv
    for r in range(len(c["matched_len"])):
        lo, hi = int(c["q_off"][r]), int(c["q_off"][r + 1])
        S, L = hi - lo, int(c["matched_len"][r])
        if S == 0:
            continue
        mask = torch.zeros(S, L + S, dtype=torch.bool)
        for i in range(S):
            mask[i, : L + i + 1] = True
        for h in range(Hq):
            K, V = assemble_kv(c, r, h // G)
            want = torch.nn.functional.scaled_dot_product_attention(
                c["q"][lo:hi, h].double()[None], K[None], V[None], attn_mask=mask[None])[0]
            assert np.allclose(out[lo:hi, h], want.numpy(), atol=1e-12)


def test_pa4_sampled_rows_equal_full_rows_and_scale_is_used():
    c = make_case(7)
    full = oracle.attention(**c)
    rows = ([0, 0, 2, 1], [3, 0, 1, 2], [0, c["q_off"][1] - 1, 0, 1])
    rows = tuple(np.asarray(x) for x in rows)
    keep = [i for i in range(4) if rows[2][i] < c["q_off"][rows[0][i] + 1] - c["q_off"][rows[0][i]]]
    rows = tuple(x[keep] for x in rows)
    got = oracle.attention(**c, rows=rows)
    for n, (r, h, i) in enumerate(zip(*rows)):
        assert np.array_equal(got[n], full[c["q_off"][r] + i, h])
    other = oracle.attention(**c, scale=0.5)
    assert not np.allclose(other, full)


def test_pa5_reuse_equals_recompute():
    """Rows [L, N) of full causal attention over all N tokens (nothing cached) equal attention of
    the suffix over the cached prefix (Section 2.1: caching only avoids recomputation)."""
    g = np.random.default_rng(8)
    Hq, Hkv, d, N, L = 4, 2, 8, 75, 48
    Q = torch.from_numpy(g.standard_normal((N, Hq, d))).float()
    K = torch.from_numpy(g.standard_normal((N, Hkv, d))).float()
    V = torch.from_numpy(g.standard_normal((N, Hkv, d))).float()
    pt0 = np.full((1, 3), -1, np.int32)
    empty = torch.zeros(4, B, Hkv, d)
    full = oracle.attention(Q, K, V, [0, N], empty, empty, [0], pt0)
    kpool, vpool = torch.zeros(4, B, Hkv, d), torch.zeros(4, B, Hkv, d)
    pages = [2, 0, 3]
    for j, p in enumerate(pages):
        kpool[p] = K[j * B: (j + 1) * B]
        vpool[p] = V[j * B: (j + 1) * B]
    reuse = oracle.attention(Q[L:], K[L:], V[L:], [0, N - L], kpool, vpool, [L],
                             np.array([pages], np.int32))
    assert np.allclose(reuse, full[L:], atol=1e-13)


def test_pg1_gather_is_a_byte_exact_page_copy_and_physical_ids_do_not_matter():
    c = make_case(9, dtype=torch.bfloat16)
    kctx, vctx = oracle.gather(c["kpool"], c["vpool"], c["matched_len"], c["page_table"])
    o = 0
    for r in range(len(c["matched_len"])):
        for j in range(c["matched_len"][r] // B):
            p = c["page_table"][r, j]
            assert torch.equal(kctx[o: o + B].view(torch.int16), c["kpool"][p].view(torch.int16))
            assert torch.equal(vctx[o: o + B].view(torch.int16), c["vpool"][p].view(torch.int16))
            o += B
    assert o == kctx.shape[0]
    # relabel the physical pages: same logical content, different ids -> same attention
    out = oracle.attention(**c)
    perm = np.random.default_rng(0).permutation(c["kpool"].shape[0])
    inv = np.argsort(perm)
    c2 = dict(c)
    c2["kpool"], c2["vpool"] = c["kpool"][perm], c["vpool"][perm]
    c2["page_table"] = np.where(c["page_table"] >= 0, inv[np.maximum(c["page_table"], 0)], -1).astype(np.int32)
    assert np.array_equal(oracle.attention(**c2), out)


def test_synthetic_values_are_device_independent_functions_of_the_index():
    w = inputs.config2()
    a = w.pool_pages("k", 5, 9)
    b = torch.cat([w.pool_pages("k", 5, 7), w.pool_pages("k", 7, 9)])
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))
    assert not torch.equal(w.pool_pages("v", 5, 9).view(torch.int16), a.view(torch.int16))
    x = a.float() * 128 ** 0.5
    assert abs(float(x.mean())) < 0.02 and abs(float(x.std()) - 1) < 0.02
    w = inputs.config1()
    ml = np.zeros(w.n_req, np.int32); ml[0] = 32
    q = w.suffix_rows("q", ml)
    assert q.shape == (len(w.req_tokens) - 32, 8, 64)
    assert torch.equal(q[0], w.token_rows("q", 32, 33)[0])
