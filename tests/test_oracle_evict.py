"""Pins for the oracle's eviction (Section 4.3.1 Evict: epoch-based LRU with protected entries; Section
4.3.2: leaf-to-root, block-by-block reclamation of compressed chains).

The paper fixes neither the tie-break nor what "in use" means; the reading taken is in the oracle's header
and the *choice* of that reading is unpinned.  What is pinned is that the oracle carries it out: the evicted
sequence is recomputed from a dictionary of whole block-prefixes (no tree, no nodes), lookups afterwards
agree with that dictionary, entries with descendants or under protection never go, and evicting everything
returns every page exactly once."""
import numpy as np

from oracle import OracleTree
from paper_2508_08438_amd import inputs
from test_oracle_insert import make_round, prefix_table, table_insert, table_match

B = 16


def table_stamp(table, x, tenant, epoch):
    for k in range(len(x) // B):
        e = table.get(x[: (k + 1) * B].tobytes())
        if e is None or (e[0] and e[1] != tenant):
            break
        e[4] = epoch


def table_evict(table, n_want, protect):
    """Oldest (epoch, id) among the prefixes no other prefix extends, protected ones left alone."""
    out = []
    for _ in range(n_want):
        has_child = set(k[:-B * 4] for k in table if len(k) > B * 4)
        cand = [(e[4], e[3], k) for k, e in table.items() if k not in has_child and e[3] not in protect]
        if not cand:
            break
        _, _, key = min(cand)
        e = table.pop(key)
        out.append((e[3], e[2]))
    return out


def stream_with_eviction(seed, n_rounds=5, n_req=10):
    block_vocab = 3 if seed % 3 == 0 else None
    w = inputs.small_random(seed=seed, n_req=8, p_sens=0.4, n_tenants=3, block_vocab=block_vocab)
    vocab = int(w.seq_tokens.max()) + 1 if len(w.seq_tokens) else 2
    tree = OracleTree.from_workload(w)
    table = prefix_table(w)
    for e in table.values():
        e.append(0)                                         # epoch of the initial content
    g = np.random.default_rng(2000 + seed)
    next_page, next_id = w.n_pages, w.n_in_blocks
    earlier = [w.req_tokens[w.req_off[r]: w.req_off[r + 1]] for r in range(w.n_req)]
    evicted_total = 0
    all_pages_back = []
    for rnd in range(n_rounds):
        epoch = rnd + 1
        tree.set_epoch(epoch)
        reqs, off, toks, tenants = make_round(g, earlier, vocab, w.n_tenants, n_req, block_vocab)
        mb = max(max(len(x) // B for x in reqs), 1)
        mlen, pt, ids = tree.match(off, toks, tenants, mb, want_ids=True)
        for r, x in enumerate(reqs):
            table_stamp(table, x, int(tenants[r]), epoch)
        new_pages = np.full((n_req, mb + 1), -1, np.int32)
        for r, x in enumerate(reqs):
            n_suffix = len(x) // B - mlen[r] // B
            new_pages[r, :n_suffix] = np.arange(next_page, next_page + n_suffix)
            next_page += n_suffix
        tree.insert(off, toks, tenants, mlen, new_pages)
        for r, x in enumerate(reqs):
            before = set(table)
            _, _, next_id = table_insert(table, x, int(tenants[r]), int(mlen[r]) // B, new_pages[r], next_id)
            for k in set(table) - before:
                table[k].append(epoch)
        # epochs agree entry by entry
        ep = tree.epochs()
        for e in table.values():
            assert ep[e[3]] == e[4], (seed, rnd)
        # evict a random amount under a random protection set (the blocks the last batch matched, thinned)
        protect = set(int(i) for i in ids[ids >= 0][:: int(g.integers(1, 4))])
        n_want = int(g.integers(0, max(len(table) // 3, 1) + 1))
        got_ids, got_pages = tree.evict(n_want, sorted(protect))
        want = table_evict(table, n_want, protect)
        assert [(int(a), int(b)) for a, b in zip(got_ids, got_pages)] == want, (seed, rnd)
        assert not (set(int(i) for i in got_ids) & protect)
        assert tree.n_blocks == len(table)
        evicted_total += len(want)
        all_pages_back += [p for _, p in want]
        earlier += reqs
        for t in range(w.n_tenants):                       # lookups after eviction
            sample = [earlier[i] for i in g.choice(len(earlier), min(20, len(earlier)), replace=False)]
            o = np.concatenate([[0], np.cumsum([len(x) for x in sample])]).astype(np.int32)
            tk = np.concatenate(sample + [np.zeros(0, np.int32)]).astype(np.int32)
            mb2 = max(max(len(x) // B for x in sample), 1)
            ml2, pt2 = tree.match(o, tk, np.full(len(sample), t, np.int32), mb2, update=False)
            for r, x in enumerate(sample):
                pages, _ = table_match(table, x, t)
                assert ml2[r] == len(pages) * B and list(pt2[r, : len(pages)]) == pages, (seed, rnd, t, r)
    assert len(set(all_pages_back)) == len(all_pages_back)   # no page is handed back twice
    return evicted_total


def test_eviction_sequence_matches_prefix_dictionary():
    total = sum(stream_with_eviction(seed) for seed in range(40))
    assert total > 800


def test_evict_everything_returns_every_page_once():
    for seed in range(10):
        w = inputs.small_random(seed=seed, n_req=8, p_sens=0.3)
        tree = OracleTree.from_workload(w)
        n = tree.n_blocks
        _, pt, ids = tree.match(w.req_off, w.req_tokens, w.req_tenant, max(w.max_blocks, 1), want_ids=True)
        got_ids, got_pages = tree.evict(10 ** 9)
        assert len(got_ids) == n and tree.n_blocks == 0
        canon = set(int(e[2]) for e in prefix_table(w).values())
        assert sorted(int(p) for p in got_pages) == sorted(canon)
        ml, _ = tree.match(w.req_off, w.req_tokens, w.req_tenant, max(w.max_blocks, 1), update=False)
        assert not ml.any()


def test_recently_used_paths_survive_and_tails_go_first():
    # one chain of 6 blocks; a request reuses its first 3 blocks at epoch 5: the 3 stale tail blocks go first,
    # far end first, and the chain's head is the very last entry to leave
    tok = np.arange(6 * B, dtype=np.int32)
    tree = OracleTree(tok, np.array([0, 6 * B]), np.zeros(6, np.uint8), np.zeros(6, np.int32), np.arange(6, dtype=np.int32))
    tree.set_epoch(5)
    ml, _ = tree.match(np.array([0, 3 * B], np.int32), tok[: 3 * B], np.array([0], np.int32), 3)
    assert ml[0] == 3 * B
    ids, pages = tree.evict(4)
    assert list(ids) == [5, 4, 3, 2]
    ids, _ = tree.evict(10, protect_ids=[1])
    assert len(ids) == 0                                   # block 1 is in use: neither it nor its ancestor can go
    ids, _ = tree.evict(10)
    assert list(ids) == [1, 0]
