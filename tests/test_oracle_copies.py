"""Pins for per-tenant copies of the same content (Section 4.1: selective isolation leaves redundant copies;
Section 4.3.1: the visibility rule is checked at every hop).

With private copies a tree position can hold several children that start with the same block, and the lookup has
to follow every visible one.  The oracle's search, insert and eviction on such trees are pinned against a model
without any tree machinery: a flat list of block entries with parent links, searched by plain recursion."""
import numpy as np

from oracle import OracleTree
from paper_2508_08438_amd import inputs
from test_oracle_insert import make_round

B = 16


class EntryModel:
    def __init__(self, w):
        self.e = []                      # dicts: parent, tok, private, owner, page, id, epoch
        self.kids = {}                   # (parent index, token bytes) -> entry indices in creation order
        self.branch_points = 0
        for s in range(len(w.seq_off) - 1):
            lo, hi = int(w.seq_off[s]), int(w.seq_off[s + 1])
            par = -1
            for j in range((hi - lo) // B):
                tok = w.seq_tokens[lo + j * B: lo + (j + 1) * B].tobytes()
                have = self.kids.get((par, tok))
                if have:
                    par = have[0]        # first insertion wins
                    continue
                b = lo // B + j
                par = self._add(par, tok, bool(w.blk_sensitive[b]), int(w.blk_owner[b]), int(w.blk_page[b]), b, 0)

    def _add(self, parent, tok, private, owner, page, bid, epoch):
        self.e.append(dict(parent=parent, tok=tok, private=private, owner=owner, page=page, id=bid, epoch=epoch,
                           alive=True))
        self.kids.setdefault((parent, tok), []).append(len(self.e) - 1)
        return len(self.e) - 1

    def search(self, x, tenant):
        nb = len(x) // B
        best = []

        def go(parent, j, cur):
            nonlocal best
            if len(cur) > len(best):
                best = list(cur)
            if j == nb:
                return
            vis = [i for i in self.kids.get((parent, x[j * B:(j + 1) * B].tobytes()), [])
                   if self.e[i]["alive"] and not (self.e[i]["private"] and self.e[i]["owner"] != tenant)]
            if len(vis) > 1:
                self.branch_points += 1
            for i in vis:                # creation order = ascending id
                cur.append(i)
                go(i, j + 1, cur)
                cur.pop()
                if len(best) == nb:
                    return
        go(-1, 0, [])
        return best

    def insert_copy(self, x, tenant, k_vis, pages_row, next_id, epoch):
        have = 0
        while have < len(pages_row) and pages_row[have] >= 0:
            have += 1
        nb = min(len(x) // B, k_vis + have)
        path = self.search(x[: nb * B], tenant)
        k = len(path)
        if k >= nb or k < k_vis:
            return k, 0, next_id
        par = path[-1] if path else -1
        for j in range(k, nb):
            par = self._add(par, x[j * B:(j + 1) * B].tobytes(), True, tenant, int(pages_row[j - k_vis]), next_id, epoch)
            next_id += 1
        return k, nb - k, next_id

    def evict(self, n_want, protect):
        out = []
        for _ in range(n_want):
            parents = set(e["parent"] for e in self.e if e["alive"])
            cand = [(e["epoch"], e["id"], i) for i, e in enumerate(self.e)
                    if e["alive"] and i not in parents and e["id"] not in protect]
            if not cand:
                break
            _, _, i = min(cand)
            self.e[i]["alive"] = False
            out.append((self.e[i]["id"], self.e[i]["page"]))
        return out

    def n_alive(self):
        return sum(e["alive"] for e in self.e)


def compare_lookups(tree, model, reqs, tenants_all, g, stamp_epoch=None):
    for t in tenants_all:
        sample = [reqs[i] for i in g.choice(len(reqs), min(20, len(reqs)), replace=False)]
        off = np.concatenate([[0], np.cumsum([len(x) for x in sample])]).astype(np.int32)
        tk = np.concatenate(sample + [np.zeros(0, np.int32)]).astype(np.int32)
        mb = max(max(len(x) // B for x in sample), 1)
        ml, pt, ids = tree.match(off, tk, np.full(len(sample), t, np.int32), mb, update=False, want_ids=True)
        for r, x in enumerate(sample):
            path = model.search(x, t)
            assert ml[r] == len(path) * B, (t, r)
            assert list(pt[r, : len(path)]) == [model.e[i]["page"] for i in path]
            assert list(ids[r, : len(path)]) == [model.e[i]["id"] for i in path]


def run_copy_stream(seed, n_rounds=5, n_req=10, with_evict=True):
    block_vocab = 3 if seed % 3 == 0 else None
    w = inputs.small_random(seed=seed, n_req=8, p_sens=0.4, n_tenants=3, block_vocab=block_vocab)
    vocab = int(w.seq_tokens.max()) + 1 if len(w.seq_tokens) else 2
    tree = OracleTree.from_workload(w)
    model = EntryModel(w)
    g = np.random.default_rng(3000 + seed)
    next_page, next_id = w.n_pages, w.n_in_blocks
    earlier = [w.req_tokens[w.req_off[r]: w.req_off[r + 1]] for r in range(w.n_req)]
    inserted = evicted = 0
    for rnd in range(n_rounds):
        epoch = rnd + 1
        tree.set_epoch(epoch)
        reqs, off, toks, tenants = make_round(g, earlier, vocab, w.n_tenants, n_req, block_vocab)
        mb = max(max(len(x) // B for x in reqs), 1)
        mlen, pt, ids = tree.match(off, toks, tenants, mb, want_ids=True)
        for r, x in enumerate(reqs):
            path = model.search(x, int(tenants[r]))
            assert mlen[r] == len(path) * B and list(ids[r, : len(path)]) == [model.e[i]["id"] for i in path]
            for i in path:
                model.e[i]["epoch"] = epoch
        new_pages = np.full((n_req, mb + 1), -1, np.int32)
        for r, x in enumerate(reqs):
            n_suffix = len(x) // B - mlen[r] // B
            new_pages[r, :n_suffix] = np.arange(next_page, next_page + n_suffix)
            next_page += n_suffix
        first, n = tree.insert(off, toks, tenants, mlen, new_pages, private_copies=True)
        for r, x in enumerate(reqs):
            f, k, next_id = model.insert_copy(x, int(tenants[r]), int(mlen[r]) // B, new_pages[r], next_id, epoch)
            assert (first[r], n[r]) == (f, k), (seed, rnd, r)
            inserted += k
        assert tree.n_in_blocks == next_id and tree.n_blocks == model.n_alive()
        # the verifier clears a random third of everything cached so far: public copies appear next to private ones
        alive_ids = np.array([e["id"] for e in model.e if e["alive"]])
        pick = alive_ids[g.random(len(alive_ids)) < 0.3]
        tree.promote(pick)
        for e in model.e:
            if e["id"] in set(pick.tolist()):
                e["private"] = False
        earlier += reqs
        compare_lookups(tree, model, earlier, range(w.n_tenants), g)
        if with_evict and rnd % 2 == 1:
            protect = set(int(i) for i in ids[ids >= 0][::3])
            n_want = int(g.integers(0, model.n_alive() // 4 + 1))
            got_ids, got_pages = tree.evict(n_want, sorted(protect))
            want = model.evict(n_want, protect)
            assert [(int(a), int(b)) for a, b in zip(got_ids, got_pages)] == want, (seed, rnd)
            evicted += len(want)
            compare_lookups(tree, model, earlier, range(w.n_tenants), g)
        ep = tree.epochs()
        for e in model.e:
            if e["alive"]:
                assert ep[e["id"]] == e["epoch"]
    return inserted, evicted, model.branch_points


def test_copy_streams_match_the_entry_list_model():
    tot = np.zeros(3, np.int64)
    for seed in range(40):
        tot += np.array(run_copy_stream(seed))
    assert tot[0] > 1500 and tot[1] > 300
    assert tot[2] > 200                      # lookups did meet positions with several visible copies


def _blocks(*ids):
    return np.concatenate([np.full(B, i, np.int32) for i in ids])


def test_lookup_backtracks_to_the_longer_copy():
    # tenant 0 caches X (private); tenant 1 cannot see it and adds its own X' followed by Z.  Once X is public,
    # tenant 1 sees two copies of X: the older one (X, nothing below it for tenant 1) and its own (X' -> Z).
    X, Y, Z = 1, 2, 3
    tree = OracleTree(_blocks(X, Y), np.array([0, 2 * B]), np.ones(2, np.uint8), np.zeros(2, np.int32),
                      np.array([10, 11], np.int32))
    req = _blocks(X, Z)
    off = np.array([0, 2 * B], np.int32)
    t1 = np.array([1], np.int32)
    ml, _ = tree.match(off, req, t1, 2)
    assert ml[0] == 0
    first, n = tree.insert(off, req, t1, ml, np.array([[20, 21]], np.int32), private_copies=True)
    assert (first[0], n[0]) == (0, 2) and tree.n_blocks == 4
    tree.promote([0])                                           # tenant 0's X becomes public
    ml, pt, ids = tree.match(off, req, t1, 2, want_ids=True)
    assert ml[0] == 2 * B and list(pt[0]) == [20, 21] and list(ids[0]) == [2, 3]    # via its own copy
    ml, pt = tree.match(np.array([0, 2 * B], np.int32), _blocks(X, Y), t1, 2)
    assert ml[0] == B and pt[0, 0] == 10                        # X via the older public copy; Y is still tenant 0's
    tree.promote([1])
    ml, pt = tree.match(np.array([0, 2 * B], np.int32), _blocks(X, Y), t1, 2)
    assert ml[0] == 2 * B and list(pt[0]) == [10, 11]
    # a third tenant sees only the public copy, and nothing of what hangs below tenant 1's private one
    ml, pt = tree.match(off, req, np.array([2], np.int32), 2)
    assert ml[0] == B and pt[0, 0] == 10


def test_copy_inside_a_compressed_edge_splits_it():
    # tenant 0 caches A B C D as one edge with C private; tenant 1 is stopped at C and adds its own C D'
    tree = OracleTree(_blocks(1, 2, 3, 4), np.array([0, 4 * B]), np.array([0, 0, 1, 0], np.uint8),
                      np.zeros(4, np.int32), np.arange(4, dtype=np.int32))
    req = _blocks(1, 2, 3, 9)
    off = np.array([0, 4 * B], np.int32)
    t1 = np.array([1], np.int32)
    ml, _ = tree.match(off, req, t1, 4)
    assert ml[0] == 2 * B
    first, n = tree.insert(off, req, t1, ml, np.array([[30, 31]], np.int32), private_copies=True)
    assert (first[0], n[0]) == (2, 2)
    ml, pt = tree.match(off, req, t1, 4)
    assert ml[0] == 4 * B and list(pt[0]) == [0, 1, 30, 31]
    ml, pt = tree.match(off, _blocks(1, 2, 3, 4), np.array([0], np.int32), 4)    # the creator's own path is intact
    assert ml[0] == 4 * B and list(pt[0]) == [0, 1, 2, 3]
