"""Pins for the oracle's safeguard step (window roll, RDR predicate, demotion; Sections 4.2.2 and 6).

The paper gives no threshold and states the trigger direction both ways, so the predicate is a parameter
and which direction is right stays unpinned.  What is pinned here is the mechanics for a given parameter
set: an independent recomputation from the counters with Python integers / fractions, the window-roll
bookkeeping, and the security property that a demoted block stops giving cross-tenant hits."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import OracleTree
from paper_2508_08438_amd import inputs

B = 16


def recompute(priv, hit, ucnt, u_pre, streak, direction, tau, min_hits, n_consec, u_pre_max):
    """Independent statement of the step with exact fractions; arrays are per input block id."""
    priv, streak = priv.copy(), streak.copy()
    demoted = 0
    for b in range(len(priv)):
        if priv[b] == 255:
            continue
        pred = False
        if hit[b] > 0 and hit[b] >= min_hits:
            rdr = Fraction(int(ucnt[b]), int(hit[b]))
            pred = rdr < Fraction(*tau) if direction == 0 else (rdr > Fraction(*tau) and u_pre[b] <= u_pre_max)
        streak[b] = streak[b] + 1 if pred else 0
        if priv[b] == 0 and streak[b] >= n_consec:
            priv[b], streak[b] = 1, 0
            demoted += 1
    return priv, streak, demoted


PARAMS = [dict(direction=0, tau=(1, 2), min_hits=1, n_consec=1, u_pre_max=1),
          dict(direction=0, tau=(2, 3), min_hits=3, n_consec=2, u_pre_max=1),
          dict(direction=1, tau=(1, 2), min_hits=2, n_consec=1, u_pre_max=1),
          dict(direction=1, tau=(1, 3), min_hits=1, n_consec=2, u_pre_max=2),
          dict(direction=0, tau=(1, 1), min_hits=1, n_consec=3, u_pre_max=0)]


@pytest.mark.parametrize("pi", range(len(PARAMS)))
def test_window_roll_matches_independent_recomputation(pi):
    kw = PARAMS[pi]
    for seed in range(25):
        w = inputs.small_random(seed=seed, n_req=60, p_sens=0.3, n_tenants=3)
        tree = OracleTree.from_workload(w)
        streak = np.zeros(w.n_in_blocks, np.int64)
        g = np.random.default_rng(seed)
        for window in range(4):
            # a different request mix per window: a random subset, tenants re-drawn
            pick = g.random(w.n_req) < 0.7
            off = np.concatenate([[0], np.cumsum(np.where(pick, np.diff(w.req_off), 0))]).astype(np.int32)
            toks = np.concatenate([w.req_tokens[w.req_off[r]: w.req_off[r + 1]] for r in range(w.n_req) if pick[r]]
                                  + [np.zeros(0, np.int32)]).astype(np.int32)
            off = np.concatenate([[0], np.cumsum(np.diff(w.req_off)[pick])]).astype(np.int32)
            ten = g.integers(0, w.n_tenants, int(pick.sum())).astype(np.int32)
            tree.match(off, toks, ten, max(w.max_blocks, 1))
            hit, ucnt = tree.counters()
            priv, hit_pre, u_pre = tree.block_state()
            want_priv, streak, want_n = recompute(priv, hit, ucnt, u_pre, streak, **kw)
            got_n = tree.window_roll(**kw)
            priv2, hit_pre2, u_pre2 = tree.block_state()
            assert got_n == want_n and np.array_equal(priv2, want_priv), (seed, window)
            assert np.array_equal(hit_pre2, hit) and np.array_equal(u_pre2, ucnt)  # the window rolled
            h0, u0 = tree.counters()
            assert h0.sum() == 0 and u0.sum() == 0                                  # and the current one is empty


def test_some_cases_do_demote_and_some_do_not():
    n = [0, 0]
    for seed in range(25):
        w = inputs.small_random(seed=seed, n_req=60, p_sens=0.3, n_tenants=3)
        for i, kw in enumerate((PARAMS[0], PARAMS[2])):
            tree = OracleTree.from_workload(w)
            tree.match(w.req_off, w.req_tokens, w.req_tenant, max(w.max_blocks, 1))
            n[i] += tree.window_roll(**kw)
    assert n[0] > 20 and n[1] > 5
    w = inputs.small_random(seed=1, n_req=60)
    tree = OracleTree.from_workload(w)
    tree.match(w.req_off, w.req_tokens, w.req_tenant, max(w.max_blocks, 1))
    assert tree.window_roll(direction=0, tau=(0, 1)) == 0          # RDR < 0 never holds
    assert tree.window_roll(direction=0, tau=(1, 2)) == 0          # empty window: nothing to judge


def test_demotion_stops_cross_tenant_hits_and_keeps_the_creator():
    """After demotion only the creator may reuse the block (Section 6: future cross-tenant hits stop)."""
    blk = lambda ids: np.repeat(np.asarray(ids, dtype=np.int32), B)
    seq = blk([5, 6, 7])
    tree = OracleTree(seq, [0, 48], [0, 0, 0], [2, 1, 2], [3, 4, 5])   # all public; creators 2, 1, 2
    off = np.array([0, 48, 96, 144, 192], dtype=np.int32)
    toks = np.concatenate([seq] * 4)
    # tenant 0 probes four times: hits 4, distinct tenants 1 -> RDR 1/4 on every block
    mlen, _ = tree.match(off, toks, [0, 0, 0, 0], 3)
    assert (mlen == 48).all()
    assert tree.window_roll(direction=0, tau=(1, 2), min_hits=2) == 3
    priv, hit_pre, u_pre = tree.block_state()
    assert list(priv) == [1, 1, 1] and list(hit_pre) == [4, 4, 4] and list(u_pre) == [1, 1, 1]
    mlen, _ = tree.match(off[:4], toks[:144], [0, 1, 2], 3)
    assert list(mlen) == [0, 0, 16]      # tenant 2 created block 0 but not block 1; the others see nothing
    # sensitive blocks are never touched, and a broad window (RDR = 1) demotes nothing below tau = 1/2
    tree = OracleTree(seq, [0, 48], [1, 0, 0], [0, 1, 2], [3, 4, 5])
    tree.match(off[:4], toks[:144], [0, 1, 2], 3)
    assert tree.window_roll(direction=0, tau=(1, 2)) == 0


def test_consecutive_windows_are_required():
    blk = lambda ids: np.repeat(np.asarray(ids, dtype=np.int32), B)
    seq = blk([9])
    off3 = np.array([0, 16, 32, 48], dtype=np.int32)
    tree = OracleTree(seq, [0, 16], [0], [1], [0])
    kw = dict(direction=0, tau=(1, 2), min_hits=1, n_consec=2)
    tree.match(off3, np.concatenate([seq] * 3), [0, 0, 0], 1)      # narrow window 1
    assert tree.window_roll(**kw) == 0
    tree.match(off3, np.concatenate([seq] * 3), [0, 1, 2], 1)      # broad window breaks the streak
    assert tree.window_roll(**kw) == 0
    tree.match(off3, np.concatenate([seq] * 3), [0, 0, 0], 1)
    assert tree.window_roll(**kw) == 0
    tree.match(off3, np.concatenate([seq] * 3), [2, 2, 2], 1)      # second narrow window in a row
    assert tree.window_roll(**kw) == 1
