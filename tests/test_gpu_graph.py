"""The hot path recorded as a HIP graph: every replay must reproduce what the eager calls produce.

The library calls of one pass (counter reset, lookup, suffix offsets, gather, attention) only enqueue kernels on
the caller's stream, so a serving loop may capture them once and replay them.  Each replay is checked against the
eager result, with eager work and synchronisations of the program between the replays."""
import numpy as np
import pytest
import torch

from paper_2508_08438_amd import inputs
from paper_2508_08438_amd.pipeline import Session

pytestmark = pytest.mark.gpu


def snapshot(s):
    torch.cuda.synchronize()
    hit, ucnt = s.counters()
    return {"matched_len": s.matched_len.cpu().numpy().copy(), "page_table": s.page_table.cpu().numpy().copy(),
            "q_off": s.q_off.cpu().numpy().copy(), "out": s.out.float().cpu().numpy().copy(),
            "kctx": s.kctx.view(torch.int16).cpu().numpy().copy(), "vctx": s.vctx.view(torch.int16).cpu().numpy().copy(),
            "hit": hit.copy(), "ucnt": ucnt.copy()}


def clobber(s):
    """eager work between replays that ruins every output of the pass"""
    s.matched_len.fill_(-7)
    s.page_table.fill_(-3)
    s.q_off.fill_(0)
    s.out.fill_(float("nan"))
    s.kctx.fill_(1.0)
    s.vctx.fill_(1.0)
    torch.cuda.synchronize()


@pytest.mark.parametrize("name", ["c2", "c3"])
def test_graph_replays_match_eager(name):
    w = inputs.CONFIGS[name]()
    s = Session(w)
    s.prepare()
    s.step()
    want = snapshot(s)
    s.capture_step()
    for rep in range(3):
        clobber(s)
        s.replay()
        got = snapshot(s)
        for key in want:
            assert np.array_equal(want[key], got[key], equal_nan=(key == "out")), (name, rep, key)
    # and an eager pass after the replays is still the same
    clobber(s)
    s.step()
    got = snapshot(s)
    for key in want:
        assert np.array_equal(want[key], got[key], equal_nan=(key == "out")), (name, "eager after", key)
