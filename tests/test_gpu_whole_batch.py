"""The whole stress batch (1,048,576 chains of 256 layers), element by element against the
oracle: ckpt_eval_peak and ckpt_eval_timeline under both objectives, ckpt_solve_linear's optimum
and canonical set.  The batch is taken in slices of chains, so that the oracle's outputs (two
4.3 GB timelines) never have to exist at once; each slice is a call of its own on the resident
batch, in the launch configuration bench.py times (position-major, one lane per chain)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2502_12499_amd import binding as B
from paper_2502_12499_amd import inputs

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
BATCH, N = 1048576, 256


def say(msg):
    print(msg, flush=True)


@pytest.fixture(scope="module")
def batch():
    d, m = inputs.config5_batch(BATCH, N)
    return d, m, torch.from_numpy(d).to(DEV), torch.from_numpy(m).to(DEV)


def test_eval_peak_whole_batch(batch):
    d, m, dt, mt = batch
    say(f"eval_peak, both objectives in one call (as bench.py times it): all {BATCH} chains")
    both, status = B.ckpt_eval_peak(dt, mt, B.OBJ_BOTH)
    both = both.cpu().numpy()
    assert int(status.abs().sum()) == 0
    for obj in (B.OBJ_STATIC, B.OBJ_DYNAMIC):
        say(f"eval_peak objective {obj}: all {BATCH} chains")
        peak, status = B.ckpt_eval_peak(dt, mt, obj)
        got = peak.cpu().numpy()
        assert int(status.abs().sum()) == 0
        for c0 in range(0, BATCH, 262144):
            sl = slice(c0, c0 + 262144)
            want = oracle.batch_peak(inputs.chain_major(d[:, sl]), inputs.chain_major(m[:, sl]), obj)
            assert np.array_equal(got[sl], want), f"objective {obj}, chains from {c0}"
            assert np.array_equal(both[obj, sl], want), f"both objectives, row {obj}, chains from {c0}"


def test_solve_linear_whole_batch(batch):
    d, m, dt, mt = batch
    say(f"solve_linear: all {BATCH} chains (the oracle's quadratic recurrence on each)")
    mask, peak, status = B.ckpt_solve_linear(dt)
    assert int(status.abs().sum()) == 0
    got_peak, got_mask = peak.cpu().numpy(), mask.cpu().numpy()
    for c0 in range(0, BATCH, 131072):
        sl = slice(c0, c0 + 131072)
        want_peak, want_mask = oracle.batch_solve_dynamic(inputs.chain_major(d[:, sl]))
        assert np.array_equal(got_peak[sl], want_peak), f"chains from {c0}"
        assert np.array_equal(got_mask[:, sl].T, want_mask), f"chains from {c0}"
        say(f"  chains {c0}..{c0 + 131071} ok")


def test_eval_timeline_whole_batch(batch):
    d, m, dt, mt = batch
    for obj in (B.OBJ_STATIC, B.OBJ_DYNAMIC):
        say(f"eval_timeline objective {obj}: all {BATCH} chains, 514 phases each")
        tl, status = B.ckpt_eval_timeline(dt, mt, obj)
        assert int(status.abs().sum()) == 0
        for c0 in range(0, BATCH, 131072):
            sl = slice(c0, c0 + 131072)
            want = oracle.batch_timeline(inputs.chain_major(d[:, sl]), inputs.chain_major(m[:, sl]), obj)
            got = tl[:, c0:c0 + 131072].cpu().numpy()
            assert np.array_equal(got.T, want), f"objective {obj}, chains from {c0}"
        del tl
        say("  ok")
