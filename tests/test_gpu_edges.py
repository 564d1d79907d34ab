"""Edge cases of the C ABI on the GPU: the longest chains the calls take, odd
strides, an empty batch.  Compared with the CPU oracle, bit-exact."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
from paper_2502_12499_amd import binding as B
from paper_2502_12499_amd import inputs

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def say(msg):
    print(msg, flush=True)


def test_longest_chain_n65535():
    """CKPT_MAX_LAYERS: eval_peak, eval_timeline and solve_linear on three chains of 65,536 sizes."""
    n = 65535
    say(f"n = {n}: eval_peak, eval_timeline, solve_linear")
    d = inputs.uniform_aligned_chains(4, n, 3, 1, 4096, unit=512)
    m = inputs.bernoulli_masks(4, n, 3)
    dt, mt = torch.from_numpy(d).to(DEV), torch.from_numpy(m).to(DEV)
    dc, mc = inputs.chain_major(d), inputs.chain_major(m)
    for obj in (B.OBJ_STATIC, B.OBJ_DYNAMIC):
        peak, status = B.ckpt_eval_peak(dt, mt, obj)
        assert (status.cpu().numpy() == 0).all()
        assert np.array_equal(peak.cpu().numpy(), oracle.batch_peak(dc, mc, obj))
        tl, status = B.ckpt_eval_timeline(dt, mt, obj)
        assert np.array_equal(tl.cpu().numpy().T, oracle.batch_timeline(dc, mc, obj))
    say("  solve_linear (the oracle's quadratic recurrence takes a few seconds per chain)")
    mask, peak, status = B.ckpt_solve_linear(dt)
    want_peak, want_mask = oracle.batch_solve_dynamic(dc)
    assert (status.cpu().numpy() == 0).all()
    assert np.array_equal(peak.cpu().numpy(), want_peak)
    assert np.array_equal(mask.cpu().numpy().T, want_mask)


def test_strided_layouts():
    """Chains laid out with padding between positions and between chains, and a chain stride too
    large for the lane-per-chain kernel's 32-bit offsets (every chain then takes the 64-bit path)."""
    n, batch = 40, 5
    d = inputs.log_uniform_chains(8, n, batch)                       # (n+1, batch)
    dc = inputs.chain_major(d)
    want_peak, want_mask = oracle.batch_solve_dynamic(dc)
    want_speak, want_smask, want_s = oracle.batch_solve_static(dc)
    for chain_stride, pos_stride in ((1, 7), (n + 9, 1), (3 * (n + 1), 3), ((1 << 22) + 5, 1)):
        say(f"strides: chain {chain_stride}, position {pos_stride}")
        span = (batch - 1) * chain_stride + n * pos_stride + 1
        buf = torch.full((span,), 123456789, dtype=torch.int64, device=DEV)
        view = torch.as_strided(buf, (n + 1, batch), (pos_stride, chain_stride))
        view.copy_(torch.from_numpy(d).to(DEV))
        mask, peak, status = B.ckpt_solve_linear(view)
        assert (status.cpu().numpy() == 0).all()
        assert np.array_equal(peak.cpu().numpy(), want_peak)
        assert np.array_equal(mask.cpu().numpy().T, want_mask)
        qmask, qpeak, qM, qstatus = B.ckpt_solve_quadratic(view)
        assert np.array_equal(qpeak.cpu().numpy(), want_peak)
        assert np.array_equal(qmask.cpu().numpy().T, want_mask)
        again, _ = B.ckpt_eval_peak(view, mask, B.OBJ_DYNAMIC)
        assert np.array_equal(again.cpu().numpy(), want_peak)
        tl, _ = B.ckpt_eval_timeline(view, mask, B.OBJ_DYNAMIC)
        assert np.array_equal(tl.cpu().numpy().T, oracle.batch_timeline(dc, want_mask, B.OBJ_DYNAMIC))
        if chain_stride < (1 << 20):
            cmask, cpeak, cbudget, cstatus = B.ckpt_solve_cubic(view)
            assert np.array_equal(cpeak.cpu().numpy(), want_speak)
            assert np.array_equal(cbudget.cpu().numpy(), want_s)
            assert np.array_equal(cmask.cpu().numpy().T, want_smask)


def test_empty_batch_is_a_no_op():
    lib = B.load()
    E = B.Layout(0, 8, 1, 1)
    assert lib.ckpt_solve_linear(None, ctypes.byref(E), None, None, None, None, 0, None) == 0
    assert lib.ckpt_eval_timeline(None, None, ctypes.byref(E), 1, None, 1, 1, None, None) == 0
    assert lib.ckpt_solve_quadratic(None, ctypes.byref(E), None, None, None, None, None) == 0
    assert lib.ckpt_select_baseline(ctypes.byref(E), 2, None, None) == 0
    assert lib.ckpt_solve_cubic_pruned(None, ctypes.byref(E), None, None, None, None, None, None, 0, None) == 0
    torch.cuda.synchronize()


def test_cubic_calls_in_flight_on_two_streams():
    """Two callers' streams, each with cubic calls of its own (workspaces apart): the calls share the
    library's side stream and its events, and every call still finds its own tables finished."""
    say("solve_cubic on two streams at once")
    chains = [inputs.config5_single(700), inputs.config4(), inputs.config5_single(1300), inputs.config2()]
    want = [oracle.solve_static(d[:, 0]) for d in chains]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    dev_in = [torch.from_numpy(d).to(DEV) for d in chains]
    torch.cuda.synchronize()
    got = [None] * len(chains)
    for rounds in range(2):                      # the second round finds stream and events in use
        for k, x in enumerate(dev_in):
            with torch.cuda.stream(streams[k % 2]):
                got[k] = (B.ckpt_solve_cubic_pruned(x) if (k + rounds) % 2 else B.ckpt_solve_cubic(x))
        torch.cuda.synchronize()
        for k, (v, mk, s) in enumerate(want):
            mask, peak, budget = got[k][0], got[k][1], got[k][2]
            assert int(peak.cpu()[0]) == v and int(budget.cpu()[0]) == s
            assert np.array_equal(mask.cpu().numpy()[:, 0], mk)
