"""Parity of ckpt_solve_quadratic (Algorithm 5, one wave per chain) with the
CPU oracle: optimum, canonical set and the whole value function M, bit-exact;
and agreement with the linear-time kernel on the device."""
import numpy as np
import pytest
import torch

import oracle
from paper_2502_12499_amd import binding as B
from paper_2502_12499_amd import inputs
from test_gpu_parity import special_chains

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def to_dev(x):
    return torch.from_numpy(np.ascontiguousarray(x)).to(DEV)


def say(msg):
    print(msg, flush=True)


def oracle_values(dc):
    """(peak, mask, M) per chain of a chain-major batch, by Algorithm 5 on the CPU."""
    peaks, masks, Ms = [], [], []
    for row in dc:
        v, mask, M = oracle.solve_dynamic(row)
        peaks.append(v); masks.append(mask); Ms.append(M)
    return np.array(peaks, dtype=np.int64), np.stack(masks), np.stack(Ms)


def check_quadratic(d, chain_major=False, values=True):
    dc = inputs.chain_major(d)
    if chain_major:
        mask, peak, M, status = B.ckpt_solve_quadratic(to_dev(dc), chain_major=True)
        got_mask, got_M = mask.cpu().numpy(), M.cpu().numpy()
    else:
        mask, peak, M, status = B.ckpt_solve_quadratic(to_dev(d))
        got_mask, got_M = mask.cpu().numpy().T, M.cpu().numpy().T
    if values:
        want_peak, want_mask, want_M = oracle_values(dc)
        assert np.array_equal(got_M, want_M)
    else:
        want_peak, want_mask = oracle.batch_solve_dynamic(dc)
    assert (status.cpu().numpy() == 0).all()
    assert np.array_equal(peak.cpu().numpy(), want_peak)
    assert np.array_equal(got_mask, want_mask)


@pytest.mark.parametrize("name,d", special_chains())
def test_solve_quadratic_special_chains(name, d):
    say(f"solve_quadratic {name}")
    check_quadratic(d.reshape(-1, 1))


def test_solve_quadratic_single_chain_configs():
    for name, d in (("config1", inputs.config1()), ("config2", inputs.config2()), ("config4", inputs.config4())):
        say(f"solve_quadratic {name}")
        check_quadratic(d)
    say("solve_quadratic n = 4095 (the longest chain it takes)")
    check_quadratic(inputs.config5_single(4095))


@pytest.mark.parametrize("batch,n,kind", [(1, 1, "log"), (64, 64, "log"), (1000, 64, "log"), (333, 17, "ties"),
                                          (512, 256, "aligned"), (130, 300, "ties"), (9000, 33, "log")])
def test_solve_quadratic_batches(batch, n, kind):
    say(f"solve_quadratic batch={batch} n={n} {kind}")
    if kind == "log":
        d = inputs.log_uniform_chains(1, n, batch)
    elif kind == "aligned":
        d = inputs.uniform_aligned_chains(2, n, batch, 256, 32768)
    else:
        d = inputs.uniform_aligned_chains(5, n, batch, 1, 3, unit=1)
    check_quadratic(d, values=batch <= 1000)
    if batch <= 1000:
        check_quadratic(d, chain_major=True)


def test_solve_quadratic_data_errors_and_limits():
    say("solve_quadratic: per-chain data errors, host checks")
    n, batch = 12, 4
    d = inputs.uniform_aligned_chains(3, n, batch, 1, 100, unit=1)
    d[5, 1] = 0
    d[:, 2] = (1 << 61)
    mask, peak, M, status = B.ckpt_solve_quadratic(to_dev(d))
    assert status.cpu().numpy().tolist() == [0, 3, 4, 0]
    assert peak.cpu().numpy()[[1, 2]].tolist() == [-1, -1]
    assert (mask.cpu().numpy()[:, [1, 2]] == 0).all() and (M.cpu().numpy()[:, [1, 2]] == -1).all()
    for c in (0, 3):
        v, mk, Mv = oracle.solve_dynamic(d[:, c])
        assert int(peak[c]) == v and np.array_equal(mask.cpu().numpy()[:, c], mk)
        assert np.array_equal(M.cpu().numpy()[:, c], Mv)
    with pytest.raises(B.CkptError):
        B.ckpt_solve_quadratic(torch.ones((4097, 1), dtype=torch.int64, device=DEV))


def test_quadratic_and_linear_kernels_agree_config3():
    say("config 3 (65,536 chains, n = 64): quadratic kernel = linear kernel = oracle")
    d, _ = inputs.config3()
    dt = to_dev(d)
    qmask, qpeak, qM, qstatus = B.ckpt_solve_quadratic(dt)
    lmask, lpeak, lstatus = B.ckpt_solve_linear(dt)
    assert int(qstatus.abs().sum()) == 0 and int(lstatus.abs().sum()) == 0
    assert bool((qpeak == lpeak).all()) and bool((qmask == lmask).all())
    want_peak, want_mask = oracle.batch_solve_dynamic(inputs.chain_major(d))
    assert np.array_equal(qpeak.cpu().numpy(), want_peak)
    assert np.array_equal(qmask.cpu().numpy().T, want_mask)
    assert bool((qM[0] == qpeak).all()) and bool((qM[64] == dt[64]).all())
