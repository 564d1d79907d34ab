"""Ragged batches (chains of different n in one call) through the C ABI against the oracle's
per-chain loops: every chain must get exactly what it gets on its own."""
import numpy as np
import pytest
import torch

import oracle
from paper_2502_12499_amd import binding as B
from paper_2502_12499_amd import inputs

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def to_dev(x):
    return torch.from_numpy(np.ascontiguousarray(x)).to(DEV)


def np_(t):
    return t.cpu().numpy()


def say(msg):
    print(msg, flush=True)


def check_eval(d, m, off):
    dd, md = to_dev(d), to_dev(m)
    off_dev = to_dev(off)
    for obj in (B.OBJ_STATIC, B.OBJ_DYNAMIC):
        peak, status = B.ckpt_ragged_eval_peak(dd, md, off, obj, offsets_dev=off_dev if obj else None)
        line, status2 = B.ckpt_ragged_eval_timeline(dd, md, off, obj, offsets_dev=None if obj else off_dev)
        torch.cuda.synchronize()
        assert (np_(status) == 0).all() and (np_(status2) == 0).all()
        assert np.array_equal(np_(peak), oracle.ragged_peak(d, m, off, obj)), f"objective {obj}"
        assert np.array_equal(np_(line), oracle.ragged_timeline(d, m, off, obj)), f"objective {obj}"
    both, status = B.ckpt_ragged_eval_peak(dd, md, off, B.OBJ_BOTH, offsets_dev=off_dev)
    torch.cuda.synchronize()
    assert (np_(status) == 0).all() and both.shape == (2, len(off) - 1)
    for obj in (B.OBJ_STATIC, B.OBJ_DYNAMIC):
        assert np.array_equal(np_(both)[obj], oracle.ragged_peak(d, m, off, obj)), f"both objectives, row {obj}"


def check_linear(d, off):
    want_peak, want_mask = oracle.ragged_solve_dynamic(d, off)
    for off_dev in (None, to_dev(off)):  # the library's own copy of the offsets, then the caller's
        mask, peak, status = B.ckpt_ragged_solve_linear(to_dev(d), off, offsets_dev=off_dev)
        torch.cuda.synchronize()
        assert (np_(status) == 0).all()
        assert np.array_equal(np_(peak), want_peak)
        assert np.array_equal(np_(mask), want_mask)


def check_cubic(d, off):
    mask, peak, budget, status = B.ckpt_ragged_solve_cubic(to_dev(d), off)
    torch.cuda.synchronize()
    want_peak, want_mask, want_s = oracle.ragged_solve_static(d, off)
    assert (np_(status) == 0).all()
    assert np.array_equal(np_(peak), want_peak)
    assert np.array_equal(np_(budget), want_s)
    assert np.array_equal(np_(mask), want_mask)


def test_networks_of_the_paper_in_one_batch():
    """One chain each of n = 1, 15, 24, 152, 257 and 1001 (Section 5's depths), the named ones with
    the layer lists' sizes, in an order that is not sorted by length."""
    lengths = [152, 1, 1001, 24, 257, 15]
    named = [(0, inputs.resnet152_chain()), (2, inputs.resnet1001_chain()), (3, inputs.vgg19_chain()),
             (5, inputs.alexnet_chain())]
    d, m, off = inputs.ragged_batch(11, lengths, named=named)
    say(f"ragged zoo: lengths {lengths}")
    check_eval(d, m, off)
    check_linear(d, off)
    check_cubic(d, off)


def test_many_short_chains_of_mixed_length():
    rng = np.random.default_rng(5)
    lengths = rng.choice([1, 2, 3, 15, 24, 63, 64, 65, 152, 257], size=6000)
    d, m, off = inputs.ragged_batch(12, lengths)
    say(f"ragged mixed: {len(lengths)} chains, {len(d)} sizes")
    check_eval(d, m, off)
    check_linear(d, off)


def test_cubic_on_mixed_lengths():
    rng = np.random.default_rng(6)
    lengths = rng.choice([1, 2, 3, 12, 15, 24, 63, 64, 65, 100], size=400)
    d, m, off = inputs.ragged_batch(13, lengths, lo_units=1, hi_units=4096)
    say(f"ragged cubic: {len(lengths)} chains")
    check_cubic(d, off)


def test_cubic_with_long_chains_in_the_batch():
    """Chains long enough for the cubic solver's launch that lays out the budgets and builds the size
    stack's links together, as a group of three inside a ragged batch (padded staging rows)."""
    lengths = [1100, 24, 1100, 15, 1100, 1030]
    d, m, off = inputs.ragged_batch(18, lengths)
    say(f"ragged cubic, long chains: lengths {lengths}")
    check_cubic(d, off)


def test_one_large_group_beside_small_ones():
    """A group of 70,001 chains spans many transposition tiles and leaves a ragged last tile."""
    lengths = np.full(70004, 24)
    lengths[[0, 35000, 70003]] = [257, 1, 64]
    d, m, off = inputs.ragged_batch(14, lengths)
    say("ragged large group")
    check_eval(d, m, off)
    check_linear(d, off)


def test_chain_with_a_bad_size_is_reported_alone():
    lengths = [15, 24, 15, 3]
    d, m, off = inputs.ragged_batch(15, lengths)
    good_peak, good_mask = oracle.ragged_solve_dynamic(d, off)
    bad = d.copy()
    bad[off[1] + 7] = 0
    mask, peak, status = B.ckpt_ragged_solve_linear(to_dev(bad), off)
    cmask, cpeak, cbudget, cstatus = B.ckpt_ragged_solve_cubic(to_dev(bad), off)
    epeak, estatus = B.ckpt_ragged_eval_peak(to_dev(bad), to_dev(m), off, B.OBJ_DYNAMIC)
    torch.cuda.synchronize()
    for st in (status, cstatus, estatus):
        assert np_(st).tolist() == [0, 3, 0, 0]
    assert np_(peak)[1] == -1 and np_(cpeak)[1] == -1 and np_(epeak)[1] == -1
    assert not np_(mask)[off[1]:off[2]].any() and not np_(cmask)[off[1]:off[2]].any()
    keep = np.ones(len(d), dtype=bool)
    keep[off[1]:off[2]] = False
    assert np.array_equal(np_(mask)[keep], good_mask[keep])
    assert np.array_equal(np_(peak)[[0, 2, 3]], good_peak[[0, 2, 3]])


def test_linear_hands_chains_of_several_groups_to_its_later_kernels():
    """Sizes that are no multiples of a power of two and need more than 30 bits leave the first
    linear kernel for the 64-bit one, which then finds each listed chain's length and staging
    from its group; a few chains whose sums pass 2^63 go on to the last kernel and come back with
    their status.  Groups on both sides of the register-log limit, short and long mixed."""
    lengths = np.array([3, 40, 300, 17, 40, 258, 1, 40, 255, 300, 17, 64] * 23, dtype=np.int64)
    d, m, off = inputs.ragged_batch(21, lengths, lo_units=1 << 20, hi_units=1 << 36, unit=1)
    d_small, _, _ = inputs.ragged_batch(22, lengths)           # every third chain stays in the first kernel
    for c in range(0, len(lengths), 3):
        d[off[c]:off[c + 1]] = d_small[off[c]:off[c + 1]]
    say(f"ragged linear, {len(lengths)} chains, 64-bit sizes in two of three")
    check_linear(d, off)
    check_eval(d, m, off)
    over = d.copy()
    hit = [5, 40, 101]                                         # chains of 258, 40 and 258 layers: sums beyond 64 bits
    for c in hit:
        over[off[c]:off[c + 1]] = (1 << 62) + 12345
    mask, peak, status = B.ckpt_ragged_solve_linear(to_dev(over), off)
    torch.cuda.synchronize()
    want_peak, want_mask = oracle.ragged_solve_dynamic(d, off)
    st = np_(status)
    ok = np.ones(len(lengths), dtype=bool)
    ok[hit] = False
    assert (st[ok] == 0).all() and (st[hit] == 4).all()        # CKPT_ERR_OVERFLOW
    assert np.array_equal(np_(peak)[ok], want_peak[ok])
    got_mask = np_(mask)
    for c in np.nonzero(ok)[0]:
        assert np.array_equal(got_mask[off[c]:off[c + 1]], want_mask[off[c]:off[c + 1]]), f"chain {c}"


def test_many_distinct_lengths_and_repeated_calls():
    """Every chain a group of its own next to large groups, twice in a row into one workspace: the
    places inside a group may differ between the calls, the results may not."""
    rng = np.random.default_rng(8)
    lengths = np.concatenate([np.arange(1, 200), rng.choice([7, 31, 64], size=5000)])
    rng.shuffle(lengths)
    d, m, off = inputs.ragged_batch(17, lengths)
    want_peak, want_mask = oracle.ragged_solve_dynamic(d, off)
    dd = to_dev(d)
    ws = torch.empty(B.load().ckpt_ragged_workspace_bytes(B.CALL_SOLVE_LINEAR, off.ctypes.data, len(lengths)),
                     dtype=torch.uint8, device=DEV)
    for _ in range(2):
        mask, peak, status = B.ckpt_ragged_solve_linear(dd, off, workspace=ws, offsets_dev=to_dev(off))
        torch.cuda.synchronize()
        assert np.array_equal(np_(peak), want_peak) and np.array_equal(np_(mask), want_mask)


def test_long_chains_counted_on_the_device():
    """Lengths on both sides of the limit up to which the device's count adds up per workgroup
    first, one group of a single chain next to another, and a batch of one chain."""
    lengths = np.array([4096, 5000, 4095, 1, 7000, 5000, 4096, 2], dtype=np.int64)
    d, m, off = inputs.ragged_batch(41, lengths)
    say(f"ragged, lengths {lengths.tolist()}")
    check_eval(d, m, off)
    check_linear(d, off)
    d, m, off = inputs.ragged_batch(42, np.array([9000], dtype=np.int64))
    check_eval(d, m, off)
    check_linear(d, off)


def test_offsets_counted_on_the_device_are_checked_there():
    """With a device copy of the offsets the lengths are counted on the GPU and the host's copy is
    not read: an offset out of range in the device copy ends the call with CKPT_ERR_SHAPE before
    any chain is touched, and the next call on the same workspace is as good as ever."""
    lengths = np.array([15, 3, 24, 15, 70, 1, 300] * 11, dtype=np.int64)
    d, m, off = inputs.ragged_batch(31, lengths)
    dd, md = to_dev(d), to_dev(m)
    need = max(B.load().ckpt_ragged_workspace_bytes(which, off.ctypes.data, len(lengths))
               for which in (B.CALL_SOLVE_LINEAR, B.CALL_EVAL_PEAK))
    ws = torch.empty(need, dtype=torch.uint8, device=DEV)
    for at, value in ((5, off[4]), (9, off[10] - 1), (0, -8), (len(lengths), 1 << 60), (20, off[19] + 70000)):
        bad = off.copy()
        bad[at] = value                                        # decreasing, one element, negative, huge, too long
        say(f"offsets_dev[{at}] = {value}")
        for call in (lambda: B.ckpt_ragged_solve_linear(dd, off, workspace=ws, offsets_dev=to_dev(bad)),
                     lambda: B.ckpt_ragged_eval_peak(dd, md, off, B.OBJ_STATIC, workspace=ws, offsets_dev=to_dev(bad))):
            with pytest.raises(B.CkptError) as err:
                call()
            assert err.value.code == 2                         # CKPT_ERR_SHAPE
        torch.cuda.synchronize()
    mask, peak, status = B.ckpt_ragged_solve_linear(dd, off, workspace=ws, offsets_dev=to_dev(off))
    want_peak, want_mask = oracle.ragged_solve_dynamic(d, off)
    assert (np_(status) == 0).all() and np.array_equal(np_(peak), want_peak) and np.array_equal(np_(mask), want_mask)
    # a workspace that holds the tables but not the staging is refused after the count
    small = torch.empty(300 * 1024, dtype=torch.uint8, device=DEV)
    with pytest.raises(B.CkptError) as err:
        B.ckpt_ragged_eval_timeline(dd, md, off, B.OBJ_DYNAMIC, workspace=small, offsets_dev=to_dev(off))
    assert err.value.code == 6                                 # CKPT_ERR_WORKSPACE


def test_host_checks_and_the_empty_batch():
    d, m, off = inputs.ragged_batch(16, [4, 5])
    dd = to_dev(d)
    for bad in ([0, 5, 4], [0, 1, 11], [-1, 5, 11]):
        with pytest.raises(B.CkptError) as e:
            B.ckpt_ragged_solve_linear(dd, np.array(bad, dtype=np.int64))
        assert e.value.code == 2
    with pytest.raises(ValueError):
        B.ckpt_ragged_solve_linear(dd, np.array([0, 5, 12], dtype=np.int64))
    mask, peak, status = B.ckpt_ragged_solve_linear(dd[:0], np.array([0], dtype=np.int64))
    torch.cuda.synchronize()
    assert peak.numel() == 0 and mask.numel() == 0
    lib = B.load()
    assert lib.ckpt_ragged_workspace_bytes(B.CALL_SOLVE_LINEAR, None, 3) == 0
    assert lib.ckpt_ragged_workspace_bytes(9, off.ctypes.data, 2) == 0
    assert lib.ckpt_ragged_workspace_bytes(B.CALL_SOLVE_CUBIC, off.ctypes.data, 2) > 0
