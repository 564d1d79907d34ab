"""Parity of the HIP library (through the C ABI) with the CPU oracle, element
by element, on seeded inputs.  All values are integers: the bar is bit-exact
peaks, budgets, statuses and checkpoint masks (the canonical sets)."""
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


# ---------------------------------------------------------------------------
# helpers: run one call and compare with the oracle
# ---------------------------------------------------------------------------

def check_eval(d, m, chain_major=False):
    """d, m: position-major numpy (n+1, batch)."""
    dc, mc = inputs.chain_major(d), inputs.chain_major(m)
    for obj in (B.OBJ_STATIC, B.OBJ_DYNAMIC):
        if chain_major:
            peak, status = B.ckpt_eval_peak(to_dev(dc), to_dev(mc), obj, chain_major=True)
        else:
            peak, status = B.ckpt_eval_peak(to_dev(d), to_dev(m), obj)
        torch.cuda.synchronize()
        want = oracle.batch_peak(dc, mc, obj)
        assert (np_(status) == 0).all()
        assert np.array_equal(np_(peak), want), f"objective {obj}"
    # both objectives from one pass over the chains
    if chain_major:
        peak, status = B.ckpt_eval_peak(to_dev(dc), to_dev(mc), B.OBJ_BOTH, chain_major=True)
    else:
        peak, status = B.ckpt_eval_peak(to_dev(d), to_dev(m), B.OBJ_BOTH)
    torch.cuda.synchronize()
    assert (np_(status) == 0).all() and peak.shape == (2, d.shape[1])
    for obj in (B.OBJ_STATIC, B.OBJ_DYNAMIC):
        assert np.array_equal(np_(peak)[obj], oracle.batch_peak(dc, mc, obj)), f"both objectives, row {obj}"


def check_linear(d, chain_major=False):
    dc = inputs.chain_major(d)
    if chain_major:
        mask, peak, status = B.ckpt_solve_linear(to_dev(dc), chain_major=True)
        got_mask = np_(mask)
    else:
        mask, peak, status = B.ckpt_solve_linear(to_dev(d))
        got_mask = np_(mask).T
    torch.cuda.synchronize()
    want_peak, want_mask = oracle.batch_solve_dynamic(dc)
    assert (np_(status) == 0).all()
    assert np.array_equal(np_(peak), want_peak)
    assert np.array_equal(got_mask, want_mask)


def check_cubic(d, chain_major=False):
    """Both forms of the call (every budget; without the budgets that cannot be optimal)."""
    dc = inputs.chain_major(d)
    want_peak, want_mask, want_s = oracle.batch_solve_static(dc)
    n = d.shape[0] - 1
    K = n * (n - 1) // 2 + 1
    for pruned in (False, True):
        x = to_dev(dc) if chain_major else to_dev(d)
        if pruned:
            mask, peak, budget, evaluated, status = B.ckpt_solve_cubic_pruned(x, chain_major=chain_major)
            # at most every budget once plus the sampled tiles (whole tiles) a second time
            assert bool((evaluated >= 1).all()) and bool((evaluated <= K + K // 64 + 512).all()), "evaluated"
            if n < 3072:
                assert bool((evaluated == K).all())
        else:
            mask, peak, budget, status = B.ckpt_solve_cubic(x, chain_major=chain_major)
        torch.cuda.synchronize()
        got_mask = np_(mask) if chain_major else np_(mask).T
        assert (np_(status) == 0).all()
        assert np.array_equal(np_(peak), want_peak), f"pruned={pruned}"
        assert np.array_equal(np_(budget), want_s), f"pruned={pruned}"
        assert np.array_equal(got_mask, want_mask), f"pruned={pruned}"


def special_chains():
    """Degenerate and adversarial single chains, as (name, 1-D int64 array)."""
    rng = np.random.default_rng(7)
    out = [
        ("n1", np.array([5, 9])),
        ("n2", np.array([5, 1, 9])),
        ("n3_ties", np.array([2, 2, 2, 2])),
        ("uniform_50", np.ones(51, dtype=np.int64) * 4096),
        ("increasing_80", np.arange(1, 82, dtype=np.int64) * 3),          # deep queues
        ("decreasing_80", np.arange(81, 0, -1, dtype=np.int64) * 5),
        ("huge_last", np.concatenate([np.ones(70, dtype=np.int64), [10 ** 12]])),
        ("huge_first", np.concatenate([[10 ** 12], np.ones(70, dtype=np.int64)])),
        ("sawtooth_97", np.tile(np.array([1, 50, 3, 40, 7], dtype=np.int64), 20)[:98]),
        ("ties_200", rng.integers(1, 4, size=201)),
        ("wide_130", rng.integers(1, 1 << 40, size=131)),                   # 64-bit arithmetic
        ("wide_900", rng.integers(1, 1 << 36, size=901)),                   # ... and more tiles of budgets than workgroups
        ("odd_bytes_65", rng.integers(1, 1 << 20, size=66) * 2 + 1),        # no common factor
        ("vgg19", inputs.vgg19_chain()[:, 0]),
        ("alexnet", inputs.alexnet_chain()[:, 0]),
    ]
    return [(k, np.asarray(v, dtype=np.int64)) for k, v in out]


# ---------------------------------------------------------------------------
# eval_peak
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("batch,n", [(1, 12), (3, 1), (64, 64), (1000, 64), (777, 257), (4096, 256)])
def test_eval_peak_batches(batch, n):
    say(f"eval_peak batch={batch} n={n}")
    d = inputs.log_uniform_chains(11, n, batch)
    m = inputs.bernoulli_masks(11, n, batch)
    check_eval(d, m)
    check_eval(d, m, chain_major=True)


def test_eval_peak_fixed_sets_and_paper_sets():
    d = inputs.vgg19_chain()
    for positions in ([3, 6, 24], [5, 10, 15, 20, 24], [2, 4, 6, 9, 11, 14, 16, 19, 21, 23, 24], [24],
                      list(range(1, 25))):
        m = np.zeros((25, 1), dtype=np.uint8)
        m[0] = 1
        m[positions] = 1
        check_eval(d, m)


def test_eval_peak_data_errors():
    n, batch = 9, 6
    d = inputs.uniform_aligned_chains(3, n, batch, 1, 100, unit=1)
    m = np.ones((n + 1, batch), dtype=np.uint8)
    d[4, 1] = 0                      # non-positive size
    d[2, 2] = -5
    d[:, 3] = (1 << 62)              # overflow of the sum
    m[0, 4] = 0                      # open ends
    m[n, 5] = 0
    for obj in (0, 1):
        peak, status = B.ckpt_eval_peak(to_dev(d), to_dev(m), obj)
        torch.cuda.synchronize()
        assert np_(status).tolist() == [0, 3, 3, 4, 5, 5]
        assert np_(peak)[1:].tolist() == [-1] * 5
        assert np_(peak)[0] == oracle.batch_peak(inputs.chain_major(d)[:1], inputs.chain_major(m)[:1], obj)[0]
    peak, status = B.ckpt_eval_peak(to_dev(d), to_dev(m), B.OBJ_BOTH)
    torch.cuda.synchronize()
    assert np_(status).tolist() == [0, 3, 3, 4, 5, 5]
    assert np_(peak)[:, 1:].tolist() == [[-1] * 5] * 2
    for obj in (0, 1):
        assert np_(peak)[obj, 0] == oracle.batch_peak(inputs.chain_major(d)[:1], inputs.chain_major(m)[:1], obj)[0]
    with pytest.raises(B.CkptError):
        B.ckpt_eval_peak(to_dev(d), to_dev(m), 3)
    with pytest.raises(B.CkptError):
        B.ckpt_eval_timeline(to_dev(d), to_dev(m), B.OBJ_BOTH)      # a timeline is of one objective


# ---------------------------------------------------------------------------
# solve_linear
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("name,d", special_chains())
def test_solve_linear_special_chains(name, d):
    say(f"solve_linear {name}")
    check_linear(d.reshape(-1, 1))


def test_solve_linear_single_chain_configs():
    for name, d in (("config1", inputs.config1()), ("config2", inputs.config2()), ("config4", inputs.config4())):
        say(f"solve_linear {name}")
        check_linear(d)
    say("solve_linear config5 single")
    check_linear(inputs.config5_single(4096))


@pytest.mark.parametrize("batch,n,kind", [(64, 64, "log"), (1000, 64, "log"), (333, 17, "ties"),
                                          (4096, 64, "log"), (2048, 256, "aligned"), (130, 300, "ties")])
def test_solve_linear_batches(batch, n, kind):
    say(f"solve_linear batch={batch} n={n} {kind}")
    if kind == "log":
        d = inputs.log_uniform_chains(1, n, batch)
    elif kind == "aligned":
        d = inputs.uniform_aligned_chains(2, n, batch, 256, 32768)
    else:
        d = inputs.uniform_aligned_chains(5, n, batch, 1, 3, unit=1)
    check_linear(d)
    if batch <= 1000:
        check_linear(d, chain_major=True)


@pytest.mark.parametrize("n", [1, 2, 3, 7, 8, 9, 15, 16, 17, 63, 64, 65, 247, 248, 249, 255, 256, 257, 258, 264])
def test_solve_linear_lengths_around_the_chunk_and_register_limits(n):
    """Chains of up to 256 layers keep their steps in registers, eight positions to a pair of them, longer
    ones park them in the mask: lengths on both sides of every such boundary, with a ragged last wave,
    aligned sizes, tied sizes and sizes whose common power of two shrinks along the chain."""
    batch = 130
    say(f"solve_linear n={n}")
    check_linear(inputs.uniform_aligned_chains(30 + n, n, batch, 256, 32768))
    check_linear(inputs.uniform_aligned_chains(31 + n, n, batch, 1, 3, unit=1))
    d = inputs.uniform_aligned_chains(32 + n, n, batch, 256, 32768)
    d[n // 2, ::2] += 12
    d[0, 1::4] += 1
    check_linear(d)
    # long steps (every interior size tiny against the ends) and a ring that fills: these chains are
    # deferred to the other kernels, their neighbours are not
    d = inputs.uniform_aligned_chains(33 + n, n, batch, 256, 32768)
    d[:, 3] = 1
    d[n, 3] = 1000
    d[n, 64] = 10 ** 13
    check_linear(d)


def test_solve_linear_mixed_alignment_and_deferred_chains():
    # sizes whose common power of two shrinks as the chain is read, chains that
    # need 64-bit values, deep queues and long steps, all in one batch
    say("solve_linear mixed batch")
    rng = np.random.default_rng(42)
    n, batch = 300, 256
    d = inputs.uniform_aligned_chains(9, n, batch, 256, 32768)
    for c in range(0, batch, 3):
        k = int(rng.integers(0, n + 1))
        d[k, c] += int(rng.integers(1, 4096))              # one unaligned size somewhere
    for c in range(1, batch, 16):
        d[:, c] *= 1 << 20                                 # still 32-bit after the common shift
    for c in range(2, batch, 16):
        d[:, c] = rng.integers(1, 1 << 45, size=n + 1)     # needs 64-bit values
    d[n, 5] = 10 ** 13                                     # every entry stays live: ring overflow
    d[:, 7] = 1
    d[n, 7] = 1000                                         # optimal steps longer than 255
    check_linear(d)


def test_solve_linear_data_errors():
    n, batch = 12, 4
    d = inputs.uniform_aligned_chains(3, n, batch, 1, 100, unit=1)
    d[5, 1] = 0
    d[:, 2] = (1 << 61)
    mask, peak, status = B.ckpt_solve_linear(to_dev(d))
    torch.cuda.synchronize()
    assert np_(status).tolist() == [0, 3, 4, 0]
    assert np_(peak)[1] == -1 and np_(peak)[2] == -1
    assert (np_(mask)[:, 1] == 0).all() and (np_(mask)[:, 2] == 0).all()
    for c in (0, 3):
        v, mk, _ = oracle.solve_dynamic(d[:, c])
        assert np_(peak)[c] == v and (np_(mask)[:, c] == mk).all()


# ---------------------------------------------------------------------------
# solve_cubic
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("name,d", special_chains())
def test_solve_cubic_special_chains(name, d):
    say(f"solve_cubic {name}")
    check_cubic(d.reshape(-1, 1))


def group_edge_chains():
    """32-bit chains of lengths around the cubic kernel's units (groups of 8 positions, rounds of 32,
    the loop starting at position 8), shaped so that queue events fall on and around the groups'
    first and last positions."""
    rng = np.random.default_rng(23)
    out = []
    for n in (39, 40, 41, 47, 48, 71, 72, 73, 103, 104, 105, 136, 167, 168, 169):
        k = np.arange(n + 1)
        shapes = {
            "random": rng.integers(256, 32769, size=n + 1),
            "constant": np.full(n + 1, 7),
            "increasing": 3 + k,
            "decreasing": 3 + n - k,                       # the size stack grows to n
            "spike_every_8": np.where(k % 8 == 0, 5000, 9 + k % 5),
            "spike_before_8": np.where(k % 8 == 7, 5000, 9 + k % 5),
            "dip_every_8": np.where(k % 8 == 0, 1, 400 + k % 3),
            "dip_before_32": np.where(k % 32 == 31, 1, 400 + k % 7),
            "two_values": rng.integers(1, 3, size=n + 1),   # ties everywhere
        }
        for kind, d in shapes.items():
            out.append((f"{kind}_{n}", d.astype(np.int64) * 4096))
    return out


def test_solve_cubic_group_edges():
    """Every budget of many short chains: one call per length, the shapes side by side as a batch."""
    chains = group_edge_chains()
    for n in sorted({len(d) - 1 for _, d in chains}):
        say(f"solve_cubic group edges n={n}")
        check_cubic(np.stack([d for _, d in chains if len(d) - 1 == n], axis=1))


def test_solve_cubic_single_chain_configs():
    for name, d in (("config1", inputs.config1()), ("config2", inputs.config2())):
        say(f"solve_cubic {name}")
        check_cubic(d)


def test_solve_cubic_resnet1001():
    say("solve_cubic config4 (n=1001)")
    check_cubic(inputs.config4())


@pytest.mark.parametrize("batch,n,kind", [(64, 64, "log"), (200, 33, "ties"), (16, 64, "aligned"), (5, 130, "log")])
def test_solve_cubic_batches(batch, n, kind):
    say(f"solve_cubic batch={batch} n={n} {kind}")
    if kind == "log":
        d = inputs.log_uniform_chains(1, n, batch)
    elif kind == "aligned":
        d = inputs.uniform_aligned_chains(2, n, batch, 256, 32768)
    else:
        d = inputs.uniform_aligned_chains(5, n, batch, 1, 3, unit=1)
    check_cubic(d)
    check_cubic(d, chain_major=True)


def test_solve_cubic_batch_of_long_chains():
    """Chains long enough for the launch that lays out the budgets and builds the size stack's
    links together: several 32-bit chains, one that needs 64-bit arithmetic, one with a bad size."""
    n, batch = 1100, 5
    say(f"solve_cubic batch={batch} n={n} mixed")
    d = inputs.uniform_aligned_chains(7, n, batch, 256, 32768)
    d[:, 1] = inputs.log_uniform_chains(7, n, 1)[:, 0]
    d[700, 3] = -5
    good = [0, 1, 2, 4]
    want_peak, want_mask, want_s = oracle.batch_solve_static(inputs.chain_major(d[:, good]))
    for pruned in (False, True):
        if pruned:
            mask, peak, budget, evaluated, status = B.ckpt_solve_cubic_pruned(to_dev(d))
        else:
            mask, peak, budget, status = B.ckpt_solve_cubic(to_dev(d))
        torch.cuda.synchronize()
        assert np_(status).tolist() == [0, 0, 0, 3, 0]
        assert np_(peak)[3] == -1 and not np_(mask)[:, 3].any()
        assert np.array_equal(np_(peak)[good], want_peak), f"pruned={pruned}"
        assert np.array_equal(np_(budget)[good], want_s), f"pruned={pruned}"
        assert np.array_equal(np_(mask)[:, good].T, want_mask), f"pruned={pruned}"


def test_solve_cubic_data_errors():
    n, batch = 12, 4
    d = inputs.uniform_aligned_chains(3, n, batch, 1, 100, unit=1)
    d[5, 1] = 0
    d[:, 2] = (1 << 61)
    mask, peak, budget, status = B.ckpt_solve_cubic(to_dev(d))
    torch.cuda.synchronize()
    assert np_(status).tolist() == [0, 3, 4, 0]
    assert np_(peak)[1] == -1 and np_(peak)[2] == -1
    assert (np_(mask)[:, 1] == 0).all() and (np_(mask)[:, 2] == 0).all()
    for c in (0, 3):
        v, mk, s = oracle.solve_static(d[:, c])
        assert np_(peak)[c] == v and np_(budget)[c] == s and (np_(mask)[:, c] == mk).all()
    mask, peak, budget, evaluated, status = B.ckpt_solve_cubic_pruned(to_dev(d))
    assert np_(status).tolist() == [0, 3, 4, 0]
    assert np_(peak)[[1, 2]].tolist() == [-1, -1] and np_(evaluated)[[1, 2]].tolist() == [0, 0]
    for c in (0, 3):
        v, mk, s = oracle.solve_static(d[:, c])
        assert np_(peak)[c] == v and np_(budget)[c] == s and (np_(mask)[:, c] == mk).all()


def test_solve_cubic_pruned_runs_every_budget_of_shorter_chains():
    """Below 3072 layers pruning costs more than it saves: the call does not prune
    (a chain of 4096 layers, where it does, is in the full-size tests)."""
    n = 2500
    say(f"solve_cubic_pruned n={n}")
    d = inputs.config5_single(n)
    K = n * (n - 1) // 2 + 1
    mask, peak, budget, evaluated, status = B.ckpt_solve_cubic_pruned(to_dev(d))
    v, mk, s = oracle.solve_static(d[:, 0])
    assert int(peak[0]) == v and int(budget[0]) == s and (np_(mask)[:, 0] == mk).all()
    assert int(evaluated[0]) == K
    d = inputs.config4()
    _, _, _, evaluated, _ = B.ckpt_solve_cubic_pruned(to_dev(d))
    assert int(evaluated[0]) == 1001 * 1000 // 2 + 1


# ---------------------------------------------------------------------------
# the n = 12 configuration: every checkpoint set; the cost of every budget
# ---------------------------------------------------------------------------

def test_config1_every_subset_and_the_solvers_sets():
    """All 4096 masks over positions 1..12 with the ends forced (2048 distinct sets, each twice),
    evaluated in one call per objective against the oracle's objective functions; the least of
    them is what the two solvers return, and their sets evaluate to it."""
    d = inputs.config1()                                   # (13, 1)
    n = d.shape[0] - 1
    masks = np.zeros((n + 1, 4096), dtype=np.uint8)
    for bits in range(4096):
        for k in range(1, n + 1):
            masks[k, bits] = (bits >> (k - 1)) & 1
    masks[0, :] = 1
    masks[n, :] = 1
    dd = np.repeat(d, 4096, axis=1)
    best = {}
    for obj in (B.OBJ_STATIC, B.OBJ_DYNAMIC):
        peak, status = B.ckpt_eval_peak(to_dev(dd), to_dev(masks), obj)
        want = oracle.batch_peak(inputs.chain_major(dd), inputs.chain_major(masks), obj)
        assert (np_(status) == 0).all() and np.array_equal(np_(peak), want)
        best[obj] = int(np_(peak).min())
    smask, speak, sbudget, _ = B.ckpt_solve_cubic(to_dev(d))
    lmask, lpeak, _ = B.ckpt_solve_linear(to_dev(d))
    assert int(speak[0]) == best[B.OBJ_STATIC] and int(lpeak[0]) == best[B.OBJ_DYNAMIC]
    assert int(B.ckpt_eval_peak(to_dev(d), smask, B.OBJ_STATIC)[0][0]) == best[B.OBJ_STATIC]
    assert int(B.ckpt_eval_peak(to_dev(d), lmask, B.OBJ_DYNAMIC)[0][0]) == best[B.OBJ_DYNAMIC]
    assert int(speak[0]) == oracle.peak_static(d[:, 0], np_(smask)[:, 0])
    assert int(lpeak[0]) == oracle.peak_dynamic(d[:, 0], np_(lmask)[:, 0])


def check_budget_costs(d):
    """Every budget's cost s + c_s from the kernels that ckpt_solve_cubic runs, against the
    literal recurrence of Equation (T): the budgets must be the oracle's list as a multiset."""
    dc = inputs.chain_major(d)
    mask, peak, budget, budgets, costs, status = B.ckpt_solve_cubic_costs(to_dev(d))
    torch.cuda.synchronize()
    assert (np_(status) == 0).all()
    want_peak, want_mask, want_s = oracle.batch_solve_static(dc)
    assert np.array_equal(np_(peak), want_peak) and np.array_equal(np_(budget), want_s)
    assert np.array_equal(np_(mask).T, want_mask)
    gb, gc = np_(budgets), np_(costs)
    for c in range(dc.shape[0]):
        used = gb[c] >= 0
        assert (gc[c][~used] == -1).all()
        s, cost = gb[c][used], gc[c][used]
        order = np.argsort(s, kind="stable")
        want_list = np.sort(oracle.budgets(dc[c]))
        assert np.array_equal(s[order], want_list), f"chain {c}: budget list"
        # equal budgets have equal costs, so the order among them does not matter
        want_cost = want_list + oracle.static_cs_list(dc[c], want_list)
        assert np.array_equal(cost[order], want_cost), f"chain {c}: costs"
        assert int(cost.min()) == want_peak[c]


def test_cubic_cost_of_every_budget():
    say("cost of every budget: configs 1, 2, 4 and the group-edge chains")
    check_budget_costs(inputs.config1())
    check_budget_costs(inputs.config2())
    chains = group_edge_chains()
    for n in (40, 73, 105, 168):
        check_budget_costs(np.stack([d for _, d in chains if len(d) - 1 == n], axis=1))
    # chains that need 64-bit values, and a mixed batch
    check_budget_costs(inputs.log_uniform_chains(21, 33, 5))
    mixed = inputs.uniform_aligned_chains(22, 50, 6, 256, 32768)
    mixed[:, 1] += 1
    mixed[:, 4] = inputs.log_uniform_chains(23, 50, 1)[:, 0]
    check_budget_costs(mixed)


def test_cubic_cost_of_every_budget_resnet1001():
    say("cost of every budget: config 4 (n = 1001), a sample of 20,000 budgets against Equation (T)")
    d = inputs.config4()
    mask, peak, budget, budgets, costs, status = B.ckpt_solve_cubic_costs(to_dev(d))
    torch.cuda.synchronize()
    gb, gc = np_(budgets)[0], np_(costs)[0]
    used = gb >= 0
    assert int(used.sum()) == 1001 * 1000 // 2 + 1
    assert np.array_equal(np.sort(gb[used]), np.sort(oracle.budgets(d[:, 0])))
    rng = np.random.default_rng(3)
    pick = rng.choice(np.nonzero(used)[0], size=20000, replace=False)
    want = gb[pick] + oracle.static_cs_list(d[:, 0], gb[pick])
    assert np.array_equal(gc[pick], want)
    assert int(gc[used].min()) == int(peak[0])
