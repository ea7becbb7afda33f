"""Pins for the oracle's greedy bit allocator (Sec. 4.2 Prob. (9), Sec. 4.3).

What can be pinned without another implementation: feasibility, the start at 8 bits,
monotonicity in the sensitivity, the prefix structure of the applied moves, and -- by
exhaustive search on small problems -- that the greedy answer is optimal for the number
of bits it actually spends (each item's cost is convex along the ladder 8->4->2->1, so a
cheapest-move-first prefix minimises the Lagrangian).  Optimality for an arbitrary
budget is not claimed by the paper (it calls the method a heuristic) and is unpinned.
"""
import itertools

import numpy as np
import pytest

import oracle

LADDER = (1, 2, 4, 8)


def _cost(w, bits):
    B = (2.0 ** np.asarray(bits, dtype=np.float64)) - 1
    return float((np.asarray(w, dtype=np.float64) / (B * B)).sum())


def test_loose_budget_keeps_eight_bits():
    w = np.array([1.0, 5.0, 0.1], dtype=np.float32)
    D = np.array([100, 200, 300], dtype=np.int64)
    assert list(oracle.allocate_bits(w, D, 8 * 600)) == [8, 8, 8]
    assert list(oracle.allocate_bits(w, D, 10 ** 9)) == [8, 8, 8]


def test_budget_below_one_bit_per_element_is_infeasible():
    w = np.ones(4, dtype=np.float32)
    D = np.full(4, 256, dtype=np.int64)
    assert list(oracle.allocate_bits(w, D, 4 * 256)) == [1, 1, 1, 1]
    with pytest.raises(oracle.OracleError) as e:
        oracle.allocate_bits(w, D, 4 * 256 - 1)
    assert e.value.code == oracle.EINFEASIBLE


def test_bad_arguments_are_rejected():
    D = np.full(2, 8, dtype=np.int64)
    for w in ([-1.0, 1.0], [np.nan, 1.0], [np.inf, 1.0]):
        with pytest.raises(oracle.OracleError) as e:
            oracle.allocate_bits(np.array(w, dtype=np.float32), D, 100)
        assert e.value.code == oracle.EINVAL
    with pytest.raises(oracle.OracleError):
        oracle.allocate_bits(np.ones(2, dtype=np.float32), np.array([8, 0], dtype=np.int64), 100)


@pytest.mark.parametrize("seed", range(6))
def test_feasible_monotone_and_tight(seed):
    rng = np.random.default_rng(seed)
    M = 200
    w = rng.lognormal(0, 2, M).astype(np.float32)
    D = np.full(M, 4096, dtype=np.int64)
    avg = rng.uniform(1.0, 7.5)
    budget = int(avg * D.sum())
    bits = oracle.allocate_bits(w, D, budget).astype(np.int64)
    assert set(bits) <= set(LADDER)
    used = int((bits * D).sum())
    assert used <= budget
    # equal sizes: a more sensitive item never gets fewer bits
    order = np.argsort(w, kind="stable")
    assert np.all(np.diff(bits[order]) >= 0)
    # tight: the budget could not have been met with one move fewer -- raising any item
    # that was lowered back by one rung frees... i.e. costs more bits than the slack left
    slack = budget - used
    lowered = bits < 8
    assert lowered.any()
    assert slack < (bits[lowered] * D[lowered]).max()  # a rung up costs b*D bits (b -> 2b)


@pytest.mark.parametrize("seed", range(5))
def test_applied_moves_form_a_cheapest_first_prefix(seed):
    """Every applied move is no dearer (per bit freed) than every move left unapplied."""
    rng = np.random.default_rng(100 + seed)
    M = 60
    w = rng.lognormal(0, 1.5, M)
    D = rng.choice([256, 1024, 4096, 25088], M).astype(np.int64)
    budget = int(rng.uniform(1.2, 6.0) * D.sum())
    bits = oracle.allocate_bits(w.astype(np.float32), D, budget)
    w32 = w.astype(np.float32).astype(np.float64)

    def price(i, b_from):           # variance added per bit freed by b_from -> b_from/2
        Bo, Bn = 2.0 ** b_from - 1, 2.0 ** (b_from // 2) - 1
        return w32[i] * (1 / Bn ** 2 - 1 / Bo ** 2) / (D[i] * (b_from - b_from // 2))

    applied = [price(i, b) for i in range(M) for b in (8, 4, 2) if bits[i] < b]
    pending = [price(i, b) for i in range(M) for b in (8, 4, 2) if bits[i] >= b]
    assert applied and pending
    assert max(applied) <= min(pending) * (1 + 1e-12)
    # and the dearest applied move was needed
    i_last = max(((price(i, b), i, b) for i in range(M) for b in (8, 4, 2) if bits[i] < b))
    undo = (bits.astype(np.int64) * D).sum() + D[i_last[1]] * (i_last[2] - i_last[2] // 2)
    assert undo > budget


@pytest.mark.parametrize("seed", range(8))
def test_optimal_for_the_bits_it_spends_by_exhaustive_search(seed):
    rng = np.random.default_rng(200 + seed)
    M = 6
    w = rng.lognormal(0, 1.5, M).astype(np.float32)
    D = rng.choice([8, 16, 24, 40], M).astype(np.int64)
    budget = int(rng.uniform(1.1, 7.0) * D.sum())
    bits = oracle.allocate_bits(w, D, budget)
    used = int((bits.astype(np.int64) * D).sum())
    mine = _cost(w, bits)
    assert abs(mine - oracle.objective(w, bits)) <= 1e-12 * max(1.0, mine)
    best = min(_cost(w, c) for c in itertools.product(LADDER, repeat=M)
               if int((np.array(c) * D).sum()) <= used)
    assert mine <= best * (1 + 1e-12)
    # for the real budget the exact optimum (what the paper's DP would return) can only be
    # better or equal; record that the greedy gap is bounded by the last unapplied move
    exact = min(_cost(w, c) for c in itertools.product(LADDER, repeat=M)
                if int((np.array(c) * D).sum()) <= budget)
    assert exact <= mine * (1 + 1e-12)


def test_ties_go_to_the_lowest_index():
    w = np.ones(4, dtype=np.float32)
    D = np.full(4, 10, dtype=np.int64)
    # one move needed: item 0 goes 8 -> 4
    assert list(oracle.allocate_bits(w, D, 8 * 40 - 1)) == [4, 8, 8, 8]
    # zero sensitivities: all prices are 0, item 0 is driven all the way down first
    z = np.zeros(3, dtype=np.float32)
    assert list(oracle.allocate_bits(z, np.full(3, 10, dtype=np.int64), 8 * 30 - 41)) == [2, 8, 8]
    assert list(oracle.allocate_bits(z, np.full(3, 10, dtype=np.int64), 8 * 30 - 70)) == [1, 8, 8]
    assert list(oracle.allocate_bits(z, np.full(3, 10, dtype=np.int64), 8 * 30 - 71)) == [1, 4, 8]


def test_tiered_sensitivities_give_the_intended_multiset():
    """The synthetic recipe used for the mixed-width workloads: decades of sensitivity
    make the allocator return exactly the requested widths at a 2.0-bit average."""
    from paper_2104_14129_amd import synth
    wl = synth.r50_stage1()
    w = synth.tiered_sensitivities(wl.bits, seed=7)
    D = np.full(wl.N, wl.D, dtype=np.int64)
    bits = oracle.allocate_bits(w, D, 2 * wl.N * wl.D)
    assert np.array_equal(bits, wl.bits)
    assert bits.astype(np.float64).mean() == 2.0
