"""Pins for the oracle's solvers of eq. (ip) (Sec. 2.1): itertools brute force on tiny
instances, the invariances the paper states (affine change of the gain, Sec. 2.3.2), the
budget end points (tau = 0 -> all high precision; large tau -> every group's best gain,
Sec. 3.2) and the J = L special case."""
import itertools

import numpy as np
import pytest

import oracle


def brute(n_choices, gain, mse, budget):
    off = np.concatenate([[0], np.cumsum(n_choices)])
    best = None
    for combo in itertools.product(*[range(n) for n in n_choices]):
        g = sum(gain[off[j] + p] for j, p in enumerate(combo))
        d = sum(mse[off[j] + p] for j, p in enumerate(combo))
        if d <= budget and (best is None or g > best[0]):
            best = (g, d, combo)
    return best


def random_instance(rng, J, max_choices=5, zero_first=True):
    n_choices = rng.integers(1, max_choices + 1, J).astype(np.int32)
    gain = rng.uniform(0, 10, n_choices.sum())
    mse = rng.uniform(0, 1, n_choices.sum())
    if zero_first:
        off = np.concatenate([[0], np.cumsum(n_choices)])[:-1]
        gain[off] = 0.0
        mse[off] = 0.0
    return n_choices, gain, mse


@pytest.mark.parametrize("seed", range(40))
def test_exhaustive_and_pareto_match_brute_force(seed):
    rng = np.random.default_rng(seed)
    J = int(rng.integers(1, 7))
    n_choices, gain, mse = random_instance(rng, J)
    budget = float(rng.uniform(0, mse.sum() * 0.6))
    want = brute(n_choices, gain, mse, budget)
    for solver in (oracle.select_exhaustive, oracle.select_pareto):
        rc, choice, tg, td = solver(n_choices, gain, mse, budget)
        assert rc == 0
        assert tg == pytest.approx(want[0], rel=1e-12, abs=1e-12)
        off = np.concatenate([[0], np.cumsum(n_choices)])[:-1]
        assert np.all((choice >= 0) & (choice < n_choices))          # exactly one choice per group
        assert gain[off + choice].sum() == pytest.approx(tg, rel=1e-12, abs=1e-12)
        assert mse[off + choice].sum() == pytest.approx(td, rel=1e-12, abs=1e-12)
        assert td <= budget


def test_infeasible_and_end_points():
    n_choices = np.array([2, 3], dtype=np.int32)
    gain = np.array([1.0, 2.0, 0.5, 4.0, 3.0])
    mse = np.array([0.5, 1.0, 0.4, 2.0, 1.0])
    assert oracle.select_exhaustive(n_choices, gain, mse, 0.8)[0] == 6
    assert oracle.select_pareto(n_choices, gain, mse, 0.8)[0] == 6
    # zero budget with a free high-precision column: all choice 0
    rng = np.random.default_rng(0)
    n_choices, gain, mse = random_instance(rng, 5)
    mse[mse == 0] = 0.0
    pos = mse > 0
    mse[pos] += 0.01
    for solver in (oracle.select_exhaustive, oracle.select_pareto):
        rc, choice, tg, td = solver(n_choices, gain, mse, 0.0)
        assert rc == 0 and np.all(choice == 0) and tg == 0.0 and td == 0.0
        rc, choice, tg, td = solver(n_choices, gain, mse, mse.sum() + 1)
        off = np.concatenate([[0], np.cumsum(n_choices)])
        want = sum(gain[off[j]:off[j + 1]].max() for j in range(5))
        assert rc == 0 and tg == pytest.approx(want, rel=1e-12)


@pytest.mark.parametrize("seed", range(10))
def test_affine_gain_invariance_and_budget_monotonicity(seed):
    rng = np.random.default_rng(100 + seed)
    n_choices, gain, mse = random_instance(rng, 5)
    budget = float(mse.sum() * 0.3)
    rc, choice, tg, td = oracle.select_exhaustive(n_choices, gain, mse, budget)
    # c -> a*c + b_j (a > 0, b_j constant within group j) leaves the arg max unchanged
    a = 3.7
    b = np.repeat(rng.uniform(-5, 5, 5), n_choices)
    rc2, choice2, tg2, td2 = oracle.select_exhaustive(n_choices, a * gain + b, mse, budget)
    off = np.concatenate([[0], np.cumsum(n_choices)])[:-1]
    assert gain[off + choice2].sum() == pytest.approx(tg, rel=1e-12)
    # the optimum never decreases with the budget
    prev = -np.inf
    for bud in np.linspace(0, mse.sum(), 9):
        rc, _, g, _ = oracle.select_pareto(n_choices, gain, mse, float(bud))
        assert rc == 0 and g >= prev - 1e-12
        prev = g


def test_tie_break_prefers_smaller_mse_then_lexicographic():
    n_choices = np.array([2, 2], dtype=np.int32)
    gain = np.array([0.0, 1.0, 0.0, 1.0])
    mse = np.array([0.0, 0.5, 0.0, 0.25])
    rc, choice, tg, td = oracle.select_exhaustive(n_choices, gain, mse, 0.5)   # only one fits
    assert (rc, list(choice), tg, td) == (0, [0, 1], 1.0, 0.25)
    mse = np.array([0.0, 0.5, 0.0, 0.5])
    rc, choice, tg, td = oracle.select_exhaustive(n_choices, gain, mse, 0.5)
    assert (rc, list(choice)) == (0, [0, 1])


def test_single_layer_groups_special_case():
    # J = L, one layer per group, F = 2: a plain 0/1 knapsack
    n_choices = np.full(6, 2, dtype=np.int32)
    w = np.array([3.0, 4.0, 5.0, 9.0, 4.0, 2.0])
    v = np.array([3.0, 4.0, 4.0, 10.0, 4.0, 1.5])
    gain = np.stack([np.zeros(6), v], axis=1).reshape(-1)
    mse = np.stack([np.zeros(6), w], axis=1).reshape(-1)
    rc, choice, tg, td = oracle.select_pareto(n_choices, gain, mse, 11.0)
    assert rc == 0 and tg == 11.5 and td == 11.0 and list(choice) == [0, 0, 0, 1, 0, 1]
