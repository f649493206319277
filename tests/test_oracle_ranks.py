"""Pins for the oracle's sequential budgeted rank selection (Sec. 3.5, App. B
Alg. 2): budget invariants, degenerate cases with a known answer, and an
independent re-statement of the greedy rule checked on exhaustive small cases."""
import itertools

import numpy as np

from oracle import skv_oracle as O


def _monotone_surface(rng, L, ck, cv, d):
    """Error falls as ranks grow; zero at full rank (App. B: Delta(d_h, d_h) = 0)."""
    s = np.empty((L, len(ck), len(cv)))
    for l in range(L):
        a, b = rng.uniform(0.5, 2.0, 2)
        for i, rk in enumerate(ck):
            for j, rv in enumerate(cv):
                s[l, i, j] = a * (1 - rk / d) + b * (1 - rv / d) ** 2
    return s


def test_first_allowance_is_rho_and_total_cost_within_budget():
    rng = np.random.default_rng(0)
    d, L = 128, 32
    ck = cv = [64, 80, 96, 112, 128]
    for rho in (0.5, 0.6, 0.7, 0.8, 0.9, 1.0):
        delta = _monotone_surface(rng, L, ck, cv, d)
        rk, rv, achieved, feasible = O.layer_ranks(L, d, rho, ck, cv, delta)
        assert feasible
        # tau_1 = B_1 / L = rho: the first layer's cost may not exceed rho
        assert (rk[0] + rv[0]) / (2 * d) <= rho + 1e-12
        # c_l <= B_l / (L-l+1) at every layer keeps the balance non-negative
        assert achieved <= rho + 1e-12
        assert abs(achieved - sum(a + b for a, b in zip(rk, rv)) / (2 * d * L)) < 1e-15


def test_full_budget_keeps_every_layer_full_rank():
    rng = np.random.default_rng(1)
    d, L = 128, 8
    ck = cv = [64, 96, 128]
    delta = _monotone_surface(rng, L, ck, cv, d) + 1e-3
    delta[:, -1, -1] = 0.0
    rk, rv, achieved, feasible = O.layer_ranks(L, d, 1.0, ck, cv, delta)
    assert rk == [128] * L and rv == [128] * L and achieved == 1.0 and feasible


def test_identical_surfaces_on_grid_budget_give_uniform_allocation():
    d, L = 128, 6
    ck = cv = [32, 64, 96, 128]
    one = np.array([[1 - (a + b) / (2 * d) + 0.01 * (a < b) for b in cv] for a in ck])
    delta = np.tile(one[None], (L, 1, 1))
    rk, rv, achieved, feasible = O.layer_ranks(L, d, 0.5, ck, cv, delta)
    assert feasible and achieved == 0.5
    assert len(set(zip(rk, rv))) == 1


def test_unspent_allowance_rolls_forward():
    # layer 1 is indifferent (zero error everywhere) so it takes the cheapest pair;
    # the saved budget lets layer 2 afford more than rho.
    d, L = 128, 2
    ck = cv = [32, 128]
    delta = np.zeros((L, 2, 2))
    delta[1] = [[3.0, 2.0], [1.5, 0.0]]
    rk, rv, achieved, feasible = O.layer_ranks(L, d, 0.625, ck, cv, delta)
    assert (rk[0], rv[0]) == (32, 32)            # equal errors -> lower cost
    assert (rk[1], rv[1]) == (128, 128)          # 2*0.625 - 0.25 = 1.0 is now affordable
    assert feasible and achieved == 0.625


def test_equal_error_equal_cost_prefers_larger_value_rank():
    d, L = 128, 1
    delta = np.full((1, 2, 2), 1.0)
    rk, rv, _, _ = O.layer_ranks(L, d, 0.75, [64, 128], [64, 128], delta)
    assert (rk[0], rv[0]) == (64, 64)            # lower cost first
    delta[0, 0, 0] = 2.0
    rk, rv, _, _ = O.layer_ranks(L, d, 0.75, [64, 128], [64, 128], delta)
    assert (rk[0], rv[0]) == (64, 128)           # cost tie 192: larger r_V


def test_infeasible_budget_takes_cheapest_pair_and_reports_it():
    d, L = 128, 3
    ck = cv = [64, 128]
    delta = np.array([[[0.5, 0.2], [0.3, 0.0]]] * L)
    rk, rv, achieved, feasible = O.layer_ranks(L, d, 0.4, ck, cv, delta)
    assert not feasible
    assert rk == [64] * L and rv == [64] * L and achieved == 0.5


def _greedy_restated(L, d, rho, ck, cv, delta):
    """Second statement of Alg. 2 in normalised units with exact rationals."""
    from fractions import Fraction
    B = Fraction(rho).limit_denominator(10 ** 6) * L
    out = []
    for l in range(1, L + 1):
        tau = B / (L - l + 1)
        feas = [(delta[l - 1, i, j], Fraction(rk + rv, 2 * d), -rv, i * len(cv) + j, rk, rv)
                for i, rk in enumerate(ck) for j, rv in enumerate(cv)
                if Fraction(rk + rv, 2 * d) <= tau]
        assert feas
        best = min(feas)
        out.append((best[4], best[5]))
        B -= Fraction(best[4] + best[5], 2 * d)
    return out


def test_greedy_rule_against_exact_rational_restatement():
    rng = np.random.default_rng(5)
    d = 128
    ck, cv = [32, 64, 128], [48, 96, 128]
    for trial in range(200):
        L = int(rng.integers(1, 6))
        rho = float(rng.choice([0.5, 0.5625, 0.625, 0.75, 0.875, 1.0]))
        delta = rng.integers(0, 6, size=(L, 3, 3)).astype(float)   # many ties on purpose
        rk, rv, _, feasible = O.layer_ranks(L, d, rho, ck, cv, delta)
        assert feasible
        assert list(zip(rk, rv)) == _greedy_restated(L, d, rho, ck, cv, delta)


def test_sequential_choice_differs_from_static_per_layer_choice():
    # exhaustive L=3, 2x2 candidates: the greedy pick at each layer is the best
    # pair affordable under the *running* allowance, not under rho alone
    d, L = 128, 3
    ck = cv = [64, 128]
    rng = np.random.default_rng(9)
    seen_rollover = False
    for trial in range(300):
        delta = rng.uniform(0, 1, (L, 2, 2))
        rho = 0.75
        rk, rv, achieved, feasible = O.layer_ranks(L, d, rho, ck, cv, delta)
        B = L * rho
        for l in range(L):
            tau = B / (L - l)
            opts = [(delta[l, i, j], a, b) for i, a in enumerate(ck) for j, b in enumerate(cv)
                    if (a + b) / (2 * d) <= tau + 1e-12]
            assert (rk[l], rv[l]) == min(opts)[1:]
            if (rk[l] + rv[l]) / (2 * d) > rho:
                seen_rollover = True
            B -= (rk[l] + rv[l]) / (2 * d)
        assert achieved <= rho + 1e-12
    assert seen_rollover
