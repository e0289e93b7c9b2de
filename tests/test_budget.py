"""Draft budget helper (Sec. 3.1): closed forms on synthetic latency curves (no GPU)."""
import pytest

from paper_2503_00784_amd import budget


def test_flat_curve_gives_floor_of_cost_coefficient():
    # T_target flat at 30 ms, T_draft 1.25 ms: c = 24, the budget the paper reports for its machine
    curve = [(2, 30.0), (4, 30.0), (8, 30.0), (16, 30.0), (32, 30.0)]
    assert budget.cost_coefficient(curve, 1.25)[8] == pytest.approx(24.0)
    assert budget.draft_budget(curve, 1.25, k_max=64) == 24
    assert budget.draft_budget(curve, 1.25) == 24  # within the measured range


def test_budget_is_capped_by_search_range_and_at_least_one():
    curve = [(2, 3.0), (16, 3.0)]
    assert budget.draft_budget(curve, 0.1) == 16  # c = 30 but nothing beyond k = 16 was measured
    assert budget.draft_budget(curve, 0.1, k_max=64) == 30
    assert budget.draft_budget(curve, 10.0) == 1  # a draft step slower than the whole pass


def test_rising_curve_fixed_point():
    # T(k) = 2 + 0.1 k, T_draft = 0.5: k * 0.5 <= 2 + 0.1 k  <=>  k <= 5
    curve = [(1, 2.1), (11, 3.1)]
    assert budget.interpolate_latency(curve, 6) == pytest.approx(2.6)
    assert budget.draft_budget(curve, 0.5) == 5


def test_invalid_inputs():
    with pytest.raises(ValueError):
        budget.draft_budget([(1, 1.0)], 0.0)
    with pytest.raises(ValueError):
        budget.interpolate_latency([], 1)
