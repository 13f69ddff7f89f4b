"""Host-side key-layer selection (which layers get a second INT4 tensor)."""
from paper_1902_06822_amd import select


def test_top_fraction_on_a_hand_built_example():
    nmse = [0.010, 0.200, 0.030, 0.200, 0.001, 0.050, 0.0, 0.049, 0.2, 0.02]
    assert select.select_top_fraction(nmse, 0.10) == [1]                  # tie 1/3/8 -> lowest index
    assert select.select_top_fraction(nmse, 0.30) == [1, 3, 8]
    assert select.select_top_fraction(nmse, 0.50) == [1, 3, 5, 7, 8]
    assert select.select_top_fraction(nmse, 0.0) == [1]                   # at least one layer
    assert select.select_top_fraction(nmse, 1.0) == list(range(10))
    assert select.select_top_fraction([0.1] * 54, 0.10) == [0, 1, 2, 3, 4]  # round(5.4) = 5 of 54
    assert select.select_top_fraction([], 0.1) == []


def test_threshold_rule_of_the_paper():
    mse = [1e-5, 9e-5, 8e-5, 2e-4]
    assert select.select_above_threshold(mse, 8e-5) == [1, 3]


def test_normalized_mse():
    assert select.normalized_mse([1.0, 0.0, 3.0], [4.0, 0.0, 6.0]) == [0.25, 0.0, 0.5]
