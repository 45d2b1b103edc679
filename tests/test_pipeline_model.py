"""Pins of the analytic pipeline model (paper Sections 3.2 and 3.4) against what the equations fix: the sum that
defines Eq. 5, the limits the paper states, Eq. 10, and a Monte-Carlo run of the two-case process."""
import numpy as np
import pytest

from paper_2603_19133_amd import pipeline_model as pm


@pytest.mark.parametrize("alpha", [0.0, 0.3, 0.8, 0.97, 1.0])
@pytest.mark.parametrize("gamma", [1, 4, 6, 16])
def test_expected_length_is_the_sum_it_abbreviates(alpha, gamma):
    p = pm.length_distribution(alpha, gamma)
    assert p.sum() == pytest.approx(1.0, abs=1e-12)
    assert pm.expected_length(alpha, gamma) == pytest.approx(float((np.arange(1, gamma + 1) * p).sum()), rel=1e-12)


def test_limits_of_the_expected_length():
    assert pm.expected_length(1.0, 5) == 5 and pm.expected_length(0.0, 5) == 1
    assert pm.expected_length(1 - 1e-9, 5) == pytest.approx(5, rel=1e-6)
    assert pm.expected_length(0.8, 4) == pytest.approx(1 + 0.8 + 0.64 + 0.512)


def test_cycle_times_and_bubble():
    assert pm.latency_sync(30e-3, 40e-3, 20e-3) == pytest.approx(90e-3)
    assert pm.latency_async_full_hit(30e-3, 40e-3, 20e-3) == pytest.approx(60e-3)     # network-bound
    assert pm.latency_async_full_hit(80e-3, 40e-3, 20e-3) == pytest.approx(80e-3)     # draft-bound: the round trip is hidden
    assert pm.bubble(30e-3, 40e-3, 20e-3) == pytest.approx(30e-3)
    assert pm.bubble(30e-3, 40e-3, 20e-3, t_pre=25e-3) == pytest.approx(5e-3)
    assert pm.bubble(80e-3, 40e-3, 20e-3) == 0.0


@pytest.mark.parametrize("alpha", [0.0, 0.2, 0.6, 0.9, 0.999])
def test_speedup_bounds_and_limit(alpha):
    """S >= 1 for every alpha (the paper's robustness bound), S -> 1 for alpha -> 0, and Eq. 10 for alpha -> 1 in the
    draft-bound regime."""
    td, tr, tv, g = 80e-3, 40e-3, 20e-3, 5
    s = pm.speedup(alpha, g, td, tr, tv)
    assert 1.0 - 1e-12 <= s <= pm.speedup_limit(td, tr, tv) + 1e-12
    assert pm.speedup(0.0, g, td, tr, tv) == pytest.approx(1.0)
    assert pm.speedup(1.0, g, td, tr, tv) == pytest.approx(pm.speedup_limit(td, tr, tv)) == pytest.approx(1.75)
    # network-bound: the overlap hides the draft instead, the limit is below Eq. 10's
    assert pm.speedup(1.0, g, 30e-3, tr, tv) == pytest.approx(90 / 60)


def test_throughput_formulas():
    a, g, td, tr, tv = 0.85, 4, 50e-3, 30e-3, 25e-3
    el = (1 - a ** g) / (1 - a)
    assert pm.throughput_sync(a, g, td, tr, tv) == pytest.approx(el / (td + tr + tv))
    et = a ** g * max(td, tr + tv) + (1 - a ** g) * (td + tr + tv)
    assert pm.expected_time_async(a, g, td, tr, tv) == pytest.approx(et)
    assert pm.throughput_async(a, g, td, tr, tv) == pytest.approx(el / et)


def test_monte_carlo_of_the_two_case_process():
    rng = np.random.default_rng(260319133)
    a, g, td, tr, tv = 0.9, 6, 60e-3, 35e-3, 15e-3
    tokens, rate = pm.simulate(a, g, td, tr, tv, 400000, rng)
    assert tokens == pytest.approx(pm.expected_length(a, g), rel=5e-3)
    assert rate == pytest.approx(pm.throughput_async(a, g, td, tr, tv), rel=5e-3)


def test_sampling_share_and_truncation():
    # 4.25 M positions/s (one MI355X, measured): a gamma = 16 draft of 256 sequences costs about a millisecond
    assert pm.sampling_time(256 * 16, 4.25e6) == pytest.approx(0.964e-3, rel=1e-3)
    rng = np.random.default_rng(3)
    g = pm.truncated_gammas(16, 5e-3, 0.5, 60e-3, 20000, rng)
    assert g.min() >= 1 and g.max() <= 16 and 6 < g.mean() < 10 and len(np.unique(g)) > 5     # ragged lengths
    assert np.all(pm.truncated_gammas(16, 5e-3, 0.0, 1.0, 10, rng) == 16)                      # no pressure: whole drafts
    assert np.all(pm.truncated_gammas(16, 5e-3, 0.0, 12e-3, 10, rng) == 2)
