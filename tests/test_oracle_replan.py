"""Pins for the checker's online re-planning of shares (Sec. III-C phase 1)."""
import pytest

import oracle


def simulate(true_thr, B, alpha, steps, start=None):
    K = len(true_thr)
    shares = start or oracle.plan_shares([1.0] * K, B)
    ema = [0.0] * K
    hist = []
    for _ in range(steps):
        times = [b / s if b else 0.0 for b, s in zip(shares, true_thr)]
        ema, shares = oracle.replan_shares(times, shares, ema, alpha, B)
        hist.append(list(shares))
    return hist, ema


def test_replan_reaches_the_static_plan():
    thr = [1.0, 1.0, 0.7, 0.7, 0.5, 0.5, 0.3, 0.3]
    target = oracle.plan_shares(thr, 2048)
    # constant speeds: the very first measurement already gives the exact time per sample
    hist, ema = simulate(thr, 2048, 0.3, 5)
    assert all(h == target for h in hist)
    for e, s in zip(ema, thr):
        assert abs(e * s - 1.0) < 1e-12
    # devices that never processed a sample have no estimate yet -> error
    with pytest.raises(ValueError):
        simulate(thr, 2048, 1.0, 2, start=[2048, 0, 0, 0, 0, 0, 0, 0])
    with pytest.raises(ValueError):
        oracle.replan_shares([1.0, 0.0], [10, 0], [0.0, 0.0], 0.5, 10)
    # alpha = 1 forgets the past at once
    e, s = oracle.replan_shares([10.0, 40.0], [10, 10], [5.0, 5.0], 1.0, 20)
    assert e == [1.0, 4.0] and s == [16, 4]


def test_replan_follows_a_slowdown_monotonically():
    B = 1024
    ema = [0.0, 0.0]
    shares = [512, 512]
    ema, shares = oracle.replan_shares([512.0, 512.0], shares, ema, 0.5, B)
    assert shares == [512, 512]
    prev = shares[1]
    for _ in range(12):          # device 1 now runs at half speed
        times = [shares[0] / 1.0, shares[1] / 0.5]
        ema, shares = oracle.replan_shares(times, shares, ema, 0.5, B)
        assert sum(shares) == B and shares[1] <= prev
        prev = shares[1]
    assert shares == oracle.plan_shares([1.0, 0.5], B)
    # the moving average is the textbook recurrence
    e, _ = oracle.replan_shares([3.0], [2], [1.0], 0.25, 4)
    assert e == [0.25 * 1.5 + 0.75 * 1.0]
    e, _ = oracle.replan_shares([3.0], [2], [0.0], 0.25, 4)
    assert e == [1.5]
    e, s = oracle.replan_shares([3.0, 7.0], [2, 0], [1.0, 2.0], 0.25, 6)
    assert e[1] == 2.0 and sum(s) == 6


def test_replan_rejects_bad_input():
    for args in (([1.0], [1], [0.0], 0.0, 4), ([1.0], [1], [0.0], 1.5, 4), ([0.0], [1], [0.0], 0.5, 4),
                 ([float("nan")], [1], [1.0], 0.5, 4), ([1.0, 1.0], [1], [0.0], 0.5, 4)):
        with pytest.raises(ValueError):
            oracle.replan_shares(*args)
