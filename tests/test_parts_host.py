"""CPU-only checks of the part-rotation planning helpers."""
import pytest

import paper_2008_12336_amd as G
from oracle import gosh_oracle as O


def test_pair_order_matches_oracle():
    for K in (1, 2, 3, 7, 20):
        assert G.gosh_pair_order(K) == O.pair_order(K)
    with pytest.raises(G.GoshError):
        G.gosh_pair_order(0)


def test_blocked_pair_order_matches_oracle():
    for K in (1, 2, 3, 7, 13, 20):
        for R in (1, 2, 3, 5, K, K + 2):
            assert G.gosh_pair_order_blocked(K, R) == O.pair_order_blocked(K, R)
    with pytest.raises(G.GoshError):
        G.gosh_pair_order_blocked(5, 0)


def test_plan_is_the_smallest_split_that_fits():
    n, d, B, P, S = 1_000_000, 128, 5, 3, 4

    def need(K):
        ps = -(-n // K)
        return min(P, K) * ps * d * 4 + S * 2 * ps * B * 4 + ((n + 63) // 64) * 8

    for budget in (need(1), need(1) - 1, need(4), need(4) + 5, need(9), 64 << 20):
        plan = G.gosh_parts_plan(n, d, 200, budget, P, S, B)
        K = plan["K"]
        assert plan["device_bytes"] == need(K) <= budget
        assert K == 1 or need(K - 1) > budget
        assert plan["rotations"] == O.rotations(200, B, K)
    with pytest.raises(G.GoshError, match="budget"):
        G.gosh_parts_plan(n, d, 200, 1000, P, S, B)
    with pytest.raises(G.GoshError):
        G.gosh_parts_plan(n, d, 200, 1 << 30, 1, S, B)  # fewer than two slots


def test_pair_level_rule():
    """gosh_pair_level_parts, the rule by which the multilevel drivers may train a resident
    level with Alg. 5 in place (the library's own, not the paper's, hence no oracle): largest
    K of 16, 8, 4, 2, 1 whose parts keep min_n vertices and whose whole rotations (B = 5)
    overshoot the level's epochs by at most an eighth; epochs that no K fits, and levels
    below min_n, keep Alg. 3."""
    unit = 1 << 20
    big = 16 * unit
    assert G.gosh_pair_level_parts(80, big, unit) == 16      # one rotation of 16 parts, exactly
    assert G.gosh_pair_level_parts(85, big, unit) == 2       # 16 -> 160, 8 -> 120, 4 -> 100; 2 -> 90 (5 over, <= 10)
    assert G.gosh_pair_level_parts(48, big, unit) == 2       # 16, 8 -> 80; 4 -> 60; 2 -> 50 (2 over, <= 6)
    assert G.gosh_pair_level_parts(10, big, unit) == 2
    assert G.gosh_pair_level_parts(8, big, unit) == 0        # K = 1 runs 10: 2 over, more than 8 / 8
    assert G.gosh_pair_level_parts(1000, big, unit) == 16    # 13 rotations = 1040: 40 over, <= 125
    assert G.gosh_pair_level_parts(80, big - 1, unit) == 8   # 16 parts would fall below 2^20 vertices
    assert G.gosh_pair_level_parts(80, 2 * unit, unit) == 2  # 80 epochs = 8 rotations of 2 parts
    assert G.gosh_pair_level_parts(80, unit - 1, unit) == 0  # level too small for even one part
    assert G.gosh_pair_level_parts(80, 3, 1) == 2            # never more parts than vertices
    for e in range(1, 400):
        for n in (unit, 5 * unit, big):
            K = G.gosh_pair_level_parts(e, n, unit)
            if K:
                assert K * unit <= n
                run = -(-e // (5 * K)) * 5 * K
                assert (run - e) * 8 <= e
            for larger in (16, 8, 4, 2, 1):
                if larger > K and larger * unit <= n:
                    over = -(-e // (5 * larger)) * 5 * larger - e
                    assert over * 8 > e


def test_tuning_record_round_trip():
    """gosh_set_tuning / gosh_get_tuning: defaults, a change, range checks, back to defaults."""
    defaults = G.gosh_tuning_defaults()
    assert defaults == dict(plain_rows=0, max_waves=1 << 18, hot_inv_eps=64, hot_all_inv_eps=4,
                            hot_min_degree=0, pair_level_min_n=1 << 22)
    assert G.gosh_get_tuning() == defaults
    try:
        G.gosh_set_tuning(hot_min_degree=17, hot_all_inv_eps=0)
        assert G.gosh_get_tuning() == dict(defaults, hot_min_degree=17, hot_all_inv_eps=0)
        for bad in (dict(max_waves=0), dict(hot_inv_eps=0), dict(hot_all_inv_eps=-1),
                    dict(hot_min_degree=-2), dict(pair_level_min_n=0)):
            with pytest.raises(G.GoshError):
                G.gosh_set_tuning(**bad)
            assert G.gosh_get_tuning()["hot_min_degree"] == 17  # a refused record changes nothing
        with pytest.raises(TypeError):
            G.gosh_set_tuning(no_such_field=1)
    finally:
        G.gosh_set_tuning()
    assert G.gosh_get_tuning() == defaults
