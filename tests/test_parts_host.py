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
