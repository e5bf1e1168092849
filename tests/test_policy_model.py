"""Checkpointing policy helpers beyond the window search (CPU only): App. B popularity variants,
the ETTR model of Sec. 2.4 / App. C and the recovery bounds of Sec. 3.6 — oracle pinned to closed
forms, library compared with the oracle."""
import math
from fractions import Fraction

import numpy as np
import pytest

from paper_2412_15411_amd import binding as B


def test_time_decayed_popularity_closed_forms(orc):
    """A(t) = a A(t-1) + (1-a) c: a = 0 gives the batch counts, a = 1 keeps the past, and a constant
    batch count c from A(0) = 0 gives c (1 - a^t)."""
    prev, cnt = [3.0, 0.0, 10.0], [1.0, 4.0, 10.0]
    assert orc.popularity_time_decayed(0.0, prev, cnt) == cnt
    assert orc.popularity_time_decayed(1.0, prev, cnt) == prev
    a, c = 0.9, [7.0, 0.5, 120.0]
    state = [0.0] * 3
    for t in range(1, 40):
        state = orc.popularity_time_decayed(a, state, c)
        for s, ci in zip(state, c):
            assert s == pytest.approx(ci * (1 - a ** t), rel=1e-12)
    rng = np.random.default_rng(0)
    for _ in range(20):
        n = int(rng.integers(1, 30))
        p, q, alpha = rng.random(n) * 100, rng.random(n) * 100, float(rng.random())
        assert B.moev_popularity_time_decayed(alpha, list(p), list(q)) == pytest.approx(
            orc.popularity_time_decayed(alpha, list(p), list(q)), rel=1e-15)
    with pytest.raises(B.MoevError):
        B.moev_popularity_time_decayed(1.5, prev, cnt)


def test_capacity_aware_popularity_changes_the_order(orc):
    """App. B: popularity normalised by capacity; an expert with many tokens but a large capacity is
    checkpointed earlier than its raw count suggests."""
    pop, cap = [100.0, 60.0, 80.0, 10.0], [4.0, 1.0, 2.0, 1.0]
    norm = orc.popularity_capacity_aware(pop, cap)
    assert norm == [25.0, 60.0, 40.0, 10.0]
    assert B.moev_popularity_capacity_aware(pop, cap) == norm
    assert orc.order_by_popularity(pop) == [3, 1, 2, 0]
    assert orc.order_by_popularity(norm) == B.moev_order_operators(norm) == [3, 0, 2, 1]
    with pytest.raises(B.MoevError):
        B.moev_popularity_capacity_aware(pop, [1.0, 0.0, 1.0, 1.0])


def test_ettr_formula(orc):
    """Sec. 2.4: ETTR = 1/(1 + T_ckpt/(T_iter I)) * 1/(1 + E[R]/MTBF), against exact rational arithmetic."""
    assert orc.ettr(0.0, 1.0, 10.0, 0.0, 600.0) == 1.0
    rng = np.random.default_rng(1)
    for _ in range(200):
        t_ckpt, t_iter, interval, er, mtbf = (float(x) for x in rng.uniform(0.01, 50, size=5))
        mtbf *= 100
        exact = 1 / (1 + Fraction(t_ckpt) / (Fraction(t_iter) * Fraction(interval))) * 1 / (1 + Fraction(er) / Fraction(mtbf))
        assert orc.ettr(t_ckpt, t_iter, interval, er, mtbf) == pytest.approx(float(exact), rel=1e-14)
        assert B.moev_ettr(t_ckpt, t_iter, interval, er, mtbf) == pytest.approx(float(exact), rel=1e-14)
    assert math.isnan(B.moev_ettr(1.0, 0.0, 1.0, 1.0, 1.0))


def test_ettr_optimal_dense_interval_matches_daly(orc):
    """With E[R] = interval * T_iter / 2 (Sec. 3.6) the model has an interior optimum; to first order it
    is Young/Daly's sqrt(2 * T_ckpt * MTBF) (the trade-off Sec. 2.4 describes)."""
    t_iter, t_ckpt, mtbf = 2.0, 30.0, 3600.0
    best = max(range(1, 2000), key=lambda i: orc.ettr(t_ckpt, t_iter, i, orc.recovery("dense", i, t_iter)[0], mtbf))
    daly = math.sqrt(2 * t_ckpt * mtbf) / t_iter
    assert abs(best - daly) / daly < 0.02
    # shorter MTBF moves the optimum to shorter intervals and lowers the achievable ETTR
    best2 = max(range(1, 2000), key=lambda i: orc.ettr(t_ckpt, t_iter, i, orc.recovery("dense", i, t_iter)[0], 600.0))
    assert best2 < best
    assert orc.ettr(t_ckpt, t_iter, best2, orc.recovery("dense", best2, t_iter)[0], 600.0) < \
        orc.ettr(t_ckpt, t_iter, best, orc.recovery("dense", best, t_iter)[0], mtbf)


def test_recovery_bounds(orc):
    """Sec. 3.6: dense 0 <= R <= I T, E[R] = I T / 2; sparse 0 <= R <= 2 W T, E[R] = 3/2 W T (so 4.5
    iterations are recomputed on average for W = 3)."""
    assert orc.recovery("dense", 10, 2.0) == (10.0, 20.0)
    assert orc.recovery("sparse", 3, 1.0) == (4.5, 6.0)
    assert math.ceil(orc.recovery("sparse", 3, 1.0)[0]) == 5
    for kind, sparse in (("dense", False), ("sparse", True)):
        for w, t in ((1, 0.5), (6, 3.0), (16, 1.25)):
            assert B.moev_recovery_time(sparse, w, t) == orc.recovery(kind, w, t)
    with pytest.raises(B.MoevError):
        B.moev_recovery_time(True, 0, 1.0)
