"""Pins for the oracle's counter-based generator and epsilon-greedy selection (Section 2.1)."""
import os

import numpy as np

from oracle import dqn as odqn
from oracle import philox

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def test_philox_known_answers():
    rows = [l.split() for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for row in rows:
        w = [int(x, 16) for x in row]
        assert philox.philox4x32_10(w[0:4], w[4:6]) == tuple(w[6:10])


def test_draw_counter_layout():
    seed, step, idx = 0x1234567890ABCDEF, (7 << 32) | 5, 11
    want = philox.philox4x32_10((idx, philox.TAG_ACT, 5, 7), (0x90ABCDEF, 0x12345678))
    assert philox.draw(seed, philox.TAG_ACT, step, idx) == want


def test_greedy_is_lowest_index_argmax_bruteforce():
    rng = np.random.default_rng(0)
    q = rng.integers(-3, 4, size=(500, 6)).astype(np.float64)   # many exact ties
    got = odqn.greedy_actions(q)
    for b in range(q.shape[0]):
        best = [k for k in range(6) if q[b, k] == q[b].max()]
        assert got[b] == best[0]


def test_epsilon_extremes_and_rate():
    rng = np.random.default_rng(1)
    q = rng.normal(size=(4000, 18))
    greedy = odqn.greedy_actions(q)
    a0 = odqn.epsilon_greedy(q, 0.0, seed=5, act_step=3)
    assert np.array_equal(a0, greedy)                       # epsilon = 0: always greedy
    a1 = odqn.epsilon_greedy(q, 1.0, seed=5, act_step=3)
    assert a1.min() >= 0 and a1.max() <= 17
    counts = np.bincount(a1, minlength=18)                   # epsilon = 1: uniform over A
    chi2 = ((counts - 4000 / 18) ** 2 / (4000 / 18)).sum()
    assert chi2 < 50.0                                        # 17 dof, p ~ 1e-5
    a = odqn.epsilon_greedy(q, 0.1, seed=5, act_step=3)
    # explored rows are exactly those whose uniform draw is below epsilon
    explored = np.array([np.float32(philox.draw(5, philox.TAG_ACT, 3, j)[0] >> 8) *
                         np.float32(2.0 ** -24) < np.float32(0.1) for j in range(4000)])
    assert abs(explored.mean() - 0.1) < 0.02
    assert np.array_equal(a[~explored], greedy[~explored])
    assert np.array_equal(a[explored], a1[explored])


def test_draws_depend_on_step_and_env():
    q = np.zeros((64, 4))
    a = odqn.epsilon_greedy(q, 1.0, seed=9, act_step=1)
    b = odqn.epsilon_greedy(q, 1.0, seed=9, act_step=2)
    c = odqn.epsilon_greedy(q, 1.0, seed=10, act_step=1)
    assert not np.array_equal(a, b) and not np.array_equal(a, c)
    assert np.array_equal(a, odqn.epsilon_greedy(q, 1.0, seed=9, act_step=1))
